/*
 * misa.h - C ABI of the MI355X (gfx950) MISA indexer library.
 *
 * The library computes the token-selection ("indexer") stage of sparse
 * attention as defined in "MISA: Mixture of Indexer Sparse Attention"
 * (Preliminaries, "Indexer in DSA"; Method, "MISA: mixture of indexer
 * experts" and "Hierarchical MISA").  Five calls, one per stage:
 *
 *   misa_pool_keys     Eq. pool                        block mean pooling
 *   misa_route_heads   Eq. misa_route_score/misa_route top-h head routing
 *   misa_score_tokens  Eq. misa_score (Eq. dsa_score)  routed token scoring
 *   misa_topk          Eq. misa_topk/misa_candidate    top-k token selection
 *   misa_rerank        Eq. misa_final_topk             dense re-rank (MISA-dagger)
 *
 * and, built from the same stages:
 *
 *   misa_select_tokens        scoring + top-k in one call, no score matrix
 *   misa_pool_keys_update     pooled keys maintained after tokens are appended
 *   misa_route_heads_proxy    the two content-free router scores of the
 *                             routing-score ablation
 *   misa_hisa_select,         the HISA and Block-Sparse comparison indexers
 *   misa_block_sparse_select
 *   misa_convert_queries      fp8 query codes -> bf16 (fp8 queries are accepted by every call)
 *   misa_probe_hbm_read,      achievable read and matrix rates of the machine,
 *   misa_probe_mfma_bf16      for roofline reports
 *
 * Conventions common to all calls
 * -------------------------------
 * - Every data pointer is DEVICE memory owned by the caller unless it is
 *   marked "host".  The library allocates nothing and frees nothing.  No
 *   result depends on an earlier call: the only things kept between calls
 *   are the thread-local error text, a per-device record of the dynamic-LDS
 *   limit already raised for a kernel (atomic; host threads may call
 *   concurrently) and the scratch array of misa_route_heads_static.  Scratch
 *   memory is passed in as (ws, ws_bytes); ask misa_workspace_bytes() for the
 *   size (it may be 0, then ws may be NULL).  ws must be 256-byte aligned.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   Calls only enqueue work on it; they never synchronise the host.
 * - Tensors are dense, row-major, innermost dimension contiguous:
 *     keys    K      [n_seq, L, d]       k_dtype
 *     kscale         [n_seq, L]          float, only for MISA_FP8_E4M3 keys:
 *                                        key value = kscale * decode(code);
 *                                        scales must be finite and >= 0
 *     queries Q      [n_seq, n_q, H, d]  q_dtype
 *     gates   W      [n_seq, n_q, H]     float (any sign)
 *   K, Q (and Kp where it is an input) must be 16-byte aligned.
 * - Causality: query t of sequence i sees the keys 0 .. n-1 with
 *     len_i = seq_len ? clamp(seq_len[i], 0, L) : L
 *     n     = q_pos  ? clamp(q_pos[t] + 1, 0, len_i) : len_i
 *   (q_pos[t] is the 0-based position of query t; its own token is visible).
 * - Ties (equal head importances, equal token scores) go to the lower
 *   index; -0.0 and +0.0 are equal.  Index lists are returned in ascending
 *   index order.  NaN inputs give unspecified selections.
 * - Errors: every call validates its host-side arguments first and launches
 *   nothing if validation fails.  The return value is a misa_status;
 *   misa_last_error() returns a thread-local description of the last failure
 *   on the calling thread.  Device data (q_pos, seq_len, heads, cand) cannot
 *   be validated on the host: out-of-range values are clamped or ignored as
 *   described per call, they never cause out-of-bounds accesses.
 * - Limits of this build: d == 128, 1 <= H <= 64, 1 <= h <= H,
 *   L <= 524288, k <= 16384; keys in F32, BF16 or FP8_E4M3 (with scales),
 *   queries in F32, BF16 or FP8_E4M3 (codes without scales, see "fp8 queries").
 */
#ifndef MISA_H
#define MISA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum misa_status {
  MISA_OK = 0,
  MISA_ERR_INVALID_ARG = 1, /* NULL required pointer, size out of range            */
  MISA_ERR_UNSUPPORTED = 2, /* legal request outside the limits of this build      */
  MISA_ERR_WORKSPACE = 3,   /* ws NULL/misaligned or ws_bytes too small            */
  MISA_ERR_HIP = 4          /* a HIP runtime call (launch) reported an error       */
} misa_status;

typedef enum misa_dtype {
  MISA_F32 = 0,
  MISA_BF16 = 1,
  MISA_FP8_E4M3 = 2, /* OCP FP8 E4M3 ("e4m3fn": bias 7, max 448, no infinity)           */
  MISA_FP8_E4M3_MATRIX = 3 /* q_dtype only: e4m3 query codes that may be contracted on the
                              fp8 matrix instruction (see "fp8 queries" below)             */
} misa_dtype;

typedef enum misa_op {
  MISA_OP_POOL = 0,
  MISA_OP_ROUTE = 1,
  MISA_OP_SCORE = 2,
  MISA_OP_TOPK = 3,
  MISA_OP_RERANK = 4,
  MISA_OP_SELECT = 5,
  MISA_OP_HISA = 6 /* misa_hisa_select and misa_block_sparse_select; k argument = m */
} misa_op;

/* Router scores of the routing-score ablation (appendix "Ablation: routing score"). */
typedef enum misa_router_score {
  MISA_ROUTER_BLOCK_POOLED = 0, /* the method's own score: misa_route_heads                 */
  MISA_ROUTER_GATE = 1,         /* variant (a): E_j = w_j, the gating weight as it is       */
  MISA_ROUTER_QUERY_NORM = 2    /* variant (b): E_j = ||q_j||_2                             */
} misa_router_score;

/* Problem description shared by all calls (host struct, passed by pointer). */
typedef struct misa_problem {
  int32_t n_seq;          /* sequences in the batch, >= 1                             */
  int32_t L;              /* keys stored per sequence (row count of K), >= 1          */
  int32_t d;              /* indexer head dimension; must be 128                      */
  int32_t n_q;            /* queries per sequence, >= 1                               */
  int32_t H;              /* indexer heads H^I, 1..64                                 */
  int32_t B;              /* router block size, >= 1 (any value, also >= L)           */
  int32_t h;              /* active heads, 1..H                                       */
  int32_t k_dtype;        /* misa_dtype of K                                          */
  int32_t q_dtype;        /* misa_dtype of Q (see "fp8 queries" below for FP8_E4M3)    */
  const int32_t* q_pos;   /* device [n_q], shared by all sequences; NULL = decode:
                             every query sits at the last position (n = len_i)       */
  const int32_t* seq_len; /* device [n_seq] or NULL (every sequence holds L keys)     */
  /* Paged key cache (optional; all three zero / NULL = contiguous K [n_seq, L, d]).
   * With a page table K is a pool of pages [n_pages, page_size, d] and kscale
   * [n_pages, page_size]; key s of sequence i is row
   *   page_table[i * max_pages + s / page_size] * page_size + s % page_size
   * of the pool.  Only entries for pages that hold keys 0 .. L-1 are read; they
   * must name pages inside the pool (not checked).  Every K / kscale argument of
   * every call is then the pool; S, Kp, indices and candidates stay logical.    */
  const int32_t* page_table; /* device [n_seq, max_pages] or NULL                      */
  int32_t page_size;         /* tokens per page: a power of two, 16 .. 65536           */
  int32_t max_pages;         /* row length of page_table, >= ceil(L / page_size)       */
} misa_problem;

/* Bytes of scratch the given op needs for this problem.  `k` is the k of
 * misa_topk, or k_cand of misa_rerank; ignored by the other ops.  Returns 0 on
 * invalid input as well (the op itself will then report the error). */
size_t misa_workspace_bytes(const misa_problem* p, int32_t op, int32_t k);

/* Text of the last error raised on this thread ("" if none).  Never NULL. */
const char* misa_last_error(void);

/* Library/ABI version: major * 1000 + minor. */
int32_t misa_version(void);

/*
 * Stage 1 - block mean pooling (Eq. pool; Method, "Block-pooled router").
 * The stored keys of each sequence are cut into M = ceil(L / B) contiguous
 * blocks; block b covers tokens b*B .. min((b+1)*B, len_i) - 1 and Kp[i, b, :]
 * is the arithmetic mean of its (de-quantised) keys, fp32.  A partial last
 * block is averaged over the tokens it holds; blocks entirely past len_i are
 * written as zeros.  Blocks longer than 2048 tokens are summed in slices that
 * pass through ws (MISA_OP_POOL reports its size, 0 for shorter blocks).
 *   K       in   [n_seq, L, d]
 *   kscale  in   [n_seq, L] (FP8 keys only, else NULL)
 *   Kp      out  [n_seq, M, d] float
 */
misa_status misa_pool_keys(const misa_problem* p, const void* K, const float* kscale,
                           float* Kp, void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 1 after tokens were appended to the cache (Eq. pool on the blocks that
 * changed): for every sequence i only the blocks from the one that holds token
 * from_token[i] up to the last block of its current length len_i are
 * recomputed, exactly as misa_pool_keys computes them; all other entries of
 * Kp are left as they are.  With from_token[i] = the previous length this is
 * the incremental maintenance of the pooled keys during decoding (normally one
 * block per sequence).
 *   from_token  in  [n_seq] int32 (device), clamped to 0..len_i
 *   max_blocks  host-side bound on the number of blocks per sequence to update
 *               (blocks beyond it are not recomputed), >= 1
 *   ws          as for misa_pool_keys (MISA_OP_POOL)
 */
misa_status misa_pool_keys_update(const misa_problem* p, const void* K, const float* kscale,
                                  float* Kp, const int32_t* from_token, int32_t max_blocks,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 2 - head routing (Eq. misa_route_score, Eq. misa_route).
 * For every query:  A[j,b] = W[j] * ReLU(Q[j] . k~_b),
 *                   E[j]   = (1/M_n) * sum_b |A[j,b]|,   M_n = ceil(n / B),
 * and the h heads with the largest E are kept.  The blocks are those of the
 * query's own visible prefix 0..n-1: complete blocks come from Kp; if
 * n is not a multiple of B, the last block is the mean of keys
 * floor(n/B)*B .. n-1 (read from K when n < len_i, so no pooled key ever
 * contains a token the query cannot see).  n == 0 gives E = 0.
 *   Q, W    in
 *   Kp      in   [n_seq, M, d] float, as written by misa_pool_keys for the
 *                same problem
 *   K,kscale in  raw keys (used only for partial last blocks of causal queries)
 *   heads   out  [n_seq, n_q, h] int32, ascending
 *   E       out  [n_seq, n_q, H] float, may be NULL
 */
misa_status misa_route_heads(const misa_problem* p, const void* Q, const float* W,
                             const float* Kp, const void* K, const float* kscale,
                             int32_t* heads, float* E, void* ws, size_t ws_bytes, void* stream);

/*
 * misa_route_heads for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and error behaviour as
 * misa_route_heads, but the partial sums of the block tiles (and the widened
 * copy of fp8 queries) live in an array of MISA_ROUTE_STATIC_SCRATCH_BYTES bytes
 * that is part of the library's device code; every GPU the library runs on
 * holds one copy of it until the process ends.  The call allocates and frees
 * nothing.  Problems whose misa_workspace_bytes(p, MISA_OP_ROUTE, 0) exceeds
 * MISA_ROUTE_STATIC_SCRATCH_BYTES are rejected with MISA_ERR_UNSUPPORTED before
 * anything is launched (4 MiB covers decode batches of up to 256 sequences and
 * prefill chunks of up to 4096 bf16 queries).  All calls on one GPU share that
 * GPU's array: calls that may overlap in time on one GPU (different streams or
 * host threads) race on it and must be serialised by the caller; nothing in
 * the array has to be cleared between calls (every word read is written first
 * by the same call).
 */
#define MISA_ROUTE_STATIC_SCRATCH_BYTES (4u << 20)
misa_status misa_route_heads_static(const misa_problem* p, const void* Q, const float* W,
                                    const float* Kp, const void* K, const float* kscale,
                                    int32_t* heads, float* E, void* stream);

/*
 * Head routing with one of the two content-free scores that the appendix
 * "Ablation: routing score" compares the method with: kind MISA_ROUTER_GATE
 * ranks the heads by their gate W[j] (signed, as printed there), kind
 * MISA_ROUTER_QUERY_NORM by the Euclidean norm of Q[j].  Same selection rule
 * and outputs as misa_route_heads (top-h, ties to the lower index, ascending);
 * the keys are not consulted, no workspace is needed.
 *   heads  out  [n_seq, n_q, h] int32
 *   E      out  [n_seq, n_q, H] float or NULL
 */
misa_status misa_route_heads_proxy(const misa_problem* p, const void* Q, const float* W,
                                   int32_t kind, int32_t* heads, float* E, void* stream);

/*
 * Stage 3 - token scoring with the active heads (Eq. misa_score).
 *   S[i,t,s] = sum_{j in heads[i,t,:]} W[j] * ReLU(Q[j] . k_s)   for s < n,
 *   S[i,t,s] = -inf                                              for n <= s < L.
 * heads == NULL scores with all H heads (h is ignored): the dense DSA indexer
 * of Eq. dsa_score.  Head indices outside 0..H-1 contribute nothing; a head
 * listed twice is counted twice.  Products of the stored bf16/fp8 values are
 * exact; accumulation is fp32.
 *   heads   in   [n_seq, n_q, h] int32 or NULL
 *   S       out  [n_seq, n_q, L] float
 */
misa_status misa_score_tokens(const misa_problem* p, const void* Q, const float* W,
                              const int32_t* heads, const void* K, const float* kscale,
                              float* S, void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 4 - top-k selection (Eq. misa_topk; with k = k' Eq. misa_candidate).
 * Selects the min(k, n) largest entries of S[i,t,0..n-1]; exact, ties to the
 * lower index.
 *   S    in   [n_seq, n_q, L] float
 *   idx  out  [n_seq, n_q, k] int32 ascending; unused tail slots = -1
 *   val  out  [n_seq, n_q, k] float or NULL: val[j] = S[idx[j]], tail = -inf
 */
misa_status misa_topk(const misa_problem* p, const float* S, int32_t k, int32_t* idx,
                      float* val, void* ws, size_t ws_bytes, void* stream);

/*
 * Stages 3 + 4 in one call (Eq. misa_score then Eq. misa_topk / Eq.
 * misa_candidate; heads == NULL: Eq. dsa_score then Eq. dsa_topk).  Writes
 * exactly what misa_score_tokens followed by misa_topk would write to idx and
 * val, but for many-query problems (bf16 queries, bf16 or FP8 keys, n_q >= 8,
 * k <= 8192, L >= 4096, p->h >= 3) the [n_seq, n_q, L] score matrix is not produced:
 * a 1/16 sample of the keys gives a per-row threshold, a second scoring pass
 * keeps only the scores that reach it, and the exact top-k is taken from
 * those.  Rows for which the threshold turns out too high or too low are
 * recomputed by the two-call path inside the same call, so the result never
 * depends on the sample.  Other problems run the two calls back to back.
 * ws (MISA_OP_SELECT) includes room for the score matrix in both cases.
 *   heads  in   [n_seq, n_q, h] int32 or NULL
 *   idx    out  [n_seq, n_q, k] int32 ascending; unused tail slots = -1
 *   val    out  [n_seq, n_q, k] float or NULL, tail = -inf
 */
misa_status misa_select_tokens(const misa_problem* p, const void* Q, const float* W,
                               const int32_t* heads, const void* K, const float* kscale,
                               int32_t k, int32_t* idx, float* val, void* ws, size_t ws_bytes,
                               void* stream);

/*
 * Monitoring aid for misa_select_tokens: byte offset inside its workspace of
 * an int32 array [n_seq, n_q] that the last call left there, 1 for every row
 * that was recomputed by the two-call path and 0 otherwise; -1 if the problem
 * does not take the sampled route at all.  routed: whether heads was non-NULL.
 */
int64_t misa_select_row_flags_offset(const misa_problem* p, int32_t routed, int32_t k);

/*
 * Stage 5 - MISA-dagger fine stage (Eq. misa_final_topk): re-score the
 * candidates with ALL H heads (Eq. dsa_score) and keep the best k.
 *   cand  in   [n_seq, n_q, k_cand] int32: distinct token indices in ascending
 *              order as misa_topk writes them; entries < 0 or >= n are skipped
 *   idx   out  [n_seq, n_q, k] int32 ascending, tail = -1
 *   val   out  [n_seq, n_q, k] float or NULL (dense scores), tail = -inf
 * Ties go to the earlier candidate slot (= lower token index for ascending
 * cand).  Requires 1 <= k <= k_cand <= 16384.
 */
misa_status misa_rerank(const misa_problem* p, const void* Q, const float* W, const void* K,
                        const float* kscale, const int32_t* cand, int32_t k_cand, int32_t k,
                        int32_t* idx, float* val, void* ws, size_t ws_bytes, void* stream);

/*
 * Comparison indexers on the same stages (not part of MISA itself).
 *
 * HISA (preliminaries, "Indexer in HISA": Eq. block_score, Eq. final_topk): the
 * pooled keys of the query's prefix are scored with ALL H heads,
 *   J[b] = sum_j W[j] * ReLU(Q[j] . k~_b);
 * the first and the last block of the prefix are always kept and the
 * best-scoring other blocks are added up to m blocks in all (every block if
 * the prefix has at most m; ties to the lower index); the tokens of those
 * blocks are then scored with all heads (Eq. dsa_score) and the best k kept,
 * as misa_rerank does for its candidates.  Kp is what misa_pool_keys wrote.
 *   m       blocks kept per query, >= 2, m * B <= 16384
 *   k       1 <= k <= m * B
 *   blocks  out  [n_seq, n_q, m] int32 ascending, tail = -1, or NULL
 *   idx     out  [n_seq, n_q, k] int32 ascending, tail = -1
 *   val     out  [n_seq, n_q, k] float or NULL (dense scores), tail = -inf
 */
misa_status misa_hisa_select(const misa_problem* p, const void* Q, const float* W, const float* Kp,
                             const void* K, const float* kscale, int32_t m, int32_t k,
                             int32_t* blocks, int32_t* idx, float* val, void* ws, size_t ws_bytes,
                             void* stream);

/*
 * Block-Sparse (Experimental results, "Baselines"; MoBA-style): the same block
 * choice as the first stage of misa_hisa_select; the visible tokens of the
 * chosen blocks are the selection (m = k / B gives a budget of k tokens).
 *   idx  out  [n_seq, n_q, m * B] int32: token o of the i-th chosen block at
 *             slot i * B + o, -1 where there is no such block or the token is
 *             not visible (ascending apart from the -1 entries)
 */
misa_status misa_block_sparse_select(const misa_problem* p, const void* Q, const float* W,
                                     const float* Kp, int32_t m, int32_t* blocks, int32_t* idx,
                                     void* ws, size_t ws_bytes, void* stream);

/*
 * fp8 queries (q_dtype = MISA_FP8_E4M3; the paper notes that DSA quantises its indexer to
 * FP8): Q is [n_seq, n_q, H, d] uint8 e4m3 codes WITHOUT a scale array.  A positive
 * per-(query, head) scale c belongs into the gate: w ReLU((c q) . k) = (c w) ReLU(q . k), so
 * the caller passes W[i,t,j] * c[i,t,j].  Every e4m3 value is also a bf16 value: each call that
 * takes Q widens the codes to bf16 at the head of its workspace (misa_workspace_bytes
 * includes that room; misa_route_heads_proxy reads the codes directly) and proceeds exactly
 * as for bf16 queries, so results equal those of the widened queries bit for bit.  A caller
 * that runs several stages on the same queries widens them once with misa_convert_queries
 * and passes the result with q_dtype = MISA_BF16.
 *
 * q_dtype = MISA_FP8_E4M3_MATRIX is the same input format, with one permission: when the keys
 * are MISA_FP8_E4M3 too and the problem has at least 8 queries per sequence (the prefill tile
 * kernel), misa_score_tokens and misa_select_tokens - and misa_rerank for any number of
 * queries - leave queries and keys as codes and
 * contract them with the fp8 matrix instruction (v_mfma_f32_32x32x64_f8f6f4): half the matrix
 * time, no widening, half the staged bytes.  The products are still exact, but that
 * instruction sums its 64 products in a narrower format than fp32: measured on MI355X, a dot
 * product of 128 terms comes out within 2^-15 of the sum of the absolute products (fp32
 * accumulation of the widened values: 2^-22).  Scores therefore carry an absolute error of up
 * to about 4e-5 of the largest score magnitudes of their row instead of 1e-5, and selections
 * may differ from the exact ones among scores that close.  All other calls (routing,
 * decode-shaped scoring, other key types, the comparison indexers) treat it exactly as
 * MISA_FP8_E4M3.
 *   Q       in   [n_seq, n_q, H, d] uint8, 16-byte aligned (p->q_dtype must be an fp8 type)
 *   Q_bf16  out  [n_seq, n_q, H, d] bf16, 16-byte aligned
 */
misa_status misa_convert_queries(const misa_problem* p, const void* Q, void* Q_bf16, void* stream);

/*
 * Measurement probes (not part of the method; for callers that report rates against
 * what the machine delivers as well as against its published peaks).
 *
 * misa_probe_hbm_read: one kernel that reads `bytes` bytes of `buf` once (short-lived
 * wavefronts, every load issued up front: the fastest read pattern found on this chip)
 * and writes nothing.  bytes / its duration is the achievable read rate.
 *   buf    in   device, 16-byte aligned, bytes a positive multiple of 8192
 *   sink   out  device, at least 1024 bytes (written only on a one-in-2^32 data match)
 *
 * misa_probe_mfma_bf16: `workgroups` workgroups of four wavefronts, each wavefront issuing
 * iters x 4 independent v_mfma_f32_32x32x16_bf16 on register operands.  *flops / its
 * duration is the achievable dense bf16 matrix rate at the clock the chip sustains.
 *   sink   out  device, workgroups * 256 floats
 *   flops  out  HOST pointer or NULL: floating-point operations of the launch
 * The operands are constants (1.0 x {0.5, 1.0}).
 *
 * misa_probe_mfma_bf16_operands: the same loop on operands the caller supplies.  The matrix rate
 * MI355X sustains depends on the operand VALUES (the clock it holds drops as more bits toggle
 * per product), so the rate reachable on data like a workload's is measured with such data.
 *   operands  in  device, 16-byte aligned, 2048 bytes: 64 x 16 bytes (eight bf16) = fragment a
 *                 of lanes 0..63, then 64 x 16 bytes = fragment b; every wavefront uses the same
 * All three enqueue on `stream` and return; time them with events.
 */
misa_status misa_probe_hbm_read(const void* buf, size_t bytes, void* sink, void* stream);
misa_status misa_probe_mfma_bf16(int32_t workgroups, int32_t iters, float* sink, double* flops,
                                 void* stream);
misa_status misa_probe_mfma_bf16_operands(int32_t workgroups, int32_t iters, const void* operands,
                                          float* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MISA_H */
