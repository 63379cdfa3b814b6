// C ABI of the MISA indexer library: argument validation, workspace sizing,
// error reporting and dispatch to the kernel launchers.  See include/misa.h
// for the contract of every entry point.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "kernels.h"

// Scratch of misa_route_heads_static: the router's partial sums (and, for fp8 queries, their
// widened copy) live here instead of in a caller workspace.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[MISA_ROUTE_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

misa_status fail(misa_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Validates the problem description and converts it for the kernels.
misa_status check_problem(const misa_problem* p, misa::Prob* out) {
  if (!p) return fail(MISA_ERR_INVALID_ARG, "problem is NULL");
  if (p->n_seq < 1 || p->L < 1 || p->n_q < 1 || p->H < 1 || p->B < 1)
    return fail(MISA_ERR_INVALID_ARG, "n_seq, L, n_q, H and B must all be >= 1 (got %d %d %d %d %d)",
                p->n_seq, p->L, p->n_q, p->H, p->B);
  if (p->h < 1 || p->h > p->H)
    return fail(MISA_ERR_INVALID_ARG, "h must be in 1..H (h=%d, H=%d)", p->h, p->H);
  if (p->k_dtype < MISA_F32 || p->k_dtype > MISA_FP8_E4M3)
    return fail(MISA_ERR_INVALID_ARG, "unknown k_dtype %d", p->k_dtype);
  if (p->q_dtype < MISA_F32 || p->q_dtype > MISA_FP8_E4M3_MATRIX)
    return fail(MISA_ERR_INVALID_ARG, "unknown q_dtype %d", p->q_dtype);
  if (p->n_q > 1 && !p->q_pos)
    return fail(MISA_ERR_INVALID_ARG, "q_pos is required when n_q > 1");
  if (p->d != misa::kD) return fail(MISA_ERR_UNSUPPORTED, "d must be 128 (got %d)", p->d);
  if (p->H > misa::kMaxH) return fail(MISA_ERR_UNSUPPORTED, "H must be <= 64 (got %d)", p->H);
  if (p->L > misa::kMaxRowLen) return fail(MISA_ERR_UNSUPPORTED, "L must be <= 524288 (got %d)", p->L);
  if (p->n_seq > 65535 || p->n_q > 65535)
    return fail(MISA_ERR_UNSUPPORTED, "n_seq and n_q must be <= 65535");
  out->n_seq = p->n_seq; out->L = p->L; out->n_q = p->n_q; out->H = p->H; out->B = p->B;
  out->h = p->h;
  out->M = (int)(((long long)p->L + p->B - 1) / p->B);
  out->q_pos = p->q_pos; out->seq_len = p->seq_len;
  out->page_table = nullptr; out->page_shift = 0; out->max_pages = 0;
  if (p->page_table) {
    const int ps = p->page_size;
    if (ps < 16 || ps > 65536 || (ps & (ps - 1)) != 0)
      return fail(MISA_ERR_INVALID_ARG, "page_size must be a power of two in 16..65536 (got %d)", ps);
    if ((long long)p->max_pages * ps < p->L)
      return fail(MISA_ERR_INVALID_ARG, "max_pages * page_size must cover L (max_pages=%d, page_size=%d, L=%d)",
                  p->max_pages, ps, p->L);
    out->page_table = p->page_table;
    out->max_pages = p->max_pages;
    while ((1 << out->page_shift) < ps) ++out->page_shift;
  } else if (p->page_size != 0 || p->max_pages != 0) {
    return fail(MISA_ERR_INVALID_ARG, "page_size / max_pages given without a page_table");
  }
  return MISA_OK;
}

misa_status check_keys(const misa_problem* p, const void* K, const float* kscale) {
  if (!K) return fail(MISA_ERR_INVALID_ARG, "K is NULL");
  if (!aligned(K, 16)) return fail(MISA_ERR_INVALID_ARG, "K must be 16-byte aligned");
  if (p->k_dtype == MISA_FP8_E4M3 && !kscale)
    return fail(MISA_ERR_INVALID_ARG, "kscale is required for fp8 keys");
  return MISA_OK;
}

misa_status check_queries(const void* Q, const float* W) {
  if (!Q || !W) return fail(MISA_ERR_INVALID_ARG, "Q or W is NULL");
  if (!aligned(Q, 16)) return fail(MISA_ERR_INVALID_ARG, "Q must be 16-byte aligned");
  return MISA_OK;
}

misa_status check_ws(size_t need, const void* ws, size_t ws_bytes) {
  if (need == 0) return MISA_OK;
  if (!ws) return fail(MISA_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
  if (!aligned(ws, 256)) return fail(MISA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (ws_bytes < need)
    return fail(MISA_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
  return MISA_OK;
}

misa_status hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) { g_err[0] = 0; return MISA_OK; }
  return fail(MISA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// fp8 query codes are widened to bf16 (exact) at the head of the workspace; the kernels then
// see bf16 queries and the rest of the workspace.
struct QView { const void* Q; int q_dtype; void* ws; size_t ws_bytes; };

bool fp8_queries(const misa_problem* p) {
  return p->q_dtype == MISA_FP8_E4M3 || p->q_dtype == MISA_FP8_E4M3_MATRIX;
}

// Scoring calls keep fp8 query codes as they are (fp8 matrix instruction) when the caller allowed
// it, the keys are fp8 as well and the problem runs on the prefill tile kernel.
bool native_fp8(const misa_problem* p, const misa::Prob& pr) {
  return p->q_dtype == MISA_FP8_E4M3_MATRIX && p->k_dtype == MISA_FP8_E4M3 &&
         misa::tile_path(pr, MISA_FP8_E4M3, MISA_FP8_E4M3);
}

size_t q_stage_bytes(const misa_problem* p) {
  if (!fp8_queries(p)) return 0;
  const size_t b = (size_t)p->n_seq * p->n_q * p->H * misa::kD * 2;
  return (b + 255) & ~(size_t)255;
}

int eff_q_dtype(const misa_problem* p) { return fp8_queries(p) ? MISA_BF16 : p->q_dtype; }

misa_status stage_queries(const misa_problem* p, const void* Q, size_t need_rest, void* ws,
                          size_t ws_bytes, void* stream, QView* v, bool keep_fp8 = false) {
  if (keep_fp8) {   // the codes go to the kernels as they are; the whole workspace is theirs
    misa_status st = check_ws(need_rest, ws, ws_bytes);
    if (st != MISA_OK) return st;
    v->Q = Q; v->q_dtype = MISA_FP8_E4M3; v->ws = ws; v->ws_bytes = ws_bytes;
    return MISA_OK;
  }
  const size_t qb = q_stage_bytes(p);
  misa_status st = check_ws(need_rest + qb, ws, ws_bytes);
  if (st != MISA_OK) return st;
  v->Q = Q; v->q_dtype = p->q_dtype; v->ws = ws; v->ws_bytes = ws_bytes;
  if (qb) {
    hipError_t e = misa::launch_widen_queries(Q, ws, (size_t)p->n_seq * p->n_q * p->H * misa::kD,
                                              (hipStream_t)stream);
    if (e != hipSuccess) return hip_result(e, "query widening launch");
    v->Q = ws; v->q_dtype = MISA_BF16;
    v->ws = static_cast<char*>(ws) + qb; v->ws_bytes = ws_bytes - qb;
  }
  return MISA_OK;
}

size_t ws_bytes_for(const misa::Prob& pr, int op, int k, int k_dtype = 0, int q_dtype = 0) {
  switch (op) {
    case MISA_OP_SELECT: return misa::select_ws_bytes(pr, k_dtype, q_dtype, k);
    case MISA_OP_HISA: return misa::hisa_ws_bytes(pr, k);
    case MISA_OP_POOL: return misa::pool_ws_bytes(pr);
    case MISA_OP_ROUTE: return misa::route_ws_bytes(pr);
    case MISA_OP_TOPK: return misa::topk_ws_bytes(pr, k);
    case MISA_OP_RERANK:
      return k >= 1 ? (size_t)pr.n_seq * pr.n_q * (size_t)k * sizeof(float) : 0;
    default: return 0;
  }
}

}  // namespace

extern "C" {

int32_t misa_version(void) { return 1000; }

const char* misa_last_error(void) { return g_err; }

size_t misa_workspace_bytes(const misa_problem* p, int32_t op, int32_t k) {
  misa::Prob pr;
  if (check_problem(p, &pr) != MISA_OK) return 0;
  if (op < MISA_OP_POOL || op > MISA_OP_HISA) return 0;
  const bool takes_queries = op == MISA_OP_ROUTE || op == MISA_OP_SCORE || op == MISA_OP_RERANK ||
                             op == MISA_OP_SELECT || op == MISA_OP_HISA;
  return ws_bytes_for(pr, op, k, p->k_dtype, eff_q_dtype(p)) + (takes_queries ? q_stage_bytes(p) : 0);
}

misa_status misa_pool_keys(const misa_problem* p, const void* K, const float* kscale, float* Kp,
                           void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!Kp) return fail(MISA_ERR_INVALID_ARG, "Kp is NULL");
  if ((st = check_ws(ws_bytes_for(pr, MISA_OP_POOL, 0), ws, ws_bytes)) != MISA_OK) return st;
  return hip_result(misa::launch_pool(pr, p->k_dtype, K, kscale, Kp, ws, (hipStream_t)stream),
                    "misa_pool_keys launch");
}

misa_status misa_pool_keys_update(const misa_problem* p, const void* K, const float* kscale, float* Kp,
                                  const int32_t* from_token, int32_t max_blocks, void* ws,
                                  size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!Kp || !from_token) return fail(MISA_ERR_INVALID_ARG, "Kp or from_token is NULL");
  if (max_blocks < 1) return fail(MISA_ERR_INVALID_ARG, "max_blocks must be >= 1 (got %d)", max_blocks);
  if ((st = check_ws(ws_bytes_for(pr, MISA_OP_POOL, 0), ws, ws_bytes)) != MISA_OK) return st;
  return hip_result(misa::launch_pool(pr, p->k_dtype, K, kscale, Kp, ws, (hipStream_t)stream, from_token,
                                      max_blocks),
                    "misa_pool_keys_update launch");
}

misa_status misa_route_heads(const misa_problem* p, const void* Q, const float* W, const float* Kp,
                             const void* K, const float* kscale, int32_t* heads, float* E, void* ws,
                             size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!Kp || !heads) return fail(MISA_ERR_INVALID_ARG, "Kp or heads is NULL");
  QView qv;
  if ((st = stage_queries(p, Q, ws_bytes_for(pr, MISA_OP_ROUTE, 0), ws, ws_bytes, stream, &qv)) != MISA_OK) return st;
  return hip_result(misa::launch_route(pr, p->k_dtype, qv.q_dtype, qv.Q, W, Kp, K, kscale, heads, E, qv.ws,
                                       (hipStream_t)stream),
                    "misa_route_heads launch");
}

misa_status misa_route_heads_static(const misa_problem* p, const void* Q, const float* W, const float* Kp,
                                    const void* K, const float* kscale, int32_t* heads, float* E,
                                    void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!Kp || !heads) return fail(MISA_ERR_INVALID_ARG, "Kp or heads is NULL");
  const size_t need = ws_bytes_for(pr, MISA_OP_ROUTE, 0) + q_stage_bytes(p);
  if (need > (size_t)MISA_ROUTE_STATIC_SCRATCH_BYTES)
    return fail(MISA_ERR_UNSUPPORTED,
                "misa_route_heads_static: the problem needs %zu bytes of scratch, the built-in array holds %zu; "
                "use misa_route_heads with a workspace",
                need, (size_t)MISA_ROUTE_STATIC_SCRATCH_BYTES);
  // Address of this device's copy of the array, looked up once per device with that device
  // current.  The array's name is only a host-side handle: kernels get the looked-up address.
  static std::atomic<void*> scratch_of_device[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_result(e, "hipGetDevice");
  void* ptr = (dev >= 0 && dev < 64) ? scratch_of_device[dev].load(std::memory_order_acquire) : nullptr;
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return hip_result(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
    if (dev >= 0 && dev < 64) scratch_of_device[dev].store(ptr, std::memory_order_release);
  }
  QView qv;
  if ((st = stage_queries(p, Q, need - q_stage_bytes(p), ptr, (size_t)MISA_ROUTE_STATIC_SCRATCH_BYTES, stream,
                          &qv)) != MISA_OK)
    return st;
  return hip_result(misa::launch_route(pr, p->k_dtype, qv.q_dtype, qv.Q, W, Kp, K, kscale, heads, E, qv.ws,
                                       (hipStream_t)stream),
                    "misa_route_heads_static launch");
}

misa_status misa_route_heads_proxy(const misa_problem* p, const void* Q, const float* W, int32_t kind,
                                   int32_t* heads, float* E, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if (!heads) return fail(MISA_ERR_INVALID_ARG, "heads is NULL");
  if (kind != MISA_ROUTER_GATE && kind != MISA_ROUTER_QUERY_NORM)
    return fail(MISA_ERR_INVALID_ARG, "kind must be MISA_ROUTER_GATE or MISA_ROUTER_QUERY_NORM (got %d)", kind);
  const int qd = fp8_queries(p) ? (int)MISA_FP8_E4M3 : p->q_dtype;
  return hip_result(misa::launch_route_proxy(pr, qd, kind, Q, W, heads, E, (hipStream_t)stream),
                    "misa_route_heads_proxy launch");
}

misa_status misa_score_tokens(const misa_problem* p, const void* Q, const float* W,
                              const int32_t* heads, const void* K, const float* kscale, float* S,
                              void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!S) return fail(MISA_ERR_INVALID_ARG, "S is NULL");
  QView qv;
  if ((st = stage_queries(p, Q, 0, ws, ws_bytes, stream, &qv, native_fp8(p, pr))) != MISA_OK) return st;
  return hip_result(misa::launch_score(pr, p->k_dtype, qv.q_dtype, qv.Q, W, heads, K, kscale, nullptr, 0,
                                       S, (hipStream_t)stream),
                    "misa_score_tokens launch");
}

misa_status misa_topk(const misa_problem* p, const float* S, int32_t k, int32_t* idx, float* val,
                      void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if (!S || !idx) return fail(MISA_ERR_INVALID_ARG, "S or idx is NULL");
  if (k < 1) return fail(MISA_ERR_INVALID_ARG, "k must be >= 1 (got %d)", k);
  if (k > misa::kMaxTopK) return fail(MISA_ERR_UNSUPPORTED, "k must be <= 16384 (got %d)", k);
  if ((st = check_ws(ws_bytes_for(pr, MISA_OP_TOPK, k), ws, ws_bytes)) != MISA_OK) return st;
  return hip_result(misa::launch_topk(pr, S, pr.L, k, nullptr, idx, val, ws, (hipStream_t)stream),
                    "misa_topk launch");
}

misa_status misa_select_tokens(const misa_problem* p, const void* Q, const float* W,
                               const int32_t* heads, const void* K, const float* kscale, int32_t k,
                               int32_t* idx, float* val, void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!idx) return fail(MISA_ERR_INVALID_ARG, "idx is NULL");
  if (k < 1) return fail(MISA_ERR_INVALID_ARG, "k must be >= 1 (got %d)", k);
  if (k > misa::kMaxTopK) return fail(MISA_ERR_UNSUPPORTED, "k must be <= 16384 (got %d)", k);
  QView qv;
  const bool native = native_fp8(p, pr);
  if ((st = stage_queries(p, Q, ws_bytes_for(pr, MISA_OP_SELECT, k, p->k_dtype, native ? (int)MISA_FP8_E4M3 : eff_q_dtype(p)),
                          ws, ws_bytes, stream, &qv, native)) != MISA_OK)
    return st;
  return hip_result(misa::launch_select(pr, p->k_dtype, qv.q_dtype, qv.Q, W, heads, K, kscale, k, idx, val,
                                        qv.ws, (hipStream_t)stream),
                    "misa_select_tokens launch");
}

int64_t misa_select_row_flags_offset(const misa_problem* p, int32_t routed, int32_t k) {
  misa::Prob pr;
  if (check_problem(p, &pr) != MISA_OK) return -1;
  const bool native = native_fp8(p, pr);
  const long long off = misa::select_row_flags_offset(pr, p->k_dtype, native ? (int)MISA_FP8_E4M3 : eff_q_dtype(p), routed != 0, k);
  return off < 0 || native ? off : off + (long long)q_stage_bytes(p);
}

namespace {
misa_status check_block_budget(const misa::Prob& pr, int32_t m) {
  if (m < 2) return fail(MISA_ERR_INVALID_ARG, "m must be >= 2: the first and the last block are always kept (got %d)", m);
  if ((long long)m * pr.B > misa::kMaxTopK)
    return fail(MISA_ERR_UNSUPPORTED, "m * B must be <= 16384 (m=%d, B=%d)", m, pr.B);
  return MISA_OK;
}
}  // namespace

misa_status misa_hisa_select(const misa_problem* p, const void* Q, const float* W, const float* Kp,
                             const void* K, const float* kscale, int32_t m, int32_t k, int32_t* blocks,
                             int32_t* idx, float* val, void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!Kp || !idx) return fail(MISA_ERR_INVALID_ARG, "Kp or idx is NULL");
  if ((st = check_block_budget(pr, m)) != MISA_OK) return st;
  if (k < 1 || (long long)k > (long long)m * pr.B)
    return fail(MISA_ERR_INVALID_ARG, "need 1 <= k <= m * B (k=%d, m=%d, B=%d)", k, m, pr.B);
  QView qv;
  if ((st = stage_queries(p, Q, ws_bytes_for(pr, MISA_OP_HISA, m), ws, ws_bytes, stream, &qv)) != MISA_OK) return st;
  return hip_result(misa::launch_hisa(pr, p->k_dtype, qv.q_dtype, qv.Q, W, Kp, K, kscale, m, k, blocks, idx,
                                      val, qv.ws, (hipStream_t)stream),
                    "misa_hisa_select launch");
}

misa_status misa_block_sparse_select(const misa_problem* p, const void* Q, const float* W,
                                     const float* Kp, int32_t m, int32_t* blocks, int32_t* idx, void* ws,
                                     size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if (!Kp || !idx) return fail(MISA_ERR_INVALID_ARG, "Kp or idx is NULL");
  if ((st = check_block_budget(pr, m)) != MISA_OK) return st;
  QView qv;
  if ((st = stage_queries(p, Q, ws_bytes_for(pr, MISA_OP_HISA, m), ws, ws_bytes, stream, &qv)) != MISA_OK) return st;
  return hip_result(misa::launch_hisa(pr, p->k_dtype, qv.q_dtype, qv.Q, W, Kp, nullptr, nullptr, m, 0, blocks,
                                      idx, nullptr, qv.ws, (hipStream_t)stream),
                    "misa_block_sparse_select launch");
}

misa_status misa_rerank(const misa_problem* p, const void* Q, const float* W, const void* K,
                        const float* kscale, const int32_t* cand, int32_t k_cand, int32_t k,
                        int32_t* idx, float* val, void* ws, size_t ws_bytes, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if ((st = check_queries(Q, W)) != MISA_OK) return st;
  if ((st = check_keys(p, K, kscale)) != MISA_OK) return st;
  if (!cand || !idx) return fail(MISA_ERR_INVALID_ARG, "cand or idx is NULL");
  if (k < 1 || k_cand < k)
    return fail(MISA_ERR_INVALID_ARG, "need 1 <= k <= k_cand (k=%d, k_cand=%d)", k, k_cand);
  if (k_cand > misa::kMaxTopK)
    return fail(MISA_ERR_UNSUPPORTED, "k_cand must be <= 16384 (got %d)", k_cand);
  QView qv;
  // the candidate gather takes fp8 codes with fp8 keys for any number of queries
  const bool native = p->q_dtype == MISA_FP8_E4M3_MATRIX && p->k_dtype == MISA_FP8_E4M3;
  if ((st = stage_queries(p, Q, ws_bytes_for(pr, MISA_OP_RERANK, k_cand), ws, ws_bytes, stream, &qv, native)) != MISA_OK) return st;
  if (misa::rerank_fused_path(pr, p->k_dtype, qv.q_dtype, k_cand))
    return hip_result(misa::launch_rerank_fused(pr, p->k_dtype, qv.q_dtype, qv.Q, W, K, kscale, cand, k_cand, k,
                                                idx, val, (hipStream_t)stream),
                      "misa_rerank launch");
  float* dense = static_cast<float*>(qv.ws);
  hipError_t e = misa::launch_score(pr, p->k_dtype, qv.q_dtype, qv.Q, W, nullptr, K, kscale, cand, k_cand,
                                    dense, (hipStream_t)stream);
  if (e != hipSuccess) return hip_result(e, "misa_rerank score launch");
  return hip_result(misa::launch_topk(pr, dense, k_cand, k, cand, idx, val, nullptr, (hipStream_t)stream),
                    "misa_rerank top-k launch");
}

misa_status misa_convert_queries(const misa_problem* p, const void* Q, void* Q_bf16, void* stream) {
  misa::Prob pr;
  misa_status st = check_problem(p, &pr);
  if (st != MISA_OK) return st;
  if (!fp8_queries(p)) return fail(MISA_ERR_INVALID_ARG, "q_dtype must be MISA_FP8_E4M3 or MISA_FP8_E4M3_MATRIX");
  if (!Q || !Q_bf16) return fail(MISA_ERR_INVALID_ARG, "Q or Q_bf16 is NULL");
  if (!aligned(Q, 16) || !aligned(Q_bf16, 16))
    return fail(MISA_ERR_INVALID_ARG, "Q and Q_bf16 must be 16-byte aligned");
  return hip_result(misa::launch_widen_queries(Q, Q_bf16, (size_t)p->n_seq * p->n_q * p->H * misa::kD,
                                               (hipStream_t)stream),
                    "misa_convert_queries launch");
}

misa_status misa_probe_hbm_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink) return fail(MISA_ERR_INVALID_ARG, "buf or sink is NULL");
  if (!aligned(buf, 16)) return fail(MISA_ERR_INVALID_ARG, "buf must be 16-byte aligned");
  if (bytes < 8192 || bytes % 8192 != 0 || bytes > ((size_t)1 << 40))
    return fail(MISA_ERR_INVALID_ARG, "bytes must be a positive multiple of 8192 (got %zu)", bytes);
  return hip_result(misa::launch_probe_read(buf, bytes, sink, (hipStream_t)stream),
                    "misa_probe_hbm_read launch");
}

misa_status misa_probe_mfma_bf16(int32_t workgroups, int32_t iters, float* sink, double* flops,
                                 void* stream) {
  if (!sink) return fail(MISA_ERR_INVALID_ARG, "sink is NULL");
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
    return fail(MISA_ERR_INVALID_ARG, "need 1 <= workgroups <= 2^20 and 1 <= iters <= 2^24");
  if (flops) *flops = (double)workgroups * 4.0 * (double)iters * misa::kProbeMfmaFlopsPerWaveIter;
  return hip_result(misa::launch_probe_mfma(workgroups, iters, nullptr, sink, (hipStream_t)stream),
                    "misa_probe_mfma_bf16 launch");
}

misa_status misa_probe_mfma_bf16_operands(int32_t workgroups, int32_t iters, const void* operands,
                                          float* sink, double* flops, void* stream) {
  if (!sink || !operands) return fail(MISA_ERR_INVALID_ARG, "sink or operands is NULL");
  if (!aligned(operands, 16)) return fail(MISA_ERR_INVALID_ARG, "operands must be 16-byte aligned");
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
    return fail(MISA_ERR_INVALID_ARG, "need 1 <= workgroups <= 2^20 and 1 <= iters <= 2^24");
  if (flops) *flops = (double)workgroups * 4.0 * (double)iters * misa::kProbeMfmaFlopsPerWaveIter;
  return hip_result(misa::launch_probe_mfma(workgroups, iters, operands, sink, (hipStream_t)stream),
                    "misa_probe_mfma_bf16_operands launch");
}

}  // extern "C"
