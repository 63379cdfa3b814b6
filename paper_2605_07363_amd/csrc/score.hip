// Stage 3: token scoring with the routed heads (Eq. misa_score; with all heads
// Eq. dsa_score).  Also used for the candidate re-scoring of Eq. misa_final_topk.
//
// score_stream_kernel (bf16 queries, bf16 or fp8 keys, whole-cache scoring):
//   the decode hot loop.  Every key byte is read exactly once, straight from
//   HBM into registers: a wavefront takes 64 consecutive keys per step as four
//   16-key tiles, each lane loading one contiguous quarter row.  The h dot
//   products per key are evaluated by the matrix core as a 16-row (heads,
//   zero-padded) x 16-column (keys) x 128 product (v_mfma_f32_16x16x32_bf16),
//   which keeps the vector ALU nearly idle so that the kernel stays bound by
//   HBM; fp8 codes are widened to bf16 exactly and the per-token scale is
//   applied after the head sum (ReLU(c x) = c ReLU(x) for c >= 0).  The sum
//   over heads is in-lane for the four rows a lane holds and then a two-step
//   exchange across the four 16-lane groups that leaves lane i with the score
//   of key i of the 64-key group, so stores are fully coalesced.
//
// score_generic_kernel: plain fp32 FMA path for every other combination
//   (fp32 inputs, candidate lists).  One thread per key or candidate; the
//   gathered query heads sit in LDS and are read by broadcast.
#include <algorithm>
#include <type_traits>

#include "kernels.h"
#include "small_topk.h"

namespace misa {

// ------------------------------------------------------------------ generic
template <int KDT, int QDT>
__global__ __launch_bounds__(256) void score_generic_kernel(
    Prob p, const void* __restrict__ Q, const float* __restrict__ W, const int* __restrict__ heads,
    const void* __restrict__ K, const float* __restrict__ kscale, const int* __restrict__ cand,
    int k_cand, float* __restrict__ out) {
  __shared__ float qs[kMaxH][kD];
  __shared__ float wsm[kMaxH];
  using KV = Vec16<KDT>;
  using QV = Vec16<QDT>;
  const int t = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  const int n = visible(p, seq, t);
  const int hc = heads ? p.h : p.H;
  const int hpad = (hc + 7) & ~7;
  const size_t qrow = (size_t)seq * p.n_q + t;

  // Gather the active heads (zero rows for padding and for invalid indices).
  for (int i = tid; i < hpad * (kD / QV::N); i += 256) {
    const int j = i / (kD / QV::N), c = i % (kD / QV::N);
    int head = -1;
    if (j < hc) head = heads ? heads[qrow * p.h + j] : j;
    float v[QV::N];
    if (head >= 0 && head < p.H) {
      QV::load(static_cast<const char*>(Q) + ((qrow * p.H + head) * kD + c * QV::N) * (QV::ROW_BYTES / kD), v);
    } else {
#pragma unroll
      for (int e = 0; e < QV::N; ++e) v[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < QV::N; ++e) qs[j][c * QV::N + e] = v[e];
  }
  for (int j = tid; j < hpad; j += 256) {
    int head = -1;
    if (j < hc) head = heads ? heads[qrow * p.h + j] : j;
    wsm[j] = (head >= 0 && head < p.H) ? W[qrow * p.H + head] : 0.f;
  }
  __syncthreads();

  const int row_len = cand ? k_cand : p.L;
  const int slot = blockIdx.x * 256 + tid;
  if (slot >= row_len) return;
  const int s = cand ? cand[qrow * k_cand + slot] : slot;
  float result = -INFINITY;
  if (s >= 0 && s < n) {
    const size_t kslot = key_slot(p, seq, s);
    const char* krow = static_cast<const char*>(K) + kslot * KV::ROW_BYTES;
    float total = 0.f;
    for (int hg = 0; hg < hpad; hg += 8) {
      float acc[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = 0.f;
      for (int c = 0; c < kD / KV::N; ++c) {
        float kv[KV::N];
        KV::load(krow + c * 16, kv);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
          for (int e = 0; e < KV::N; ++e) acc[j] = fmaf(qs[hg + j][c * KV::N + e], kv[e], acc[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) total = fmaf(wsm[hg + j], relu(acc[j]), total);
    }
    if (KDT == MISA_FP8_E4M3) total *= kscale[kslot];
    result = total;
  }
  out[qrow * row_len + slot] = result;
}

// ------------------------------------------------------------------ streaming
// Widen 4 packed fp8 codes to 4 bf16 (exact: 3 mantissa bits fit in 7; scale 1).
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
__device__ __forceinline__ void fp8x4_to_bf16x4(uint32_t w, uint32_t& lo, uint32_t& hi) {
  union { bf16x2 v; uint32_t u; } a, b;
  a.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);  // codes 0,1
  b.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);   // codes 2,3
  lo = a.u;
  hi = b.u;
}

union Frag {
  bf16x8 v;
  uint4 u;
  uint32_t w[4];
};

typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8;
union Frag8 {   // 32 fp8 codes: one operand of the fp8 matrix instruction
  i32x8 v;
  uint4 u[2];
};

// Buffer descriptors (raw, unstrided): accesses at byte offsets >= num_bytes read zeros and
// drop stores.  Addresses are descriptor base + per-lane byte offset + wave-uniform byte offset.
using BufferRsrc = __amdgpu_buffer_rsrc_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
// base and num_bytes must be the same in every lane: they are moved to scalar registers here,
// so that the compiler keeps the descriptor there instead of looping over "distinct" lanes.
__device__ __forceinline__ BufferRsrc make_rsrc(const void* base, uint32_t num_bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  void* uniform = reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(uniform, 0, (int)__builtin_amdgcn_readfirstlane(num_bytes), 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load16(BufferRsrc r, uint32_t lane_off, uint32_t wave_off = 0) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)wave_off, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
__device__ __forceinline__ void buffer_store8(BufferRsrc r, uint32_t lane_off, uint32_t x, uint32_t y) {
  const u32x2 v = {x, y};
  __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)lane_off, 0, 0);
}
// Per lane: a where the lane's bit of the wave mask is set, else b (one v_cndmask on the mask).
template <typename T>
__device__ __forceinline__ T select_by_mask(unsigned long long mask, T a, T b) {
  static_assert(sizeof(T) == 4, "32-bit values");
  uint32_t r;
  asm("v_cndmask_b32 %0, %1, %2, %3" : "=v"(r) : "v"((uint32_t)b), "v"((uint32_t)a), "s"(mask));
  return (T)r;
}
__device__ __forceinline__ void buffer_store4(BufferRsrc r, uint32_t lane_off, uint32_t wave_off, float x) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(x), r, (int)lane_off, (int)wave_off, 0);
}

// NT = 16-row head tiles (heads <= 16 * NT); a wavefront takes STEPS pipeline
// steps of G 64-key groups each.
template <int KDT, int NT, int STEPS, int G, bool PAGED>
__global__ __launch_bounds__(256) void score_stream_kernel(
    Prob p, const uint16_t* __restrict__ Q, const float* __restrict__ W,
    const int* __restrict__ heads, const void* __restrict__ K, const float* __restrict__ kscale,
    float* __restrict__ S) {
  constexpr int ROW_BYTES = KDT == MISA_BF16 ? 256 : 128;
  constexpr int NLD = KDT == MISA_BF16 ? 4 : 2;  // 16-byte loads per lane and 16-key tile
  constexpr int KPW = 256 * STEPS * G;           // keys per workgroup
  const int t = blockIdx.y, seq = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, g = lane >> 4;
  const int n = visible(p, seq, t);
  const int hc = heads ? p.h : p.H;
  const size_t qrow = (size_t)seq * p.n_q + t;

  const char* kbase = static_cast<const char*>(K) + (size_t)seq * p.L * ROW_BYTES;
  const float* sbase = kscale + (size_t)seq * p.L;
  float* srow = S + qrow * p.L;
  const int k_begin = blockIdx.x * KPW;
  const int k_end = min(k_begin + KPW, p.L);

  Frag a[NT][4];   // query operand and gates, filled after the first key loads are issued
  float wv[NT][4];

  // A workgroup whose whole key range is invisible only writes -inf.
  if (k_begin >= n) {
    for (int key = k_begin + threadIdx.x; key < k_end; key += 256) srow[key] = -INFINITY;
    return;
  }

  // Raw 16-byte key chunks of one 64-key group: 4 tiles x NLD loads per lane.
  // Loads are unconditional and branch-free (rows clamped into the cache), so
  // that the number of loads in flight is known at every wait.
  struct Raw { uint4 v[4][NLD]; float scale; };
  // Page pool: a 64-key group starts at a multiple of 64, so with pages of 64 tokens or more
  // all its keys (and the last key, when rows are clamped to it) lie in one page, found with
  // one wavefront-uniform table read; smaller pages are looked up per lane.
  auto issue_loads = [&](Raw& r, int kg) {
    size_t group_slot = 0;
    const bool one_page = PAGED && p.page_shift >= 6;
    if (one_page)
      group_slot = (size_t)p.page_table[(size_t)seq * p.max_pages + (min(kg, p.L - 1) >> p.page_shift)] << p.page_shift;
    const int in_page = (1 << p.page_shift) - 1;
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      const int row = min(kg + tt * 16 + c, p.L - 1);
      const uint4* src;
      if (!PAGED) src = reinterpret_cast<const uint4*>(kbase + (size_t)row * ROW_BYTES) + g;
      else {
        const size_t slot = one_page ? group_slot + (row & in_page) : key_slot<true>(p, seq, row);
        src = reinterpret_cast<const uint4*>(static_cast<const char*>(K) + slot * ROW_BYTES) + g;
      }
#pragma unroll
      for (int i = 0; i < NLD; ++i) r.v[tt][i] = src[4 * i];
    }
    r.scale = 1.f;
    if (KDT == MISA_FP8_E4M3) {
      const int row = min(kg + lane, p.L - 1);
      if (!PAGED) r.scale = sbase[row];
      else r.scale = kscale[one_page ? group_slot + (row & in_page) : key_slot<true>(p, seq, row)];
    }
  };

  auto finish_group = [&](const Raw& r, int kg) {
    const int key = kg + lane;  // the key this lane finally owns
    if (kg >= k_end) return;
    if (kg >= n) {              // whole group invisible
      if (key < p.L) srow[key] = -INFINITY;
      return;
    }
    float part[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      Frag b[4];
      if (KDT == MISA_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i].u = r.v[tt][i % NLD];
      } else {
        const uint4 lo = r.v[tt][0], hi = r.v[tt][NLD - 1];
        const uint32_t w8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          fp8x4_to_bf16x4(w8[2 * i], b[i].w[0], b[i].w[1]);
          fp8x4_to_bf16x4(w8[2 * i + 1], b[i].w[2], b[i].w[3]);
        }
      }
      float s = 0.f;
#pragma unroll
      for (int T = 0; T < NT; ++T) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[T][i].v, b[i].v, acc, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) s = fmaf(wv[T][j], relu(acc[j]), s);
      }
      part[tt] = s;
    }
    // Sum over the four lane groups so that group g ends with tile g.
    const bool up2 = (g & 2) != 0, up1 = (g & 1) != 0;
    const float r0 = __shfl_xor(up2 ? part[0] : part[2], 32);
    const float r1 = __shfl_xor(up2 ? part[1] : part[3], 32);
    const float k0 = (up2 ? part[2] : part[0]) + r0;
    const float k1 = (up2 ? part[3] : part[1]) + r1;
    const float r2 = __shfl_xor(up1 ? k0 : k1, 16);
    const float fin = (up1 ? k1 : k0) + r2;
    if (key < p.L) srow[key] = key < n ? fin * r.scale : -INFINITY;
  };

  // Software pipeline with two register buffers, fully unrolled: the loads of
  // the next group are all in flight before the current one is consumed.  The
  // first key loads are issued before the query operand is gathered, so the
  // dependent head-index -> gate / query loads overlap with them.
  Raw buf[2][G];
  const int kg0 = k_begin + wave * (64 * G);
#pragma unroll
  for (int q = 0; q < G; ++q) issue_loads(buf[0][q], kg0 + 64 * q);
  __builtin_amdgcn_sched_barrier(0);

  __shared__ int s_head[kMaxH];
  __shared__ float s_gate[kMaxH];
  if (threadIdx.x < kMaxH) {
    const int r = threadIdx.x;
    int head = -1;
    if (r < hc) head = heads ? heads[qrow * p.h + r] : r;
    const bool ok = head >= 0 && head < p.H;
    s_head[r] = ok ? head : -1;
    s_gate[r] = ok ? W[qrow * p.H + head] : 0.f;
  }
  __syncthreads();

  // A operand: head rows.  The four lanes (c, g = 0..3) that share key column c
  // read 64 contiguous bytes of a key row per load instruction (16-byte chunk
  // 4 i + g for load i), so for bf16 keys k-step i covers components
  // 8 (4 i + g) .. + 7, and for fp8 keys load i feeds k-steps 2 i and 2 i + 1
  // with components 16 (4 i + g) + 8 j .. + 7.  The query fragments use the same
  // component mapping, so the contraction still runs over all 128.
#pragma unroll
  for (int T = 0; T < NT; ++T) {
    const int head = s_head[T * 16 + c];
    const uint16_t* src = Q + (qrow * p.H + max(head, 0)) * kD;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int comp = KDT == MISA_BF16 ? 8 * (4 * i + g) : 16 * (4 * (i >> 1) + g) + 8 * (i & 1);
      const uint4 v = *reinterpret_cast<const uint4*>(src + comp);
      a[T][i].u = head >= 0 ? v : make_uint4(0, 0, 0, 0);
    }
    // The accumulator of lane (c, g) holds head rows 4 g + j (j = 0..3) for key column c.
#pragma unroll
    for (int j = 0; j < 4; ++j) wv[T][j] = s_gate[T * 16 + 4 * g + j];
  }

#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    if (st + 1 < STEPS) {
#pragma unroll
      for (int q = 0; q < G; ++q) issue_loads(buf[(st + 1) & 1][q], kg0 + (st + 1) * 256 * G + 64 * q);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < G; ++q) finish_group(buf[st & 1][q], kg0 + st * 256 * G + 64 * q);
  }
}

// ------------------------------------------------------------------ prefill
// score_tile_kernel (bf16 queries, bf16 or fp8 keys, many queries per sequence):
//   a dense contraction [queries x heads, 128] x [128, keys] on the matrix core
//   (v_mfma_f32_32x32x16_bf16).  A workgroup owns a tile of queries and a range
//   of keys.  Each wavefront keeps the gathered head rows of its own queries
//   in registers for the whole key range (the query operand is stationary),
//   while 64-key tiles stream through LDS, double buffered, widened to bf16
//   once when they are staged, rows padded by one 16-byte slot so that fragment reads are
//   free of bank conflicts.  Head rows are placed so that all active heads of
//   a query fall into accumulator registers of the same lane: a lane of the
//   lower half-wave holds rows {0-3, 8-11, 16-19, 24-27} of a 32-row tile,
//   the upper half the others, so ReLU, gate and the sum over heads need no
//   cross-lane traffic, and 32 consecutive lanes store 32 consecutive keys.
//   blockIdx.x is the key range and a multiple of 8 of them is launched, so
//   workgroups that share a key range run on the same XCD and its L2.
//
// HS = head slots per query (h rounded up to 8, 16, 32 or 64).
// WIDE (fp8 operands, 8 head slots, scores stored): four row tiles as well - the operands are half
// as wide, and that kernel is bound by the vector work per key tile, which a wavefront with 16
// queries shares over twice as many products (0.40 ms against 0.46 ms on the 131072-key prefill
// workload).  The filter mode stays with two (its list work needs the second wavefront per SIMD
// to hide behind: 0.99 ms against 0.67 ms for the fused call with four).
template <int HS, bool WIDE>
struct TileGeom {
  static constexpr int RT = (HS > 32 || (WIDE && HS == 8)) ? 4 : 2;   // 32-row tiles per wavefront
  static constexpr int QW = RT * 32 / HS;       // queries per wavefront
  static constexpr int QWG = 4 * QW;            // queries per workgroup
  // query (within the wavefront) and head slot of accumulator register r of
  // row tile rt in half-wave hf
  __device__ static __forceinline__ int query_of(int rt, int hf, int r) {
    if (HS == 8) return rt * 4 + hf * 2 + (r >> 3);
    if (HS == 16) return rt * 2 + hf;
    return hf;
  }
  __device__ static __forceinline__ int slot_of(int rt, int r) {
    if (HS == 8) return r & 7;
    if (HS == 16) return r;
    return rt * 16 + r;
  }
};

constexpr int kKT = 64;  // keys per LDS tile
constexpr int kKP = 17;  // 16-byte slots per key row in LDS: 16 of data + 1 of padding
constexpr int kKP8 = 9;  // the same for rows kept as fp8 codes: 8 of data + 1 of padding
// Queries per sequence from which the tiled matrix-core kernel is used.
constexpr int kTileMinQueries = 8;

// MODE kTileStore: scores of all keys go to S [rows, L].
// MODE kTileSample: only one key of every group of kSampleStride consecutive
//   keys is scored (at a hashed position inside its group); the result is a
//   score matrix [rows, L / kSampleStride] in which a query sees the first
//   n / kSampleStride entries.
// MODE kTileFilter: nothing is stored densely; (key, score) pairs whose score reaches the row's
//   threshold aux.tau go to the row's candidate list.  The list of a row is cut into one
//   segment per key range (aux.seg: offsets [rows, ranges + 1], sized by the caller from the
//   sampled scores of that range), and the workgroup of a (query tile, key range) is the only
//   writer of its segments: a wavefront keeps the fill of its queries' segments in scalar
//   registers, computes the slots of a column tile's hits from the ballot, and stores them
//   straight to the list through a buffer descriptor - lanes without a hit, or past the end of
//   the segment, store to an offset outside the descriptor's range, which drops the store, so
//   there is no branch, no staging list and no atomic.  At the end the fills are written to
//   aux.seg_count [rows, ranges] (a fill above the segment's length tells the caller that it
//   overflowed).
// The work of one workgroup: query tile q_tile of sequence blockIdx.z, key range blockIdx.x.
template <int KDT, int HS, int MODE, bool PAGED, bool Q8>
__device__ __forceinline__ void score_tile_body(
    const Prob& p, int keys_per_wg, const uint16_t* __restrict__ Q, const float* __restrict__ W,
    const int* __restrict__ heads, const void* __restrict__ K, const float* __restrict__ kscale,
    float* __restrict__ S, const TileAux& aux, int q_tile) {
  using G = TileGeom<HS, Q8 && MODE == kTileStore>;
  constexpr int RT = G::RT, QW = G::QW, QWG = G::QWG;
  constexpr bool FILTER = MODE == kTileFilter, SAMPLE = MODE == kTileSample;
  constexpr int NQL_ = HS == 8 ? RT * 2 : (HS == 16 ? RT : 1);  // queries per lane
  constexpr int ROW_BYTES = KDT == MISA_BF16 ? 256 : 128;
  constexpr int NLD = KDT == MISA_BF16 ? 4 : 2;  // 16-byte global loads per thread and tile
  // Q8: queries and keys are both e4m3 codes and stay so: the tile holds raw key rows (8 slots +
  // 1 of padding) and the products run on the fp8 matrix instruction (K = 64 per instruction).
  static_assert(!Q8 || KDT == MISA_FP8_E4M3, "fp8 queries contract with fp8 keys only");
  constexpr int KP = Q8 ? kKP8 : kKP;     // 16-byte slots per key row in LDS
  constexpr int KS = Q8 ? 2 : 8;          // matrix instructions per 32 x 32 output tile
  __shared__ uint4 ktile[2][kKT * KP];
  __shared__ float kscl[2][kKT];
  __shared__ int nvis[QWG];
  __shared__ int s_head[QWG][HS];
  __shared__ float s_tau[FILTER ? QWG : 1];  // thresholds of the workgroup's queries (+inf: no such query)

  const int LT = SAMPLE ? p.L / kSampleStride : p.L;  // keys in tile space
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, hf = lane >> 5;
  const int seq = blockIdx.z;
  const int q_base = q_tile * QWG;
  const int k_begin = blockIdx.x * keys_per_wg;
  const int k_end = min(k_begin + keys_per_wg, LT);
  const int hc = heads ? p.h : p.H;

  for (int i = tid; i < QWG; i += 256) {
    const int n = q_base + i < p.n_q ? visible(p, seq, q_base + i) : 0;
    nvis[i] = SAMPLE ? n / kSampleStride : n;
    if (FILTER) s_tau[i] = q_base + i < p.n_q ? aux.tau[(size_t)seq * p.n_q + q_base + i] : INFINITY;
  }
  for (int i = tid; i < QWG * HS; i += 256) {
    const int qi = i / HS, slot = i % HS, q = q_base + qi;
    int head = -1;
    if (q < p.n_q && slot < hc) head = heads ? heads[((size_t)seq * p.n_q + q) * p.h + slot] : slot;
    s_head[qi][slot] = (head >= 0 && head < p.H) ? head : -1;
  }
  __syncthreads();
  int n_max = 0;
  for (int i = 0; i < QWG; ++i) n_max = max(n_max, nvis[i]);
  const int k_stop = min(k_end, n_max);  // keys at or beyond this are invisible to every query here

  // Stationary operand: row m = col of row tile rt belongs to half-wave (m >> 2) & 1 of the
  // accumulator and to its register r = (m >> 3) * 4 + (m & 3).
  Frag a[RT][Q8 ? 1 : 8];
  Frag8 a8[RT][Q8 ? 2 : 1];   // fp8 operands: k-step ks, half-wave hf: components 64 ks + 32 hf .. + 31
  float gate[RT][16];
  {
    const int m = col, mhf = (m >> 2) & 1, mr = (m >> 3) * 4 + (m & 3);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int qi = wave * QW + G::query_of(rt, mhf, mr), slot = G::slot_of(rt, mr);
      const int head = s_head[qi][slot];
      const size_t qhead = (((size_t)seq * p.n_q + min(q_base + qi, p.n_q - 1)) * p.H + max(head, 0)) * kD;
      if (Q8) {
        const uint8_t* src = reinterpret_cast<const uint8_t*>(Q) + qhead + hf * 32;
#pragma unroll
        for (int ks = 0; ks < (Q8 ? 2 : 0); ++ks)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const uint4 v = *reinterpret_cast<const uint4*>(src + ks * 64 + u * 16);
            a8[rt][ks].u[u] = head >= 0 ? v : make_uint4(0, 0, 0, 0);
          }
      } else {
        const uint16_t* src = Q + qhead + hf * 8;
#pragma unroll
        for (int ks = 0; ks < (Q8 ? 0 : 8); ++ks) {
          const uint4 v = *reinterpret_cast<const uint4*>(src + ks * 16);
          a[rt][ks].u = head >= 0 ? v : make_uint4(0, 0, 0, 0);
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qj = wave * QW + G::query_of(rt, hf, r);
        const int hd = s_head[qj][G::slot_of(rt, r)];
        gate[rt][r] = hd >= 0 ? W[((size_t)seq * p.n_q + min(q_base + qj, p.n_q - 1)) * p.H + hd] : 0.f;
      }
    }
  }

  const char* kbase = static_cast<const char*>(K) + (PAGED ? (size_t)0 : (size_t)seq * p.L * ROW_BYTES);
  // Staging registers of the next key tile (global -> registers -> LDS).  Thread
  // tid moves the 16-byte chunks tid + 256 i of the tile.
  constexpr int CPR = ROW_BYTES / 16;  // chunks per key row
  // Which chunk of the tile a thread stages: chunk stid + 256 i.  fp8 rows that are widened on
  // the way (each 16-byte chunk becomes two LDS slots) permute the chunks inside every group of
  // 16 lanes (= two key rows), so that eight consecutive lanes cover four chunks of one row and
  // the same four of the next: their LDS stores then fall into eight different 16-byte bank
  // groups (rows are 17 slots apart), where eight chunks of one row hit only the four even ones
  // (measured: 24 % of this kernel's LDS cycles were bank conflicts, none with bf16 rows).
  const int stid = (KDT == MISA_FP8_E4M3 && !Q8)
                       ? ((tid & ~15) | (((tid >> 2) & 1) << 3) | ((tid & 3) + 4 * ((tid >> 3) & 1)))
                       : tid;
  uint4 st0 = make_uint4(0, 0, 0, 0), st1 = st0, st2 = st0, st3 = st0;
  float st_scale = 1.f;
  // A contiguous, unsampled cache is read through a buffer descriptor of the sequence's keys:
  // a tile is one linear piece (thread tid takes bytes 16 tid + 4096 i of it), so a thread's
  // offsets only advance by the tile size, and rows past the end of the cache read as zeros
  // (the descriptor's range check) instead of being clamped per lane.
  constexpr bool LINEAR = !SAMPLE && !PAGED;
  const BufferRsrc krsrc = make_rsrc(kbase, (uint32_t)p.L * (uint32_t)ROW_BYTES);
  uint32_t koff = (uint32_t)k_begin * ROW_BYTES + (uint32_t)stid * 16u;  // next tile to request
  // Cache row of key j of tile space (clamped into the cache).  Sampling takes key
  // 16 j + (top four bits of a multiplicative hash of j) of every group of 16.
  // With a page table the row is the one in the page pool and kbase the pool itself.
  auto key_row = [&](int j) -> size_t {
    j = min(j, LT - 1);
    if (SAMPLE) j = j * kSampleStride + (int)(((uint32_t)j * 2654435761u) >> 28);
    return PAGED ? key_slot<true>(p, seq, j) : (size_t)j;
  };
  // Requests the tile that starts at key k0; successive calls ask for successive tiles.
#define MISA_TILE_LOAD(k0)                                                                        \
  do {                                                                                            \
    if (LINEAR) {                                                                                 \
      st0 = buffer_load16(krsrc, koff);                                                           \
      st1 = buffer_load16(krsrc, koff + 4096u);                                                   \
      if (NLD == 4) {                                                                             \
        st2 = buffer_load16(krsrc, koff + 8192u);                                                 \
        st3 = buffer_load16(krsrc, koff + 12288u);                                                \
      }                                                                                           \
      koff += kKT * ROW_BYTES;                                                                    \
    } else {                                                                                      \
      st0 = *reinterpret_cast<const uint4*>(kbase + key_row((k0) + stid / CPR) * ROW_BYTES + (stid % CPR) * 16); \
      st1 = *reinterpret_cast<const uint4*>(kbase + key_row((k0) + (stid + 256) / CPR) * ROW_BYTES + (stid % CPR) * 16); \
      if (NLD == 4) {                                                                             \
        st2 = *reinterpret_cast<const uint4*>(kbase + key_row((k0) + (stid + 512) / CPR) * ROW_BYTES + (stid % CPR) * 16); \
        st3 = *reinterpret_cast<const uint4*>(kbase + key_row((k0) + (stid + 768) / CPR) * ROW_BYTES + (stid % CPR) * 16); \
      }                                                                                           \
    }                                                                                             \
    if (KDT == MISA_FP8_E4M3 && tid < kKT) st_scale = kscale[(PAGED ? (size_t)0 : (size_t)seq * p.L) + key_row((k0) + tid)]; \
  } while (0)
  // registers -> LDS (bf16, padded rows): chunk stid + 256 i is chunk stid % CPR of row
  // stid / CPR + (256 / CPR) i, so the four writes differ by a constant
  uint4* const lds_put = &ktile[0][0] + (stid / CPR) * KP + (KDT == MISA_BF16 || Q8 ? stid % CPR : 2 * (stid % CPR));
  auto put_chunk = [&](int b, int i, const uint4& v) {
    uint4* dst = lds_put + b * (kKT * KP) + i * ((256 / CPR) * KP);
    if (KDT == MISA_BF16 || Q8) {
      dst[0] = v;
    } else {
      uint4 lo, hi;
      fp8x4_to_bf16x4(v.x, lo.x, lo.y);
      fp8x4_to_bf16x4(v.y, lo.z, lo.w);
      fp8x4_to_bf16x4(v.z, hi.x, hi.y);
      fp8x4_to_bf16x4(v.w, hi.z, hi.w);
      dst[0] = lo;
      dst[1] = hi;
    }
  };
#define MISA_TILE_STORE(b)                                        \
  do {                                                            \
    put_chunk((b), 0, st0);                                       \
    put_chunk((b), 1, st1);                                       \
    if (NLD == 4) {                                               \
      put_chunk((b), 2, st2);                                     \
      put_chunk((b), 3, st3);                                     \
    }                                                             \
    if (KDT == MISA_FP8_E4M3 && tid < kKT) kscl[(b)][tid] = st_scale; \
  } while (0)

  // queries this lane reports: prefix lengths and 32-bit offsets of their score
  // rows relative to the first row of the tile (uniform base + lane offset stores)
  constexpr int NQL = HS == 8 ? RT * 2 : (HS == 16 ? RT : 1);  // queries per lane
  float* s_tile = S + ((size_t)seq * p.n_q + q_base) * LT;
  // Unmasked tiles store through a descriptor of the workgroup's score rows: the address of a
  // store is a per-lane constant (row, column inside the tile) plus the wave-uniform tile start.
  const BufferRsrc srsrc = make_rsrc(s_tile, (uint32_t)QWG * (uint32_t)LT * 4u);
  int qn[NQL];
  uint32_t qoff[NQL];
  // filter mode: thresholds of this lane's queries and the lengths of the wavefront's
  // staging lists (wavefront-uniform, so they live in scalar registers)
  float tauv[NQL];
  // fill of the list segments of the two queries in accumulator slot j (lower / upper half-wave):
  // wavefront-uniform; this lane's segment: first element (relative to the first list of the
  // query tile) and length
  int cnt[NQL], cnt_up[NQL];
  uint32_t seg_lo[NQL];
  int seg_len[NQL];
  const BufferRsrc crsrc = make_rsrc(FILTER ? static_cast<const void*>(aux.cand + ((size_t)seq * p.n_q + q_base) * aux.cap) : nullptr,
                                     FILTER ? (uint32_t)QWG * (uint32_t)aux.cap * 8u : 0u);
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  int n_min = 0x7FFFFFFF;
#pragma unroll
  for (int j = 0; j < NQL; ++j) {
    const int qi = wave * QW + (HS == 8 ? (j >> 1) * 4 + hf * 2 + (j & 1) : (HS == 16 ? j * 2 + hf : hf));
    const bool ok = q_base + qi < p.n_q;
    qn[j] = ok ? nvis[qi] : -1;   // -1: query does not exist, nothing is stored
    qoff[j] = (uint32_t)qi * (uint32_t)LT;
    cnt[j] = 0;
    cnt_up[j] = 0;
    tauv[j] = FILTER ? s_tau[qi] : 0.f;
    seg_lo[j] = 0;
    seg_len[j] = 0;
    if (FILTER && ok) {
      const int* sg = aux.seg + ((size_t)seq * p.n_q + q_base + qi) * (aux.ranges + 1) + blockIdx.x;
      const int lo = sg[0];
      seg_lo[j] = (uint32_t)qi * (uint32_t)aux.cap + (uint32_t)lo;
      seg_len[j] = sg[1] - lo;
    }
  }
  // Stores the hits of accumulator slot j named by the ballot m (score sc, key key of this
  // lane) into the segments of its two queries and advances their fills.
  const unsigned long long upper_half = 0xFFFFFFFF00000000ull;
  auto append_hits = [&](int j, unsigned long long m, int key, float sc) {
    const uint32_t m_lo = (uint32_t)m, m_hi = (uint32_t)(m >> 32);
    const int n_lo = __popc(m_lo);
    // slot = fill of the lane's own segment + hits of its half-wave below it (upper lanes see
    // all n_lo lower hits in the running count, so their fill is entered less n_lo)
    const int base = select_by_mask(upper_half, cnt_up[j] - n_lo, cnt[j] - cnt_up[j]);
    const int slot = __builtin_amdgcn_mbcnt_hi(m_hi, __builtin_amdgcn_mbcnt_lo(m_lo, base));
    const unsigned long long fits = __ballot(slot < seg_len[j]) & m;
    const uint32_t off = select_by_mask(fits, (seg_lo[j] + (uint32_t)slot) << 3, 0xFFFFFFF8u);
    buffer_store8(crsrc, off, (uint32_t)key, __float_as_uint(sc));
    cnt[j] += n_lo + __popc(m_hi);      // (cnt: both halves, cnt_up: the upper one)
    cnt_up[j] += __popc(m_hi);
  };

  for (int i = 0; i < QWG; ++i) n_min = min(n_min, q_base + i < p.n_q ? nvis[i] : -1);
  // tiles that end at or before plain_end are visible to every query of the
  // workgroup, all of which exist: no masks are needed there
  const int plain_end = min(n_min, k_end);

  // LDS fragment position of this lane (16-byte units): row col of column tile 0, chunk
  // 2 ks + hf.  Rows are 17 slots apart, so the 16 lanes that read together hit 16 different
  // bank groups, and the k-step only adds a constant: one address register per step.
  // (fp8 rows: 9 slots apart, chunks 4 ks + 2 hf and the next one)
  const int frag0 = Q8 ? col * KP + 2 * hf : col * KP + hf;
  // The key fragments of one 32-key column tile (tile: (buffer * 64 + column tile * 32) * KP)
  // and one matrix instruction of it: row tile rt, k-step ks, onto acc (first: onto zero).
  struct KeyFrags {
    Frag b[Q8 ? 1 : 8];
    Frag8 b8[Q8 ? 2 : 1];
  };
  auto load_frags = [&](KeyFrags& f, int tile) {
    if (Q8) {
#pragma unroll
      for (int ks = 0; ks < (Q8 ? 2 : 0); ++ks) {
        f.b8[ks].u[0] = (&ktile[0][0])[frag0 + tile + 4 * ks];
        f.b8[ks].u[1] = (&ktile[0][0])[frag0 + tile + 4 * ks + 1];
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < (Q8 ? 0 : 8); ++ks) f.b[ks].u = (&ktile[0][0])[frag0 + tile + 2 * ks];
    }
  };
  auto mma = [&](const KeyFrags& f, int rt, int ks, const f32x16& acc, bool first) -> f32x16 {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (Q8)
      return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8[rt][ks].v, f.b8[ks].v, first ? zero : acc, 0, 0, 0, 0, 0, 0);
    else
      return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, f.b[ks].v, first ? zero : acc, 0, 0, 0);
  };
  // One 32-key column tile: KS x RT matrix instructions.
  auto mfma_tile = [&](f32x16 (&acc)[RT], int tile) {
    KeyFrags f;
    load_frags(f, tile);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) acc[rt] = mma(f, rt, ks, acc[rt], ks == 0);
  };
  // ReLU, gate, head sum and store of one finished column tile.  PLAIN: every
  // query of the workgroup exists and sees the whole tile, so nothing is masked.
  // the gated ReLU of accumulator register r of row tile rt, added to its query's sum
  auto head_term = [&](float (&out)[NQL], const f32x16 (&acc)[RT], int rt, int r) {
    const int j = HS == 8 ? rt * 2 + (r >> 3) : (HS == 16 ? rt : 0);
    out[j] = fmaf(gate[rt][r], relu(acc[rt][r]), out[j]);
  };
  auto finish = [&](auto plain_tag, float (&out)[NQL], int key, float scale) {
    constexpr bool PLAIN = decltype(plain_tag)::value;
    const int key0 = __builtin_amdgcn_readfirstlane(key - col);   // first key of the column tile
    if (KDT == MISA_FP8_E4M3) {
#pragma unroll
      for (int j = 0; j < NQL; ++j) out[j] *= scale;
    }
    if (FILTER) {
#pragma unroll
      for (int j = 0; j < NQL; ++j) {
        const bool pass = out[j] >= tauv[j] && (PLAIN || (key < k_end && key < qn[j]));
        append_hits(j, __ballot(pass), key, out[j]);
      }
    } else if (PLAIN) {
#pragma unroll
      for (int j = 0; j < NQL; ++j) buffer_store4(srsrc, (qoff[j] + (uint32_t)col) * 4u, (uint32_t)key0 * 4u, out[j]);
    } else {
#pragma unroll
      for (int j = 0; j < NQL; ++j)
        if (key < k_end && qn[j] >= 0) s_tile[qoff[j] + (uint32_t)key] = key < qn[j] ? out[j] : -INFINITY;
    }
  };
  auto epilogue = [&](auto plain_tag, const f32x16 (&acc)[RT], int key, float scale) {
    float out[NQL];
#pragma unroll
    for (int j = 0; j < NQL; ++j) out[j] = 0.f;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) head_term(out, acc, rt, r);
    finish(plain_tag, out, key, scale);
  };
  constexpr int TPM = 16 / KS;   // head-sum terms that follow each matrix instruction
  static_assert(KS * RT >= NQL, "one list append per matrix instruction must cover all lists");
  // The matrix instructions of column tile ct into acc_new, each followed by its share
  // (TPM accumulator registers) of the head sums of the previous column tile acc_old;
  // scheduling barriers pin that order, so a wavefront feeds both pipes at once.
  auto tile_step = [&](auto plain_tag, f32x16 (&acc_new)[RT], int tile,
                       const f32x16 (&acc_old)[RT], int key, float scale) {
    KeyFrags f;
    load_frags(f, tile);
    float out[NQL];
#pragma unroll
    for (int j = 0; j < NQL; ++j) out[j] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        acc_new[rt] = mma(f, rt, ks, acc_new[rt], ks == 0);
        const int e = (ks * RT + rt) * TPM;   // KS RT steps x TPM = the 16 RT accumulator registers
#pragma unroll
        for (int u = 0; u < TPM; ++u) head_term(out, acc_old, (e + u) / 16, (e + u) % 16);
        // an empty volatile statement on the running sum keeps these operations between
        // the two scheduling barriers (plain arithmetic would be free to move past them)
        asm volatile("" : "+v"(out[HS == 8 ? (e / 16) * 2 + ((e % 16) >> 3) : (HS == 16 ? e / 16 : 0)]));
        __builtin_amdgcn_sched_barrier(0);
      }
    finish(plain_tag, out, key, scale);
  };
  // Filter mode uses the same fixed pattern, with the list bookkeeping of a column tile put off
  // by one step: a step ends with the compare and ballot of its own sums only (the masks stay
  // in scalar registers, the sums in NQL vector registers), and the slot arithmetic and the
  // staged writes of those candidates sit between the first matrix instructions of the next
  // step instead of after the last one, where nothing of this wavefront would cover them.
  unsigned long long pend_m[NQL];
  float pend_out[NQL];
  int pend_key = 0;  // the lane's key of the step the pending sums are from
#pragma unroll
  for (int j = 0; j < NQL; ++j) {
    pend_m[j] = 0;
    pend_out[j] = 0.f;
  }
  auto append_pending = [&](int j) { append_hits(j, pend_m[j], pend_key, pend_out[j]); };
  auto drain_pending = [&]() {
#pragma unroll
    for (int j = 0; j < NQL; ++j) {
      append_pending(j);
      pend_m[j] = 0;
    }
  };
  auto filter_step = [&](auto plain_tag, f32x16 (&acc_new)[RT], int tile, const f32x16 (&acc_old)[RT],
                         int key, float scale) {
    constexpr bool PLAIN = decltype(plain_tag)::value;
    KeyFrags f;
    load_frags(f, tile);
    float out[NQL];
#pragma unroll
    for (int j = 0; j < NQL; ++j) out[j] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        acc_new[rt] = mma(f, rt, ks, acc_new[rt], ks == 0);
        const int e = (ks * RT + rt) * TPM;
#pragma unroll
        for (int u = 0; u < TPM; ++u) head_term(out, acc_old, (e + u) / 16, (e + u) % 16);
        if (ks * RT + rt < NQL) append_pending(ks * RT + rt);
        asm volatile("" : "+v"(out[HS == 8 ? (e / 16) * 2 + ((e % 16) >> 3) : (HS == 16 ? e / 16 : 0)]));
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
    for (int j = 0; j < NQL; ++j) {
      const float o = KDT == MISA_FP8_E4M3 ? out[j] * scale : out[j];
      const bool pass = o >= tauv[j] && (PLAIN || (key < k_end && key < qn[j]));
      pend_m[j] = __ballot(pass);
      pend_out[j] = o;
    }
    pend_key = key;
  };
  using Yes = std::true_type;
  using No = std::false_type;
  // The column tiles of the key range form one stream; the MFMAs of a tile are
  // issued together with the epilogue of the tile before it (two accumulator
  // sets), so matrix and vector pipes overlap inside a wavefront.  Per 64-key
  // LDS tile: [tile i, columns 32..63 | epilogue of columns 0..31], stage tile
  // i+1 into the other LDS buffer, barrier, [tile i+1, columns 0..31 | epilogue
  // of tile i, columns 32..63].
  // Per iteration j, in one straight line: request tile j + 2, [tile j+1, columns 0..31 |
  // epilogue of tile j, columns 32..63], [tile j+1, columns 32..63 | epilogue of tile j+1,
  // columns 0..31], stage tile j + 2 into the LDS buffer tile j has left, barrier.  Requests
  // and staging are unconditional (tiles past the range read zeros or clamped rows into a
  // buffer nobody reads), so an iteration has no branch between a request and its use and
  // every wait counts exactly the score stores issued in between.
  const int n_tiles = k_begin < k_stop ? (k_stop - k_begin + kKT - 1) / kKT : 0;
  if (n_tiles > 0) {
    MISA_TILE_LOAD(k_begin);
    {   // the second tile is requested before the first is staged (the registers are still free)
      const uint4 f0 = st0, f1 = st1, f2 = st2, f3 = st3;
      const float fs = st_scale;
      MISA_TILE_LOAD(k_begin + kKT);
      put_chunk(0, 0, f0);
      put_chunk(0, 1, f1);
      if (NLD == 4) {
        put_chunk(0, 2, f2);
        put_chunk(0, 3, f3);
      }
      if (KDT == MISA_FP8_E4M3 && tid < kKT) kscl[0][tid] = fs;
    }
    MISA_TILE_STORE(1);
    // Every load of the prologue (query operand, gates) has landed before the loop
    // starts, so the waits inside the loop only concern loads issued inside it.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    f32x16 accA[RT], accB[RT];
    float scaleA = 1.f, scaleB = 1.f;
    mfma_tile(accA, 0);
    if (KDT == MISA_FP8_E4M3) scaleA = kscl[0][col];
    // leading tiles that need no masks, then the rest
    const int n_plain = min(n_tiles, max(0, (plain_end - k_begin) / kKT));
    auto half = [&](auto tag) {   // tile 0, columns 32..63 | epilogue of its columns 0..31
      if (FILTER) filter_step(tag, accB, 32 * KP, accA, k_begin + col, scaleA);
      else tile_step(tag, accB, 32 * KP, accA, k_begin + col, scaleA);
      if (KDT == MISA_FP8_E4M3) scaleB = kscl[0][32 + col];
    };
    if (n_plain > 0) half(Yes{});
    else half(No{});
    auto body = [&](auto tag, int j) {
      const int nb = (j + 1) & 1, k0 = k_begin + j * kKT;
      MISA_TILE_LOAD(k0 + 2 * kKT);
      if (FILTER) filter_step(tag, accA, nb * 64 * KP, accB, k0 + 32 + col, scaleB);
      else tile_step(tag, accA, nb * 64 * KP, accB, k0 + 32 + col, scaleB);
      if (KDT == MISA_FP8_E4M3) scaleA = kscl[nb][col];
      if (FILTER) filter_step(tag, accB, (nb * 64 + 32) * KP, accA, k0 + kKT + col, scaleA);
      else tile_step(tag, accB, (nb * 64 + 32) * KP, accA, k0 + kKT + col, scaleA);
      if (KDT == MISA_FP8_E4M3) scaleB = kscl[nb][32 + col];
      MISA_TILE_STORE(nb ^ 1);
      __syncthreads();
    };
    // iteration j finishes columns of the tiles j and j + 1: unmasked when both are
    for (int j = 0; j < n_plain - 1; ++j) body(Yes{}, j);
    for (int j = max(n_plain - 1, 0); j < n_tiles - 1; ++j) body(No{}, j);
    if (FILTER) drain_pending();   // the last column tile is finished at once, after the pending one
    const int k_last = k_begin + (n_tiles - 1) * kKT + 32 + col;
    if (n_plain == n_tiles) epilogue(Yes{}, accB, k_last, scaleB);
    else epilogue(No{}, accB, k_last, scaleB);
  }
  if (FILTER) {
    // fills of this key range's segments (zero when no key of the range is visible): lanes 0
    // and 32 write those of the lower and the upper half-wave's queries
#pragma unroll
    for (int j = 0; j < NQL; ++j) {
      const int qi = wave * QW + (HS == 8 ? (j >> 1) * 4 + hf * 2 + (j & 1) : (HS == 16 ? j * 2 + hf : hf));
      if (col == 0 && q_base + qi < p.n_q)
        aux.seg_count[((size_t)seq * p.n_q + q_base + qi) * aux.ranges + blockIdx.x] = hf ? cnt_up[j] : cnt[j] - cnt_up[j];
    }
  }
#undef MISA_TILE_LOAD
#undef MISA_TILE_STORE
  if (MODE != kTileStore) return;
  // keys of this range that no query of the tile can see
  const int done = k_begin < k_stop ? k_begin + (k_stop - k_begin + kKT - 1) / kKT * kKT : k_begin;
#pragma unroll
  for (int j = 0; j < NQL; ++j) {
    if (qn[j] < 0) continue;
    for (int key = done + col; key < k_end; key += 32) s_tile[qoff[j] + (uint32_t)key] = -INFINITY;
  }
}

// Two wavefronts per SIMD (at most 256 vector registers) except with four row tiles, which
// need the whole register file.
template <int KDT, int HS, int MODE, bool PAGED, bool Q8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TileGeom<HS, Q8 && MODE == kTileStore>::RT == 4 ? 1 : 2, TileGeom<HS, Q8 && MODE == kTileStore>::RT == 4 ? 1 : 2)))
void score_tile_kernel(
    Prob p, int keys_per_wg, const uint16_t* __restrict__ Q, const float* __restrict__ W,
    const int* __restrict__ heads, const void* __restrict__ K, const float* __restrict__ kscale,
    float* __restrict__ S, TileAux aux) {
  score_tile_body<KDT, HS, MODE, PAGED, Q8>(p, keys_per_wg, Q, W, heads, K, kscale, S, aux, blockIdx.y);
}

// Store mode for the flagged query tiles only (aux.run).  Normally none is
// flagged, so the grid is kept small: blockIdx.y strides over the query tiles.
template <int KDT, int HS, bool PAGED, bool Q8>
__global__ __launch_bounds__(256) void score_tile_repair_kernel(
    Prob p, int keys_per_wg, int q_tiles, const uint16_t* __restrict__ Q,
    const float* __restrict__ W, const int* __restrict__ heads, const void* __restrict__ K,
    const float* __restrict__ kscale, float* __restrict__ S, TileAux aux) {
  for (int qt = blockIdx.y; qt < q_tiles; qt += gridDim.y) {
    if (!aux.run[blockIdx.z * q_tiles + qt]) continue;
    score_tile_body<KDT, HS, kTileStore, PAGED, Q8>(p, keys_per_wg, Q, W, heads, K, kscale, S, aux, qt);
    __syncthreads();
  }
}

// ------------------------------------------------------------------ candidate re-scoring
// score_gather_kernel (bf16 queries, bf16 or fp8 keys, candidate lists): the
// fine stage of MISA-dagger scores k' gathered keys of one query with ALL heads
// (Eq. dsa_score on the candidate set).  The query's H head rows are the
// stationary operand (RT 32-row tiles in registers); each wavefront gathers 32
// candidate keys per step straight from the (cache-resident) key cache into
// MFMA fragments - a lane reads one contiguous half row - and the head sum is
// in-lane over its accumulator registers plus one exchange between half-waves.
// Candidates per workgroup: at most kGatherChunk.  The set-up of a workgroup (head rows, gates,
// candidate indices) costs about a fifth of the kernel with 2048 candidates each, so many-query
// problems take 4096 (0.37 ms against 0.39 ms on the 2048 x 8192 re-rank); few-query problems
// take shorter pieces to put more workgroups on the chip.
// FUSED (the whole re-rank of a query in one workgroup, Eq. misa_final_topk): the workgroup takes
// all k' <= 8192 candidates, the scores replace the candidate indices in LDS as they are
// produced (a slot's index has been consumed by then) and the row's top-k is taken from there by
// small_row_topk - no dense score matrix, no second launch.
constexpr int kGatherChunk = 4096;

template <int KDT, int RT, bool Q8, bool FUSED>
__global__ __launch_bounds__(256) void score_gather_kernel(
    Prob p, const uint16_t* __restrict__ Q, const float* __restrict__ W,
    const void* __restrict__ K, const float* __restrict__ kscale, const int* __restrict__ cand,
    int k_cand, int chunk, float* __restrict__ out, int k, int* __restrict__ idx,
    float* __restrict__ val) {
  constexpr int ROW_BYTES = KDT == MISA_BF16 ? 256 : 128;
  constexpr int NLD = KDT == MISA_BF16 ? 8 : 4;  // 16-byte loads per lane and key (half a row)
  const int t = blockIdx.y, seq = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hf = lane >> 5;
  const int n = visible(p, seq, t);
  const size_t qrow = (size_t)seq * p.n_q + t;
  const int c_begin = blockIdx.x * chunk;            // chunk: a multiple of 128, at most kGatherChunk
  const int c_end = min(c_begin + chunk, k_cand);
  const int* crow = cand + qrow * k_cand;
  float* orow = out + qrow * k_cand;

  // The candidate indices of this workgroup go through LDS, so that reading them
  // in the loop does not wait on the key loads in flight.
  __shared__ int s_cand[FUSED ? kSmallTopkMax : kGatherChunk];
  for (int i = threadIdx.x; i < chunk; i += 256) s_cand[i] = c_begin + i < c_end ? crow[c_begin + i] : -1;

  // Row m of tile rt is head rt*32 + m; half-wave hf holds components 64 hf .. 64 hf + 63,
  // k-step ks the eight from 64 hf + 8 ks (the key fragments use the same mapping).
  // Q8 (fp8 query codes and fp8 keys, fp8 matrix instruction): k-step ks of 64 components,
  // half-wave hf the 32 from 64 ks + 32 hf.
  static_assert(!Q8 || KDT == MISA_FP8_E4M3, "fp8 queries contract with fp8 keys only");
  Frag a[RT][Q8 ? 1 : 8];
  Frag8 a8[RT][Q8 ? 2 : 1];
  __shared__ float s_gate[2][RT * 16];   // [half-wave][accumulator register]: gates of the rows a lane holds
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int head = rt * 32 + col;
    if (Q8) {
      const uint8_t* src = reinterpret_cast<const uint8_t*>(Q) + (qrow * p.H + min(head, p.H - 1)) * kD + 32 * hf;
#pragma unroll
      for (int ks = 0; ks < (Q8 ? 2 : 0); ++ks)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const uint4 v = *reinterpret_cast<const uint4*>(src + 64 * ks + 16 * u);
          a8[rt][ks].u[u] = head < p.H ? v : make_uint4(0, 0, 0, 0);
        }
    } else {
      const uint16_t* src = Q + (qrow * p.H + min(head, p.H - 1)) * kD + 64 * hf;
#pragma unroll
      for (int ks = 0; ks < (Q8 ? 0 : 8); ++ks) {
        const uint4 v = *reinterpret_cast<const uint4*>(src + 8 * ks);
        a[rt][ks].u = head < p.H ? v : make_uint4(0, 0, 0, 0);
      }
    }
  }
  if (threadIdx.x < 2 * RT * 16) {
    const int h2 = threadIdx.x / (RT * 16), e = threadIdx.x % (RT * 16), rt = e / 16, r = e % 16;
    const int hd = rt * 32 + 8 * (r >> 2) + 4 * h2 + (r & 3);
    s_gate[h2][e] = hd < p.H ? W[qrow * p.H + hd] : 0.f;
  }

  // Loads are unconditional and branch-free (slot and row clamped), so the number
  // of loads in flight is the same on every path and waits stay exact.
  struct Raw { uint4 v[NLD]; float scale; int s; };
  auto issue = [&](Raw& r, int c0) {
    const int slot = c0 + col;
    int s = s_cand[min(slot - c_begin, chunk - 1)];
    if (slot >= c_end || s >= n) s = -1;
    r.s = s;
    const int row = max(s, 0);
    const size_t kslot = key_slot(p, seq, row);
    const uint4* src = reinterpret_cast<const uint4*>(static_cast<const char*>(K) + kslot * ROW_BYTES + hf * (Q8 ? 32 : ROW_BYTES / 2));
#pragma unroll
    for (int i = 0; i < NLD; ++i) r.v[i] = src[Q8 ? 4 * (i >> 1) + (i & 1) : i];   // Q8: chunks 0, 1 and 4, 5 from 32 hf
    r.scale = 1.f;
    if (KDT == MISA_FP8_E4M3) r.scale = kscale[kslot];
  };
  auto finish = [&](const Raw& r, int c0) {
    if (c0 >= c_end) return;
    f32x16 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[rt][q] = 0.f;
    if constexpr (Q8) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        Frag8 b;
        b.u[0] = r.v[(2 * ks) % NLD];
        b.u[1] = r.v[(2 * ks + 1) % NLD];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          acc[rt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8[rt][ks].v, b.v, acc[rt], 0, 0, 0, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        Frag b;
        if (KDT == MISA_BF16) {
          b.u = r.v[ks % NLD];
        } else {
          const uint4 w = r.v[(ks >> 1) % NLD];
          fp8x4_to_bf16x4((ks & 1) ? w.z : w.x, b.w[0], b.w[1]);
          fp8x4_to_bf16x4((ks & 1) ? w.w : w.y, b.w[2], b.w[3]);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, b.v, acc[rt], 0, 0, 0);
      }
    }
    float sum = 0.f;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int q = 0; q < 16; ++q) sum = fmaf(s_gate[hf][rt * 16 + q], relu(acc[rt][q]), sum);
    sum += __shfl_xor(sum, 32);
    const int slot = c0 + col;
    if (hf == 0 && slot < c_end) {
      const float score = r.s >= 0 ? sum * r.scale : -INFINITY;
      if (FUSED) s_cand[slot] = __float_as_int(score);   // (c_begin = 0; this slot's index was read at issue)
      else orow[slot] = score;
    }
  };

  // kDepth register buffers: the loads of a step are issued kDepth - 1 steps before they are
  // used (a step of one wavefront is far shorter than the latency of a gathered row).
  constexpr int kDepth = 2;
  __builtin_amdgcn_s_waitcnt(0);  // the query operand has landed; in-loop waits concern only loop loads
  __syncthreads();                // candidate indices are in LDS
  auto stream_candidates = [&]() {
    Raw buf[kDepth];
    int c0 = c_begin + wave * 32;
#pragma unroll
    for (int d = 0; d < kDepth - 1; ++d) issue(buf[d], c0 + 128 * d);
    while (true) {
#pragma unroll
      for (int d = 0; d < kDepth; ++d) {
        issue(buf[(d + kDepth - 1) % kDepth], c0 + 128 * (kDepth - 1));
        __builtin_amdgcn_sched_barrier(0);
        finish(buf[d], c0);
        c0 += 128;
        if (c0 >= c_end) return;
      }
    }
  };
  stream_candidates();
  if constexpr (FUSED) {
    __shared__ SmallTopkLds topk_lds;
    __syncthreads();                // all scores of the row are in LDS
    small_row_topk(s_cand, k_cand, k, crow, idx + qrow * k, val ? val + qrow * k : nullptr, topk_lds);
  }
}

// score_cand_kernel (bf16 queries, bf16 or fp8 keys, candidate lists): the same re-scoring with
// the operand layout of the decode kernel.  A wavefront takes 64 candidates per step as four
// 16-key tiles on v_mfma_f32_16x16x32_bf16; the four lanes that share a key column read 64
// contiguous bytes of its row per load instruction, so an instruction touches 16 cache lines
// instead of the 32 of one-lane-per-half-row (the gather is bound by the number of lines its
// load instructions touch, not by bytes).  All H head rows are the stationary operand (NT 16-row
// tiles); the head sum is in-lane over the accumulator registers plus the two exchanges that
// leave lane i with candidate i of the group.  Chunks, the two-buffer pipeline and the FUSED
// tail are those of score_gather_kernel.  Used for bf16 keys (256-byte rows: 0.54 ms against
// 0.59 ms for the re-rank of 2048 x 8192 candidates); with fp8 keys the 32-row-tile kernel, whose
// half rows are 64 contiguous bytes as well, is 2-6 % faster (three wavefronts per SIMD instead
// of two) and stays in use.
template <int KDT, int NT, bool FUSED>
__global__ __launch_bounds__(256) void score_cand_kernel(
    Prob p, const uint16_t* __restrict__ Q, const float* __restrict__ W,
    const void* __restrict__ K, const float* __restrict__ kscale, const int* __restrict__ cand,
    int k_cand, int chunk, float* __restrict__ out, int k, int* __restrict__ idx,
    float* __restrict__ val) {
  constexpr int ROW_BYTES = KDT == MISA_BF16 ? 256 : 128;
  constexpr int NLD = KDT == MISA_BF16 ? 4 : 2;  // 16-byte loads per lane and 16-key tile
  const int t = blockIdx.y, seq = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int n = visible(p, seq, t);
  const size_t qrow = (size_t)seq * p.n_q + t;
  const int c_begin = blockIdx.x * chunk;            // chunk: a multiple of 256
  const int c_end = min(c_begin + chunk, k_cand);
  const int* crow = cand + qrow * k_cand;
  float* orow = out + qrow * k_cand;

  __shared__ int s_cand[FUSED ? kSmallTopkMax : kGatherChunk];
  for (int i = threadIdx.x; i < chunk; i += 256) s_cand[i] = c_begin + i < c_end ? crow[c_begin + i] : -1;

  // Head rows and gates; component mapping of the k-steps as in score_stream_kernel.
  Frag a[NT][4];
  float wv[NT][4];
#pragma unroll
  for (int T = 0; T < NT; ++T) {
    const int head = T * 16 + c;
    const uint16_t* src = Q + (qrow * p.H + min(head, p.H - 1)) * kD;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int comp = KDT == MISA_BF16 ? 8 * (4 * i + g) : 16 * (4 * (i >> 1) + g) + 8 * (i & 1);
      const uint4 v = *reinterpret_cast<const uint4*>(src + comp);
      a[T][i].u = head < p.H ? v : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int hd = T * 16 + 4 * g + j;   // the accumulator of lane (c, g) holds head rows 4 g + j
      wv[T][j] = hd < p.H ? W[qrow * p.H + min(hd, p.H - 1)] : 0.f;
    }
  }

  struct Raw { uint4 v[4][NLD]; float scale; int s; };
  // candidate of list slot `slot` (-1: none, hole, or not visible to the query)
  auto candidate = [&](int slot) {
    int s = s_cand[min(slot - c_begin, chunk - 1)];
    if (slot >= c_end || s >= n) s = -1;
    return s;
  };
  // Loads are unconditional and branch-free (absent candidates read key 0), so the number of
  // loads in flight is the same on every path and waits stay exact.
  auto issue = [&](Raw& r, int c0) {
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      const size_t kslot = key_slot(p, seq, max(candidate(c0 + tt * 16 + c), 0));
      const uint4* src = reinterpret_cast<const uint4*>(static_cast<const char*>(K) + kslot * ROW_BYTES) + g;
#pragma unroll
      for (int i = 0; i < NLD; ++i) r.v[tt][i] = src[4 * i];
    }
    r.s = candidate(c0 + lane);            // the candidate this lane finally owns
    r.scale = 1.f;
    if (KDT == MISA_FP8_E4M3) r.scale = kscale[key_slot(p, seq, max(r.s, 0))];
  };
  auto finish = [&](const Raw& r, int c0) {
    if (c0 >= c_end) return;
    float part[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      Frag b[4];
      if (KDT == MISA_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i].u = r.v[tt][i % NLD];
      } else {
        const uint4 lo = r.v[tt][0], hi = r.v[tt][NLD - 1];
        const uint32_t w8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          fp8x4_to_bf16x4(w8[2 * i], b[i].w[0], b[i].w[1]);
          fp8x4_to_bf16x4(w8[2 * i + 1], b[i].w[2], b[i].w[3]);
        }
      }
      float sum = 0.f;
#pragma unroll
      for (int T = 0; T < NT; ++T) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[T][i].v, b[i].v, acc, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) sum = fmaf(wv[T][j], relu(acc[j]), sum);
      }
      part[tt] = sum;
    }
    // sum over the four lane groups so that group g ends with tile g: lane i owns slot c0 + i
    const bool up2 = (g & 2) != 0, up1 = (g & 1) != 0;
    const float r0 = __shfl_xor(up2 ? part[0] : part[2], 32);
    const float r1 = __shfl_xor(up2 ? part[1] : part[3], 32);
    const float k0 = (up2 ? part[2] : part[0]) + r0;
    const float k1 = (up2 ? part[3] : part[1]) + r1;
    const float r2 = __shfl_xor(up1 ? k0 : k1, 16);
    const float fin = (up1 ? k1 : k0) + r2;
    const int slot = c0 + lane;
    if (slot < c_end) {
      const float score = r.s >= 0 ? fin * r.scale : -INFINITY;
      if (FUSED) s_cand[slot] = __float_as_int(score);   // (c_begin = 0; this slot's index was read at issue)
      else orow[slot] = score;
    }
  };

  __builtin_amdgcn_s_waitcnt(0);  // the query operand has landed; in-loop waits concern only loop loads
  __syncthreads();                // candidate indices are in LDS
  auto stream_candidates = [&]() {
    Raw buf[2];
    int c0 = c_begin + wave * 64;
    issue(buf[0], c0);
    while (true) {
      issue(buf[1], c0 + 256);
      __builtin_amdgcn_sched_barrier(0);
      finish(buf[0], c0);
      c0 += 256;
      if (c0 >= c_end) return;
      issue(buf[0], c0 + 256);
      __builtin_amdgcn_sched_barrier(0);
      finish(buf[1], c0);
      c0 += 256;
      if (c0 >= c_end) return;
    }
  };
  stream_candidates();
  if constexpr (FUSED) {
    __shared__ SmallTopkLds topk_lds;
    __syncthreads();                // all scores of the row are in LDS
    small_row_topk(s_cand, k_cand, k, crow, idx + qrow * k, val ? val + qrow * k : nullptr, topk_lds);
  }
}

template <int KDT, int QDT>
static hipError_t launch_generic(const Prob& p, const void* Q, const float* W, const int* heads,
                                 const void* K, const float* kscale, const int* cand, int k_cand,
                                 float* out, hipStream_t st) {
  const int row_len = cand ? k_cand : p.L;
  const dim3 grid((row_len + 255) / 256, p.n_q, p.n_seq);
  score_generic_kernel<KDT, QDT><<<grid, 256, 0, st>>>(p, Q, W, heads, K, kscale, cand, k_cand, out);
  return hipGetLastError();
}

template <int KDT>
static hipError_t launch_stream(const Prob& p, const void* Q, const float* W, const int* heads,
                                const void* K, const float* kscale, float* S, hipStream_t st) {
  const int hc = heads ? p.h : p.H;
  const int nt = (hc + 15) / 16;
  // bf16 keys: 4 pipeline steps of one 64-key group per wavefront, 1024 keys (256 KB) per
  // workgroup.  fp8 keys with up to 16 heads: one step, 256 keys (32 KB) per workgroup -
  // every wavefront loads its 8 KB, computes and retires, and latency is hidden by the
  // other resident wavefronts alone (4 per SIMD).  Measured best of 256 .. 4096 keys per
  // workgroup on MI355X for each type (fp8: 96 us against 102 us with 1024 keys; bf16: 94 us
  // against 97 us with 256 keys); with more head tiles fewer wavefronts fit a SIMD and the
  // pipelined form is faster again (32 heads, fp8: 105 us against 134 us).
  const uint16_t* q = static_cast<const uint16_t*>(Q);
#define GO(NT, STEPS)                                                                             \
  do {                                                                                            \
    constexpr int KPW = 256 * (STEPS);                                                            \
    const dim3 grid((p.L + KPW - 1) / KPW, p.n_q, p.n_seq);                                       \
    if (p.page_table)                                                                             \
      score_stream_kernel<KDT, NT, STEPS, 1, true><<<grid, 256, 0, st>>>(p, q, W, heads, K, kscale, S);  \
    else                                                                                          \
      score_stream_kernel<KDT, NT, STEPS, 1, false><<<grid, 256, 0, st>>>(p, q, W, heads, K, kscale, S); \
  } while (0)
  switch (nt) {
    case 1:
      if (KDT == MISA_FP8_E4M3) GO(1, 1);
      else GO(1, 4);
      break;
    case 2: GO(2, 4); break;
    case 3: GO(3, 4); break;
    default: GO(4, 4); break;
  }
#undef GO
  return hipGetLastError();
}

// q8: the store-mode geometry of fp8 query codes (the wider query tile)
int tile_queries_per_wg(const Prob& p, bool routed, bool q8) {
  const int hc = routed ? p.h : p.H;
  return hc <= 8 ? (q8 ? 64 : 32) : (hc <= 16 ? 16 : 8);
}

int tile_key_ranges(const Prob& p, bool routed, bool q8, int mode, int* keys_per_wg) {
  const int qwg = tile_queries_per_wg(p, routed, q8 && mode == kTileStore);
  const int q_tiles = (p.n_q + qwg - 1) / qwg;
  const int lt = mode == kTileSample ? p.L / kSampleStride : p.L;  // keys in tile space
  // Key ranges: a multiple of 8 (one set per XCD), enough workgroups to fill
  // the chip several times, at least 1024 keys each.
  int splits = 8;
  while (splits < 64 && (long long)splits * q_tiles * p.n_seq < 2048 && lt / (splits * 2) >= 1024) splits *= 2;
  *keys_per_wg = ((lt + splits - 1) / splits + kKT - 1) / kKT * kKT;
  return (lt + *keys_per_wg - 1) / *keys_per_wg;
}

template <int KDT, int MODE, bool Q8>
static hipError_t launch_tile(const Prob& p, const void* Q, const float* W, const int* heads,
                              const void* K, const float* kscale, float* S, const TileAux& aux,
                              hipStream_t st) {
  const int hc = heads ? p.h : p.H;
  const int hs = hc <= 8 ? 8 : (hc <= 16 ? 16 : (hc <= 32 ? 32 : 64));
  const int qwg = tile_queries_per_wg(p, heads != nullptr, Q8 && MODE == kTileStore);
  const int q_tiles = (p.n_q + qwg - 1) / qwg;
  int keys_per_wg = 0;
  const int ranges = tile_key_ranges(p, heads != nullptr, Q8, MODE, &keys_per_wg);
  dim3 grid(ranges, q_tiles, p.n_seq);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if (MODE == kTileStore && aux.run) {
    // about one resident set of workgroups, each striding over the query tiles
    grid.y = (unsigned)std::max(1, std::min(q_tiles, (int)(512 / ((long long)grid.x * p.n_seq))));
#define GO(HS)                                                                                                      \
  if (p.page_table)                                                                                                 \
    score_tile_repair_kernel<KDT, HS, true, Q8><<<grid, 256, 0, st>>>(p, keys_per_wg, q_tiles, q, W, heads, K, kscale, S, aux); \
  else                                                                                                              \
    score_tile_repair_kernel<KDT, HS, false, Q8><<<grid, 256, 0, st>>>(p, keys_per_wg, q_tiles, q, W, heads, K, kscale, S, aux)
    switch (hs) {
      case 8: GO(8); break;
      case 16: GO(16); break;
      case 32: GO(32); break;
      default: GO(64); break;
    }
#undef GO
    return hipGetLastError();
  }
#define GO(HS)                                                                                               \
  if (p.page_table)                                                                                          \
    score_tile_kernel<KDT, HS, MODE, true, Q8><<<grid, 256, 0, st>>>(p, keys_per_wg, q, W, heads, K, kscale, S, aux); \
  else                                                                                                       \
    score_tile_kernel<KDT, HS, MODE, false, Q8><<<grid, 256, 0, st>>>(p, keys_per_wg, q, W, heads, K, kscale, S, aux)
  switch (hs) {
    case 8: GO(8); break;
    case 16: GO(16); break;
    case 32: GO(32); break;
    default: GO(64); break;
  }
#undef GO
  return hipGetLastError();
}

// The matrix-core tile kernel takes bf16 queries with bf16 or fp8 keys, and fp8 query codes with
// fp8 keys (both operands then stay fp8).
bool tile_path(const Prob& p, int k_dtype, int q_dtype) {
  const bool types = (q_dtype == MISA_BF16 && k_dtype != MISA_F32) ||
                     (q_dtype == MISA_FP8_E4M3 && k_dtype == MISA_FP8_E4M3);
  return types && p.n_q >= kTileMinQueries;
}

hipError_t launch_tile_mode(const Prob& p, int k_dtype, int q_dtype, int mode, const TileAux& aux,
                            const void* Q, const float* W, const int* heads, const void* K,
                            const float* kscale, float* S, hipStream_t st) {
#define GO(KD, Q8)                                                                                      \
  switch (mode) {                                                                                       \
    case kTileSample: return launch_tile<KD, kTileSample, Q8>(p, Q, W, heads, K, kscale, S, aux, st);   \
    case kTileFilter: return launch_tile<KD, kTileFilter, Q8>(p, Q, W, heads, K, kscale, S, aux, st);   \
    default: return launch_tile<KD, kTileStore, Q8>(p, Q, W, heads, K, kscale, S, aux, st);             \
  }
  if (q_dtype == MISA_FP8_E4M3) GO(MISA_FP8_E4M3, true)
  if (k_dtype == MISA_BF16) GO(MISA_BF16, false)
  GO(MISA_FP8_E4M3, false)
#undef GO
}

template <int KDT, bool Q8>
static hipError_t launch_gather(const Prob& p, const void* Q, const float* W, const void* K,
                                const float* kscale, const int* cand, int k_cand, float* out,
                                hipStream_t st) {
  // pieces of 512 .. kGatherChunk candidates (a step of the four wavefronts covers 128 or 256): halved
  // while fewer than 1024 workgroups would result
  int chunk = kGatherChunk;
  const long long rows = (long long)p.n_q * p.n_seq;
  while (chunk > 512 && rows * ((k_cand + chunk - 1) / chunk) < 1024) chunk /= 2;
  const dim3 grid((k_cand + chunk - 1) / chunk, p.n_q, p.n_seq);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if constexpr (KDT == MISA_BF16) {   // 256-byte rows: 16-row head tiles, four lanes per key row (see score_cand_kernel)
#define GO(NT) score_cand_kernel<KDT, NT, false><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, out, 0, nullptr, nullptr)
    switch ((p.H + 15) / 16) {
      case 1: GO(1); break;
      case 2: GO(2); break;
      case 3: GO(3); break;
      default: GO(4); break;
    }
#undef GO
  } else if (p.H <= 32) {
    score_gather_kernel<KDT, 1, Q8, false><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, out, 0, nullptr, nullptr);
  } else {
    score_gather_kernel<KDT, 2, Q8, false><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, out, 0, nullptr, nullptr);
  }
  return hipGetLastError();
}

// Re-rank with the top-k inside the gather kernel: for many queries with short candidate lists
// (one workgroup per query fills the chip, the list fits LDS) and the types the gather kernel
// takes.
bool rerank_fused_path(const Prob& p, int k_dtype, int q_dtype, int k_cand) {
  const bool types = (q_dtype == MISA_BF16 && k_dtype != MISA_F32) ||
                     (q_dtype == MISA_FP8_E4M3 && k_dtype == MISA_FP8_E4M3);
  return types && k_cand <= kSmallTopkMax && (long long)p.n_q * p.n_seq >= kRerankFusedMinRows;
}

template <int KDT, bool Q8>
static hipError_t launch_gather_topk(const Prob& p, const void* Q, const float* W, const void* K,
                                     const float* kscale, const int* cand, int k_cand, int k, int* idx,
                                     float* val, hipStream_t st) {
  const int chunk = (k_cand + 255) / 256 * 256;
  const dim3 grid(1, p.n_q, p.n_seq);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if constexpr (KDT == MISA_BF16) {
#define GO(NT) score_cand_kernel<KDT, NT, true><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, nullptr, k, idx, val)
    switch ((p.H + 15) / 16) {
      case 1: GO(1); break;
      case 2: GO(2); break;
      case 3: GO(3); break;
      default: GO(4); break;
    }
#undef GO
  } else if (p.H <= 32) {
    score_gather_kernel<KDT, 1, Q8, true><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, nullptr, k, idx, val);
  } else {
    score_gather_kernel<KDT, 2, Q8, true><<<grid, 256, 0, st>>>(p, q, W, K, kscale, cand, k_cand, chunk, nullptr, k, idx, val);
  }
  return hipGetLastError();
}

hipError_t launch_rerank_fused(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                               const void* K, const float* kscale, const int* cand, int k_cand, int k,
                               int* idx, float* val, hipStream_t st) {
  if (!rerank_fused_path(p, k_dtype, q_dtype, k_cand)) return hipErrorInvalidValue;
  if (q_dtype == MISA_FP8_E4M3) return launch_gather_topk<MISA_FP8_E4M3, true>(p, Q, W, K, kscale, cand, k_cand, k, idx, val, st);
  if (k_dtype == MISA_BF16) return launch_gather_topk<MISA_BF16, false>(p, Q, W, K, kscale, cand, k_cand, k, idx, val, st);
  return launch_gather_topk<MISA_FP8_E4M3, false>(p, Q, W, K, kscale, cand, k_cand, k, idx, val, st);
}

hipError_t launch_score(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const int* heads, const void* K, const float* kscale, const int* cand,
                        int k_cand, float* out, hipStream_t st) {
  if (cand && !heads && q_dtype == MISA_FP8_E4M3 && k_dtype == MISA_FP8_E4M3)
    return launch_gather<MISA_FP8_E4M3, true>(p, Q, W, K, kscale, cand, k_cand, out, st);
  if (cand && !heads && q_dtype == MISA_BF16 && k_dtype != MISA_F32) {
    if (k_dtype == MISA_BF16) return launch_gather<MISA_BF16, false>(p, Q, W, K, kscale, cand, k_cand, out, st);
    return launch_gather<MISA_FP8_E4M3, false>(p, Q, W, K, kscale, cand, k_cand, out, st);
  }
  if (!cand && tile_path(p, k_dtype, q_dtype))
    return launch_tile_mode(p, k_dtype, q_dtype, kTileStore, TileAux{}, Q, W, heads, K, kscale, out, st);
  if (q_dtype == MISA_FP8_E4M3) return hipErrorInvalidValue;   // fp8 codes reach only the tile kernel
  const bool mfma_ok = !cand && q_dtype == MISA_BF16 && k_dtype != MISA_F32;
  if (mfma_ok) {
    if (k_dtype == MISA_BF16) return launch_stream<MISA_BF16>(p, Q, W, heads, K, kscale, out, st);
    return launch_stream<MISA_FP8_E4M3>(p, Q, W, heads, K, kscale, out, st);
  }
#define GEN(KD, QD) return launch_generic<KD, QD>(p, Q, W, heads, K, kscale, cand, k_cand, out, st)
  if (q_dtype == MISA_F32) {
    if (k_dtype == MISA_F32) GEN(MISA_F32, MISA_F32);
    if (k_dtype == MISA_BF16) GEN(MISA_BF16, MISA_F32);
    GEN(MISA_FP8_E4M3, MISA_F32);
  }
  if (k_dtype == MISA_F32) GEN(MISA_F32, MISA_BF16);
  if (k_dtype == MISA_BF16) GEN(MISA_BF16, MISA_BF16);
  GEN(MISA_FP8_E4M3, MISA_BF16);
#undef GEN
}

}  // namespace misa
