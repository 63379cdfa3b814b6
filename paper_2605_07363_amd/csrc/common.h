// Shared device helpers for the MISA indexer kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "misa.h"

namespace misa {

constexpr int kD = 128;      // indexer head dimension
constexpr int kMaxH = 64;    // most indexer heads handled
constexpr int kWave = 64;    // CDNA wavefront

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;

// Device-side view of misa_problem (host fills it after validation).
struct Prob {
  int n_seq, L, n_q, H, B, h, M;
  const int* q_pos;
  const int* seq_len;
  const int* page_table;   // nullptr: keys contiguous per sequence
  int page_shift, max_pages;
};

// Row of key s of sequence seq in the key array (contiguous cache or page pool).
template <bool PAGED>
__device__ __forceinline__ size_t key_slot(const Prob& p, int seq, int s) {
  if (!PAGED) return (size_t)seq * p.L + s;
  const int page = p.page_table[(size_t)seq * p.max_pages + (s >> p.page_shift)];
  return ((size_t)page << p.page_shift) + (s & ((1 << p.page_shift) - 1));
}
__device__ __forceinline__ size_t key_slot(const Prob& p, int seq, int s) {
  return p.page_table ? key_slot<true>(p, seq, s) : key_slot<false>(p, seq, s);
}

__device__ __forceinline__ int seq_length(const Prob& p, int seq) {
  int len = p.L;
  if (p.seq_len) len = min(max(p.seq_len[seq], 0), p.L);
  return len;
}

// Number of keys query t of sequence seq may see (its causal prefix length).
__device__ __forceinline__ int visible(const Prob& p, int seq, int t) {
  int len = seq_length(p, seq);
  if (!p.q_pos) return len;
  long long n = (long long)p.q_pos[t] + 1;
  n = n < 0 ? 0 : n;
  return n > len ? len : (int)n;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// 16 bytes of stored values -> floats.  DT: 0 = f32 (4 values), 1 = bf16 (8), 2 = fp8 e4m3 (16).
template <int DT>
struct Vec16;
template <>
struct Vec16<MISA_F32> {
  static constexpr int N = 4;
  static constexpr int ROW_BYTES = kD * 4;
  __device__ static __forceinline__ void load(const void* p, float* out) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
};
template <>
struct Vec16<MISA_BF16> {
  static constexpr int N = 8;
  static constexpr int ROW_BYTES = kD * 2;
  __device__ static __forceinline__ void load(const void* p, float* out) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
};
template <>
struct Vec16<MISA_FP8_E4M3> {
  static constexpr int N = 16;
  static constexpr int ROW_BYTES = kD;
  __device__ static __forceinline__ void load(const void* p, float* out) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // gfx950 decodes OCP E4M3 here (bias 7, max 448).
      const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], false);
      const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], true);
      out[4 * i] = lo[0]; out[4 * i + 1] = lo[1];
      out[4 * i + 2] = hi[0]; out[4 * i + 3] = hi[1];
    }
  }
};

// ReLU as one integer max: non-negative floats have non-negative bit patterns,
// negative ones (and -0.0) are negative integers, so max(bits, 0) is max(x, +0.0)
// without the NaN-quieting instruction an IEEE fmaxf needs.
__device__ __forceinline__ float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

// Order-preserving image of a float: a > b (as floats, -0 == +0) <=> key(a) > key(b).
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0;  // -0.0 ties with +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
constexpr uint32_t kKeyNegInf = 0x007FFFFFu;  // order_key(-inf)

// Inclusive prefix sum inside each row of 16 lanes: four shifted adds (data-parallel-primitive
// moves with zero shifted in).  All lanes of the wavefront must be active.
__device__ __forceinline__ int row16_inclusive_scan(int v) {
  int x = v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);  // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);  // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);  // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);  // row_shr:8
  return x;
}

// Inclusive prefix sum over the 64 lanes of a wavefront, all of them active: the row scans,
// then the totals of the rows before a lane's own are added from lanes 15, 31 and 47.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int x = row16_inclusive_scan(v);
  const int t0 = __builtin_amdgcn_readlane(x, 15);
  const int t1 = __builtin_amdgcn_readlane(x, 31);
  const int t2 = __builtin_amdgcn_readlane(x, 47);
  const int lane = threadIdx.x & 63;
  return x + (lane >= 16 ? t0 : 0) + (lane >= 32 ? t1 : 0) + (lane >= 48 ? t2 : 0);
}

// Given the totals of the block's wavefronts in wave_total[0 .. nw-1] (nw <= 16), returns the
// sum of the totals of the wavefronts before this one and, in *total, the sum of all: the
// first 16 lanes of every wavefront read one total each and scan them.
__device__ __forceinline__ int waves_before(const int* wave_total, int nw, int* total) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int x = row16_inclusive_scan(lane < nw ? wave_total[lane] : 0);
  *total = __builtin_amdgcn_readlane(x, 15);
  return wave > 0 ? __builtin_amdgcn_readlane(x, wave - 1) : 0;
}

// Exclusive prefix sum over a 1-D thread block (blockDim.x a multiple of 64,
// at most 1024).  `scratch` holds 16 ints of LDS.  Also returns the block
// total in *total.  Contains two barriers.
__device__ __forceinline__ int block_exclusive_scan(int v, int* scratch, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int inc = wave_inclusive_scan(v);
  __syncthreads();  // scratch may still be read from a previous call
  if (lane == 63) scratch[wave] = inc;
  __syncthreads();
  return waves_before(scratch, nw, total) + inc - v;
}

}  // namespace misa
