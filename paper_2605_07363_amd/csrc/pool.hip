// Stage 1: block mean pooling of the indexer keys (Eq. pool).
//
// One workgroup per (pooled block, sequence).  The block's rows are streamed
// with 16-byte loads, a row being covered by 128/N consecutive lanes, so every
// wavefront load instruction reads whole contiguous rows.  Each thread sums a
// strided subset of rows in fp32; the subsets are combined through LDS in a
// fixed order, so the result is deterministic.
#include "kernels.h"

namespace misa {

template <int DT>
__global__ __launch_bounds__(256) void pool_kernel(Prob p, const void* __restrict__ K,
                                                   const float* __restrict__ kscale,
                                                   float* __restrict__ Kp) {
  using V = Vec16<DT>;
  constexpr int N = V::N;             // values per 16-byte load
  constexpr int TPR = kD / N;         // threads per key row
  constexpr int RPP = 256 / TPR;      // rows per pass of the workgroup
  __shared__ float red[RPP][kD];

  const int b = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int len = seq_length(p, seq);
  const long long lo = (long long)b * p.B;
  const long long hi = min(lo + (long long)p.B, (long long)len);
  const int c = tid % TPR, r = tid / TPR;

  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;

  const char* base = static_cast<const char*>(K) + (size_t)seq * p.L * V::ROW_BYTES;
  for (long long row = lo + r; row < hi; row += RPP) {
    float v[N];
    V::load(base + (size_t)row * V::ROW_BYTES + c * 16, v);
    float s = 1.f;
    if (DT == MISA_FP8_E4M3) s = kscale[(size_t)seq * p.L + row];
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = fmaf(v[e], s, acc[e]);
  }
#pragma unroll
  for (int e = 0; e < N; ++e) red[r][c * N + e] = acc[e];
  __syncthreads();
  if (tid < kD) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RPP; ++i) s += red[i][tid];
    const long long cnt = hi - lo;
    Kp[((size_t)seq * p.M + b) * kD + tid] = cnt > 0 ? s / (float)cnt : 0.f;
  }
}

hipError_t launch_pool(const Prob& p, int k_dtype, const void* K, const float* kscale, float* Kp,
                       hipStream_t st) {
  const dim3 grid(p.M, p.n_seq), block(256);
  switch (k_dtype) {
    case MISA_F32: pool_kernel<MISA_F32><<<grid, block, 0, st>>>(p, K, kscale, Kp); break;
    case MISA_BF16: pool_kernel<MISA_BF16><<<grid, block, 0, st>>>(p, K, kscale, Kp); break;
    default: pool_kernel<MISA_FP8_E4M3><<<grid, block, 0, st>>>(p, K, kscale, Kp); break;
  }
  return hipGetLastError();
}

}  // namespace misa
