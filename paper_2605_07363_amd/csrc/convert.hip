// fp8 (e4m3) query codes -> bf16.  Every e4m3 value is a bf16 value, so the widened queries
// give exactly the products the codes would; the scoring kernels then run on bf16 operands.
#include "kernels.h"

namespace misa {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

// 16 codes per thread and round: one 16-byte load, two 16-byte stores.
__global__ __launch_bounds__(256) void widen_queries_kernel(const uint4* __restrict__ q8,
                                                            uint4* __restrict__ q16, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 v = q8[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      union { bf16x2_t b; uint32_t u; } lo, hi;
      lo.b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[j], 1.0f, false);  // codes 0, 1
      hi.b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[j], 1.0f, true);   // codes 2, 3
      o[2 * j] = lo.u;
      o[2 * j + 1] = hi.u;
    }
    q16[2 * i] = make_uint4(o[0], o[1], o[2], o[3]);
    q16[2 * i + 1] = make_uint4(o[4], o[5], o[6], o[7]);
  }
}

hipError_t launch_widen_queries(const void* q8, void* q16, size_t n_elems, hipStream_t st) {
  const size_t n16 = n_elems / 16;  // rows hold 128 codes
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 4096);
  widen_queries_kernel<<<grid, 256, 0, st>>>(static_cast<const uint4*>(q8), static_cast<uint4*>(q16), n16);
  return hipGetLastError();
}

}  // namespace misa
