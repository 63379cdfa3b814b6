// Two probes of what the machine delivers, for the roofline report: a pure read of a
// device buffer and a loop of dependent-free bf16 matrix instructions.  Neither is part of
// the indexer; bench.py runs them next to the indexer kernels so that every achieved rate
// can be quoted against the measured as well as the published peak.
#include "kernels.h"

namespace misa {

// Every wavefront reads 8 KB (eight 16-byte loads per lane, all issued before the first is
// used) and retires; a workgroup of four wavefronts covers 32 KB.
constexpr int kProbeWaveBytes = 8192;

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ buf,
                                                         size_t n_groups,
                                                         uint32_t* __restrict__ sink) {
  const size_t group = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (group >= n_groups) return;
  const uint4* src = buf + group * (kProbeWaveBytes / 16) + (threadIdx.x & 63);
  uint4 v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = src[i * 64];
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  if (acc == 0x9E3779B9u) sink[threadIdx.x] = acc;   // keeps the loads alive; practically never taken
}

// Every wavefront issues iters x 4 independent 32x32x16 bf16 matrix instructions on
// register operands (four accumulators, so consecutive instructions never wait for each
// other).  No memory traffic but the final store.
constexpr int kProbeMfmaPerIter = 4;

// operands == nullptr: constant operands (1.0 x {0.5, 1.0}).  Otherwise lane l of every wavefront
// takes its two fragments from operands[l] and operands[64 + l] (16 bytes each): the rate the
// chip sustains depends on the operand values (its clock drops as more bits toggle per product).
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, const uint4* __restrict__ operands,
                                                         float* __restrict__ sink) {
  union { bf16x8 v; uint32_t u[4]; uint4 q; } a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a.u[i] = 0x3F803F80u;                                  // bf16 1.0, 1.0
    b.u[i] = (threadIdx.x & 1) ? 0x3F803F80u : 0x3F003F00u;  // 1.0 or 0.5
  }
  if (operands) {
    a.q = operands[threadIdx.x & 63];
    b.q = operands[64 + (threadIdx.x & 63)];
  }
  f32x16 acc[kProbeMfmaPerIter];
#pragma unroll
  for (int j = 0; j < kProbeMfmaPerIter; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProbeMfmaPerIter; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kProbeMfmaPerIter; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_probe_read(const void* buf, size_t bytes, void* sink, hipStream_t st) {
  const size_t n_groups = bytes / kProbeWaveBytes;
  const unsigned grid = (unsigned)((n_groups + 3) / 4);
  probe_read_kernel<<<grid, 256, 0, st>>>(static_cast<const uint4*>(buf), n_groups,
                                          static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

hipError_t launch_probe_mfma(int workgroups, int iters, const void* operands, float* sink, hipStream_t st) {
  probe_mfma_kernel<<<workgroups, 256, 0, st>>>(iters, static_cast<const uint4*>(operands), sink);
  return hipGetLastError();
}

}  // namespace misa
