// Stage 1: block mean pooling of the indexer keys (Eq. pool).
//
// One workgroup per (pooled block, sequence) - or, for blocks longer than 2048
// tokens, per 1024-token slice of a block, whose fp32 partial sums go through
// the workspace and are added in a fixed order by a second small kernel, so
// that a few huge blocks (B up to the whole prefix) still fill the chip and
// the result stays deterministic.  The block's rows are streamed
// with 16-byte loads, a row being covered by 128/N consecutive lanes, so every
// wavefront load instruction reads whole contiguous rows.  Each thread sums a
// strided subset of rows in fp32; the subsets are combined through LDS in a
// fixed order, so the result is deterministic.
#include <algorithm>

#include "kernels.h"

namespace misa {

constexpr int kPoolSlice = 1024;    // tokens per slice of a long block
constexpr int kPoolSplitFrom = 2048;  // blocks longer than this are sliced

// slices == 1: Kp receives the block means.  slices > 1: blockIdx.x = block * slices + slice
// and `Kp` is the workspace [n_seq, M, slices, 128] of partial SUMS.
// from_token == nullptr: blockIdx.x / slices is the block.  Otherwise (update after tokens were
// appended) it counts from the block that holds token from_token[seq], and blocks past the
// sequence end are left alone.
template <int DT, bool PAGED>
__global__ __launch_bounds__(256) void pool_kernel(Prob p, int slices, const int* __restrict__ from_token,
                                                   const void* __restrict__ K,
                                                   const float* __restrict__ kscale,
                                                   float* __restrict__ Kp) {
  using V = Vec16<DT>;
  constexpr int N = V::N;             // values per 16-byte load
  constexpr int TPR = kD / N;         // threads per key row
  constexpr int RPP = 256 / TPR;      // rows per pass of the workgroup
  __shared__ float red[RPP][kD];

  const int slice = blockIdx.x % slices, seq = blockIdx.y, tid = threadIdx.x;
  const int len = seq_length(p, seq);
  int b = blockIdx.x / slices;
  if (from_token) {
    b += min(max(from_token[seq], 0), len) / p.B;
    if ((long long)b * p.B >= len) return;
  }
  const long long blo = (long long)b * p.B;
  const long long bhi = min(blo + (long long)p.B, (long long)len);
  const long long lo = slices == 1 ? blo : blo + (long long)slice * kPoolSlice;
  const long long hi = slices == 1 ? bhi : min(lo + kPoolSlice, bhi);
  const int c = tid % TPR, r = tid / TPR;

  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;

  const char* base = static_cast<const char*>(K);
  // four rows per round: their loads (with a page table: their table entries, then their keys)
  // are in flight together; rows past the end are clamped and masked, the order of the additions
  // is that of the rows
  for (long long row0 = lo + r; row0 < hi; row0 += 4 * RPP) {
    size_t slot[4];
    float v[4][N], s[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) slot[u] = key_slot<PAGED>(p, seq, (int)min(row0 + u * RPP, hi - 1));
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      V::load(base + slot[u] * V::ROW_BYTES + c * 16, v[u]);
      s[u] = 1.f;
      if (DT == MISA_FP8_E4M3) s[u] = kscale[slot[u]];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (row0 + u * RPP < hi) {
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] = fmaf(v[u][e], s[u], acc[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < N; ++e) red[r][c * N + e] = acc[e];
  __syncthreads();
  if (tid < kD) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RPP; ++i) s += red[i][tid];
    if (slices == 1) {
      const long long cnt = hi - lo;
      Kp[((size_t)seq * p.M + b) * kD + tid] = cnt > 0 ? s / (float)cnt : 0.f;
    } else {
      Kp[(((size_t)seq * p.M + b) * slices + slice) * kD + tid] = s;  // empty slices write 0
    }
  }
}

// Adds the slice sums of every block in a fixed order (eight interleaved
// subsets, then those in order) and divides by the token count.
__global__ __launch_bounds__(1024) void pool_combine_kernel(Prob p, int slices,
                                                            const int* __restrict__ from_token,
                                                            const float* __restrict__ part,
                                                            float* __restrict__ Kp) {
  __shared__ float red[8][kD];
  const int seq = blockIdx.y, c = threadIdx.x % kD, g = threadIdx.x / kD;
  int b = blockIdx.x;
  if (from_token) {
    const int len = seq_length(p, seq);
    b += min(max(from_token[seq], 0), len) / p.B;
    if ((long long)b * p.B >= len) return;
  }
  const float* src = part + ((size_t)seq * p.M + b) * slices * kD + c;
  float s = 0.f;
#pragma unroll 4
  for (int i = g; i < slices; i += 8) s += src[(size_t)i * kD];
  red[g][c] = s;
  __syncthreads();
  if (g == 0) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += red[i][c];
    const int len = seq_length(p, seq);
    const long long lo = (long long)b * p.B;
    const long long cnt = min(lo + (long long)p.B, (long long)len) - lo;
    Kp[((size_t)seq * p.M + b) * kD + c] = cnt > 0 ? t / (float)cnt : 0.f;
  }
}

static int pool_slices(const Prob& p) {
  return p.B > kPoolSplitFrom ? (int)(((long long)min(p.B, p.L) + kPoolSlice - 1) / kPoolSlice) : 1;
}

size_t pool_ws_bytes(const Prob& p) {
  const int sl = pool_slices(p);
  return sl == 1 ? 0 : (size_t)p.n_seq * p.M * sl * kD * sizeof(float);
}

hipError_t launch_pool(const Prob& p, int k_dtype, const void* K, const float* kscale, float* Kp,
                       void* ws, hipStream_t st, const int* from_token, int max_blocks) {
  const int sl = pool_slices(p);
  const int nb = from_token ? std::min(max_blocks, p.M) : p.M;
  const dim3 grid(nb * sl, p.n_seq), block(256);
  float* dst = sl == 1 ? Kp : static_cast<float*>(ws);
#define GO(DT)                                                                                   \
  if (p.page_table) pool_kernel<DT, true><<<grid, block, 0, st>>>(p, sl, from_token, K, kscale, dst); \
  else pool_kernel<DT, false><<<grid, block, 0, st>>>(p, sl, from_token, K, kscale, dst)
  switch (k_dtype) {
    case MISA_F32: GO(MISA_F32); break;
    case MISA_BF16: GO(MISA_BF16); break;
    default: GO(MISA_FP8_E4M3); break;
  }
#undef GO
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sl == 1) return e;
  pool_combine_kernel<<<dim3(nb, p.n_seq), 1024, 0, st>>>(p, sl, from_token, dst, Kp);
  return hipGetLastError();
}

}  // namespace misa
