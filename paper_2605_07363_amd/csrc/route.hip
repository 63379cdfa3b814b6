// Stage 2: block-pooled head router (Eq. misa_route_score, Eq. misa_route).
//
// route_partial_kernel: lane = head.  Each lane keeps its query head in
// registers; the pooled key of the block being visited is the same for the
// whole wavefront, so it is fetched with wave-uniform (scalar) loads and every
// FMA takes one scalar and one vector operand.  The four wavefronts of a
// workgroup stride over the blocks of one split of the prefix; partial sums of
// ReLU(q.k~) go to the workspace.
// route_finalize_kernel: adds the causal tail block (mean of the raw keys of
// the last, partial block of a query that does not sit at the end of the
// cache), scales by |w| / M_n and selects the top-h heads by rank counting.
#include "kernels.h"

namespace misa {

template <int QDT>
__device__ __forceinline__ void load_query_head(const void* Q, size_t head_index, float* qv) {
  using V = Vec16<QDT>;
  const char* src = static_cast<const char*>(Q) + head_index * V::ROW_BYTES;
#pragma unroll
  for (int c = 0; c < kD / V::N; ++c) V::load(src + c * 16, qv + c * V::N);
}

// Blocks whose pooled key in Kp is valid for a query with prefix n: all
// ceil(n/B) when the query sits at the end of the cache (the partial block in
// Kp then holds exactly its tokens), else only the complete ones.
__device__ __forceinline__ int pooled_blocks(int n, int len, int B) {
  return n == len ? (int)(((long long)n + B - 1) / B) : n / B;
}

template <int QDT>
__global__ __launch_bounds__(256) void route_partial_kernel(Prob p, int splits,
                                                            const void* __restrict__ Q,
                                                            const float* __restrict__ Kp,
                                                            float* __restrict__ part) {
  __shared__ float red[4][kWave];
  const int split = blockIdx.x, t = blockIdx.y, seq = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = visible(p, seq, t), len = seq_length(p, seq);
  const int nb = pooled_blocks(n, len, p.B);
  const int per = (p.M + splits - 1) / splits;
  const int b_lo = split * per, b_hi = min(b_lo + per, nb);

  float qv[kD];
  if (lane < p.H) {
    load_query_head<QDT>(Q, ((size_t)seq * p.n_q + t) * p.H + lane, qv);
  } else {
#pragma unroll
    for (int c = 0; c < kD; ++c) qv[c] = 0.f;
  }

  float acc = 0.f;
  for (int b = b_lo + wave; b < b_hi; b += 4) {
    const float* __restrict__ kp = Kp + ((size_t)seq * p.M + b) * kD;  // wave-uniform
    float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
    for (int c = 0; c < kD; c += 4) {
      d0 = fmaf(qv[c], kp[c], d0);
      d1 = fmaf(qv[c + 1], kp[c + 1], d1);
      d2 = fmaf(qv[c + 2], kp[c + 2], d2);
      d3 = fmaf(qv[c + 3], kp[c + 3], d3);
    }
    acc += fmaxf((d0 + d1) + (d2 + d3), 0.f);
  }
  red[wave][lane] = acc;
  __syncthreads();
  if (wave == 0) {
    const float s = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    part[(((size_t)seq * p.n_q + t) * splits + split) * kWave + lane] = s;
  }
}

template <int KDT, int QDT>
__global__ __launch_bounds__(128) void route_finalize_kernel(
    Prob p, int splits, const void* __restrict__ Q, const float* __restrict__ W,
    const void* __restrict__ K, const float* __restrict__ kscale, const float* __restrict__ part,
    int* __restrict__ heads, float* __restrict__ E) {
  __shared__ float tailk[kD];
  __shared__ float Es[kMaxH];
  __shared__ int sel[kMaxH];
  using KV = Vec16<KDT>;
  const int t = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int n = visible(p, seq, t), len = seq_length(p, seq);
  const int nfull = n / p.B, r = n - nfull * p.B;
  const int Mn = nfull + (r > 0 ? 1 : 0);
  const bool tail = r > 0 && n < len;

  if (tail) {  // mean of keys nfull*B .. n-1, component tid
    const char* base = static_cast<const char*>(K) + (size_t)seq * p.L * KV::ROW_BYTES;
    float s = 0.f;
    for (int row = nfull * p.B; row < n; ++row) {
      const char* src = base + (size_t)row * KV::ROW_BYTES;
      float v;
      if (KDT == MISA_F32) {
        v = reinterpret_cast<const float*>(src)[tid];
      } else if (KDT == MISA_BF16) {
        v = bf16_bits_to_float(reinterpret_cast<const uint16_t*>(src)[tid]);
      } else {
        const uint32_t w = reinterpret_cast<const uint32_t*>(src)[tid >> 2];
        const f32x2 pr = __builtin_amdgcn_cvt_pk_f32_fp8(w >> ((tid & 2) * 8), false);
        v = pr[tid & 1] * kscale[(size_t)seq * p.L + row];
      }
      s += v;
    }
    tailk[tid] = s / (float)r;
  }
  __syncthreads();

  if (tid < p.H) {
    const size_t qi = ((size_t)seq * p.n_q + t) * p.H + tid;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp)
      s += part[(((size_t)seq * p.n_q + t) * splits + sp) * kWave + tid];
    if (tail) {
      float qv[kD];
      load_query_head<QDT>(Q, qi, qv);
      float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
      for (int c = 0; c < kD; c += 4) {
        d0 = fmaf(qv[c], tailk[c], d0);
        d1 = fmaf(qv[c + 1], tailk[c + 1], d1);
        d2 = fmaf(qv[c + 2], tailk[c + 2], d2);
        d3 = fmaf(qv[c + 3], tailk[c + 3], d3);
      }
      s += fmaxf((d0 + d1) + (d2 + d3), 0.f);
    }
    const float e = Mn > 0 ? fabsf(W[qi]) * s / (float)Mn : 0.f;
    Es[tid] = e;
    if (E) E[qi] = e;
  }
  __syncthreads();
  if (tid < p.H) {
    const float e = Es[tid];
    int rank = 0;
    for (int i = 0; i < p.H; ++i) {
      const float o = Es[i];
      rank += (o > e || (o == e && i < tid)) ? 1 : 0;
    }
    sel[tid] = rank < p.h ? 1 : 0;
  }
  __syncthreads();
  if (tid < p.H && sel[tid]) {
    int pos = 0;
    for (int i = 0; i < tid; ++i) pos += sel[i];
    heads[((size_t)seq * p.n_q + t) * p.h + pos] = tid;
  }
}

int route_splits(const Prob& p) {
  // Enough workgroups to cover the chip a few times, but at least 8 blocks per split.
  const long long rows = (long long)p.n_seq * p.n_q;
  long long s = (1024 + rows - 1) / rows;
  const long long cap = (p.M + 7) / 8;
  if (s > cap) s = cap;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return (int)s;
}

size_t route_ws_bytes(const Prob& p) {
  return (size_t)p.n_seq * p.n_q * route_splits(p) * kWave * sizeof(float);
}

hipError_t launch_route(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const float* Kp, const void* K, const float* kscale, int* heads, float* E,
                        void* ws, hipStream_t st) {
  const int splits = route_splits(p);
  float* part = static_cast<float*>(ws);
  const dim3 g1(splits, p.n_q, p.n_seq);
  if (q_dtype == MISA_F32)
    route_partial_kernel<MISA_F32><<<g1, 256, 0, st>>>(p, splits, Q, Kp, part);
  else
    route_partial_kernel<MISA_BF16><<<g1, 256, 0, st>>>(p, splits, Q, Kp, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 g2(p.n_q, p.n_seq);
#define FIN(KD, QD) \
  route_finalize_kernel<KD, QD><<<g2, 128, 0, st>>>(p, splits, Q, W, K, kscale, part, heads, E)
  if (q_dtype == MISA_F32) {
    if (k_dtype == MISA_F32) FIN(MISA_F32, MISA_F32);
    else if (k_dtype == MISA_BF16) FIN(MISA_BF16, MISA_F32);
    else FIN(MISA_FP8_E4M3, MISA_F32);
  } else {
    if (k_dtype == MISA_F32) FIN(MISA_F32, MISA_BF16);
    else if (k_dtype == MISA_BF16) FIN(MISA_BF16, MISA_BF16);
    else FIN(MISA_FP8_E4M3, MISA_BF16);
  }
#undef FIN
  return hipGetLastError();
}

}  // namespace misa
