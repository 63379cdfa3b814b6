// Comparison indexers assembled from the library's own stages: HISA (preliminaries,
// "Indexer in HISA": Eq. block_score, Eq. final_topk) and the MoBA-style Block-Sparse
// selector (Experimental results, "Baselines").
//
//   block scores  J[t,b] = sum over ALL heads of w_j ReLU(q_j . k~_b) for the complete
//                 blocks inside the query's visible prefix (block_score_kernel, fp32
//                 FMA on the fp32 pooled keys: these scores only rank blocks);
//   block choice  the first and the last block always, the best other blocks up to m in
//                 all: both get score +inf and the row top-k kernel takes m;
//   HISA          the tokens of those blocks are the candidate list of the dense fine
//                 stage (the re-rank kernels of misa_rerank);
//   Block-Sparse  the tokens of those blocks are the selection.
#include "kernels.h"

namespace misa {

// One thread per pooled block of one query; the query's head rows sit in LDS as floats.
// Only complete blocks strictly inside the prefix are scored, from Kp: the first block
// and the last one (the only one that can be partial) are always kept, so their scores
// are never compared and are set to +inf; blocks past the prefix get -inf.
template <int QDT>
__global__ __launch_bounds__(256) void block_score_kernel(Prob p, const void* __restrict__ Q,
                                                          const float* __restrict__ W,
                                                          const float* __restrict__ Kp,
                                                          float* __restrict__ J) {
  __shared__ float qs[kMaxH][kD];
  __shared__ float wsm[kMaxH];
  using QV = Vec16<QDT>;
  const int t = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  const int n = visible(p, seq, t);
  const int Mn = (int)(((long long)n + p.B - 1) / p.B);
  const size_t qrow = (size_t)seq * p.n_q + t;
  const int b = blockIdx.x * 256 + tid;

  for (int i = tid; i < p.H * (kD / QV::N); i += 256) {
    const int j = i / (kD / QV::N), c = i % (kD / QV::N);
    float v[QV::N];
    QV::load(static_cast<const char*>(Q) + ((qrow * p.H + j) * kD + c * QV::N) * (QV::ROW_BYTES / kD), v);
#pragma unroll
    for (int e = 0; e < QV::N; ++e) qs[j][c * QV::N + e] = v[e];
  }
  for (int j = tid; j < p.H; j += 256) wsm[j] = W[qrow * p.H + j];
  __syncthreads();
  if (b >= p.M) return;
  float out = -INFINITY;
  if (b < Mn) {
    if (b == 0 || b == Mn - 1) {
      out = INFINITY;  // always kept
    } else {
      float kv[kD];
      const float* src = Kp + ((size_t)seq * p.M + b) * kD;
#pragma unroll
      for (int c = 0; c < kD; c += 4) {
        const float4 v = *reinterpret_cast<const float4*>(src + c);
        kv[c] = v.x; kv[c + 1] = v.y; kv[c + 2] = v.z; kv[c + 3] = v.w;
      }
      float total = 0.f;
      for (int j = 0; j < p.H; ++j) {
        float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
        for (int c = 0; c < kD; c += 4) {
          d0 = fmaf(qs[j][c], kv[c], d0);
          d1 = fmaf(qs[j][c + 1], kv[c + 1], d1);
          d2 = fmaf(qs[j][c + 2], kv[c + 2], d2);
          d3 = fmaf(qs[j][c + 3], kv[c + 3], d3);
        }
        total = fmaf(wsm[j], relu((d0 + d1) + (d2 + d3)), total);
      }
      out = total;
    }
  }
  J[qrow * p.M + b] = out;
}

// cand[row, i * B + o] = token o of the i-th selected block, -1 if the block slot is
// empty or the token is not visible.
__global__ __launch_bounds__(256) void expand_blocks_kernel(Prob p, int m, const int* __restrict__ blocks,
                                                            int* __restrict__ cand) {
  const int t = blockIdx.y, seq = blockIdx.z;
  const size_t row = (size_t)seq * p.n_q + t;
  const int n = visible(p, seq, t);
  const long long slot = (long long)blockIdx.x * 256 + threadIdx.x;
  if (slot >= (long long)m * p.B) return;
  const int i = (int)(slot / p.B), o = (int)(slot % p.B);
  const int b = blocks[row * m + i];
  const long long tok = (long long)b * p.B + o;
  cand[row * (size_t)m * p.B + slot] = (b >= 0 && tok < n) ? (int)tok : -1;
}

namespace {
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
}

size_t hisa_ws_bytes(const Prob& p, int m) {
  if (m < 2) return 0;
  const size_t rows = (size_t)p.n_seq * p.n_q, kc = (size_t)m * p.B;
  return up256(rows * p.M * sizeof(float)) + up256(rows * m * sizeof(int)) + up256(rows * kc * sizeof(int)) +
         up256(rows * kc * sizeof(float));
}

// k == 0: Block-Sparse (idx receives the m * B candidate tokens); otherwise HISA.
hipError_t launch_hisa(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                       const float* Kp, const void* K, const float* kscale, int m, int k, int* blocks,
                       int* idx, float* val, void* ws, hipStream_t st) {
  const size_t rows = (size_t)p.n_seq * p.n_q, kc = (size_t)m * p.B;
  char* base = static_cast<char*>(ws);
  float* J = reinterpret_cast<float*>(base);
  int* C = reinterpret_cast<int*>(base + up256(rows * p.M * sizeof(float)));
  int* cand = reinterpret_cast<int*>(reinterpret_cast<char*>(C) + up256(rows * m * sizeof(int)));
  float* dense = reinterpret_cast<float*>(reinterpret_cast<char*>(cand) + up256(rows * kc * sizeof(int)));
  if (blocks) C = blocks;
  if (k == 0) cand = idx;

  const dim3 g1((p.M + 255) / 256, p.n_q, p.n_seq);
  if (q_dtype == MISA_F32) block_score_kernel<MISA_F32><<<g1, 256, 0, st>>>(p, Q, W, Kp, J);
  else block_score_kernel<MISA_BF16><<<g1, 256, 0, st>>>(p, Q, W, Kp, J);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the m best blocks of every row of J (all M slots are scanned, -inf slots never chosen)
  e = launch_topk(p, J, p.M, m, nullptr, C, nullptr, nullptr, st, nullptr, true);
  if (e != hipSuccess) return e;
  const dim3 g3((unsigned)((kc + 255) / 256), p.n_q, p.n_seq);
  expand_blocks_kernel<<<g3, 256, 0, st>>>(p, m, C, cand);
  if ((e = hipGetLastError()) != hipSuccess || k == 0) return e;
  e = launch_score(p, k_dtype, q_dtype, Q, W, nullptr, K, kscale, cand, (int)kc, dense, st);
  if (e != hipSuccess) return e;
  return launch_topk(p, dense, (int)kc, k, cand, idx, val, nullptr, st);
}

}  // namespace misa
