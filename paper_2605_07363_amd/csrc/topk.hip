// Stage 4: exact per-row top-k (Eq. dsa_topk, Eq. misa_topk, Eq. misa_candidate).
//
// One 1024-thread workgroup per score row.  The k-th largest value is found by
// a most-significant-digit-first radix select (11 + 11 + 10 bits) on an
// order-preserving integer image of the fp32 scores, with the digit histograms
// in LDS.  Elements that are certainly selected (a more significant digit
// above the threshold digit) are marked in an LDS bitmap as soon as that is
// known; elements equal to the threshold value go to a second bitmap from
// which the lowest-index ones are taken, which implements "ties to the lower
// index" exactly.  The selected set is finally expanded from the bitmap in
// index order with one block-wide prefix sum, so the output is ascending and
// bit-reproducible without any sort.
#include "kernels.h"

namespace misa {

constexpr int kTopkThreads = 1024;
constexpr int kBins = 2048;

// Finds the digit d (scanning from the top) with count(digit > d) < need <= count(digit >= d).
// Thread i owns bins 2047-2i and 2046-2i.  Writes {d, need - count(digit > d)} to out[0..1].
__device__ __forceinline__ void find_threshold_bin(const int* hist, int need, int* scan_scratch,
                                                   int* out) {
  const int tid = threadIdx.x;
  const int ba = kBins - 1 - 2 * tid, bb = ba - 1;
  const int ha = hist[ba], hb = hist[bb];
  int total;
  const int above = block_exclusive_scan(ha + hb, scan_scratch, &total);
  if (above < need && need <= above + ha) {
    out[0] = ba; out[1] = need - above;
  } else if (above + ha < need && need <= above + ha + hb) {
    out[0] = bb; out[1] = need - above - ha;
  }
  __syncthreads();
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(Prob p, const float* __restrict__ S,
                                                            int row_len, int k,
                                                            const int* __restrict__ map,
                                                            int* __restrict__ idx,
                                                            float* __restrict__ val) {
  extern __shared__ uint32_t bitmaps[];  // sel[nwords_max] then eq[nwords_max]
  __shared__ int hist[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[2];

  const int t = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const float* s = S + row * row_len;
  const int n = map ? row_len : visible(p, seq, t);
  const int nwords_max = (row_len + 31) / 32;
  uint32_t* sel = bitmaps;
  uint32_t* eq = bitmaps + nwords_max;
  const int nwords = (n + 31) / 32;
  int* out_idx = idx + row * k;
  float* out_val = val ? val + row * k : nullptr;

  for (int i = tid; i < nwords; i += kTopkThreads) { sel[i] = 0; eq[i] = 0; }
  for (int i = tid; i < kBins; i += kTopkThreads) hist[i] = 0;
  __syncthreads();

  // ---- pass 1: histogram of the top 11 bits
  for (int i = tid; i < n; i += kTopkThreads) atomicAdd(&hist[order_key(s[i]) >> 21], 1);
  __syncthreads();

  int selectable = n;
  if (map) {  // never select -inf slots (skipped candidates): they live in bins <= 3
    selectable = n - (hist[0] + hist[1] + hist[2] + hist[3]);
  }
  const int k_eff = min(k, selectable);
  for (int i = k_eff + tid; i < k; i += kTopkThreads) {
    out_idx[i] = -1;
    if (out_val) out_val[i] = -INFINITY;
  }
  if (k_eff == 0) return;

  if (k_eff == n) {
    for (int i = tid; i < nwords; i += kTopkThreads) {
      const int rem = n - i * 32;
      sel[i] = rem >= 32 ? 0xFFFFFFFFu : ((1u << rem) - 1u);
    }
    __syncthreads();
  } else {
    find_threshold_bin(hist, k_eff, scan_scratch, thr);
    const uint32_t d1 = thr[0];
    int need = thr[1];
    __syncthreads();
    for (int i = tid; i < kBins; i += kTopkThreads) hist[i] = 0;
    __syncthreads();

    // ---- pass 2: mark digit1 > d1; histogram digit 2 within digit1 == d1
    for (int i = tid; i < n; i += kTopkThreads) {
      const uint32_t key = order_key(s[i]);
      const uint32_t a = key >> 21;
      if (a > d1) atomicOr(&sel[i >> 5], 1u << (i & 31));
      else if (a == d1) atomicAdd(&hist[(key >> 10) & 0x7FF], 1);
    }
    __syncthreads();
    find_threshold_bin(hist, need, scan_scratch, thr);
    const uint32_t d2 = thr[0];
    need = thr[1];
    __syncthreads();
    for (int i = tid; i < kBins; i += kTopkThreads) hist[i] = 0;
    __syncthreads();

    // ---- pass 3: within digit1 == d1: mark digit2 > d2; histogram digit 3 within == d2
    const uint32_t pre22 = (d1 << 11) | d2;
    for (int i = tid; i < n; i += kTopkThreads) {
      const uint32_t key = order_key(s[i]);
      if ((key >> 21) != d1) continue;
      const uint32_t b = (key >> 10) & 0x7FF;
      if (b > d2) atomicOr(&sel[i >> 5], 1u << (i & 31));
      else if (b == d2) atomicAdd(&hist[key & 0x3FF], 1);
    }
    __syncthreads();
    find_threshold_bin(hist, need, scan_scratch, thr);
    const uint32_t d3 = thr[0];
    need = thr[1];  // how many elements equal to the threshold value are taken
    __syncthreads();
    const uint32_t tkey = (pre22 << 10) | d3;

    // ---- pass 4: within the 22-bit prefix: mark > threshold, collect == threshold
    for (int i = tid; i < n; i += kTopkThreads) {
      const uint32_t key = order_key(s[i]);
      if ((key >> 10) != pre22) continue;
      if (key > tkey) atomicOr(&sel[i >> 5], 1u << (i & 31));
      else if (key == tkey) atomicOr(&eq[i >> 5], 1u << (i & 31));
    }
    __syncthreads();

    // ---- take the `need` lowest-index elements among the ties
    const int wpt = (nwords + kTopkThreads - 1) / kTopkThreads;
    const int w_lo = min(tid * wpt, nwords), w_hi = min(w_lo + wpt, nwords);
    int cnt = 0;
    for (int w = w_lo; w < w_hi; ++w) cnt += __popc(eq[w]);
    int total;
    int before = block_exclusive_scan(cnt, scan_scratch, &total);
    for (int w = w_lo; w < w_hi && before < need; ++w) {
      uint32_t bits = eq[w];
      const int c = __popc(bits);
      int take = min(c, need - before);
      before += c;
      uint32_t kept = 0;
      while (take-- > 0) {
        const uint32_t low = bits & (0u - bits);
        kept |= low;
        bits ^= low;
      }
      sel[w] |= kept;  // words are owned by one thread here
    }
    __syncthreads();
  }

  // ---- expand the bitmap in index order
  const int wpt = (nwords + kTopkThreads - 1) / kTopkThreads;
  const int w_lo = min(tid * wpt, nwords), w_hi = min(w_lo + wpt, nwords);
  int cnt = 0;
  for (int w = w_lo; w < w_hi; ++w) cnt += __popc(sel[w]);
  int total;
  int pos = block_exclusive_scan(cnt, scan_scratch, &total);
  for (int w = w_lo; w < w_hi; ++w) {
    uint32_t bits = sel[w];
    while (bits) {
      const int i = w * 32 + __ffs(bits) - 1;
      bits &= bits - 1;
      if (pos < k) {  // always true when the selection is consistent
        out_idx[pos] = map ? map[row * row_len + i] : i;
        if (out_val) out_val[pos] = s[i];
      }
      ++pos;
    }
  }
}

hipError_t launch_topk(const Prob& p, const float* S, int row_len, int k, const int* map, int* idx,
                       float* val, hipStream_t st) {
  const size_t lds = (size_t)2 * ((row_len + 31) / 32) * sizeof(uint32_t);
  static size_t attr_bytes = 48 * 1024;  // default dynamic LDS limit
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(topk_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  const dim3 grid(p.n_q, p.n_seq);
  topk_kernel<<<grid, kTopkThreads, lds, st>>>(p, S, row_len, k, map, idx, val);
  return hipGetLastError();
}

}  // namespace misa
