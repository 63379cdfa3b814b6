// Stage 4: exact per-row top-k (Eq. dsa_topk, Eq. misa_topk, Eq. misa_candidate).
//
// The k-th largest value of a row is found by a most-significant-digit-first
// radix select (11 + 11 + 10 bits) on an order-preserving integer image of the
// fp32 scores.  Selected elements are marked in an LDS bitmap of the row and
// the result is expanded from the bitmap in index order with one block-wide
// prefix sum, so the output is ascending and bit-reproducible without a sort.
//
// Common case: after the first digit, the elements that share the threshold
// digit ("boundary" elements) are few.  They are compacted into a small list
// and every later digit, and the tie rule (equal values: lower index first),
// is resolved on that list in LDS, so the row itself is read only twice.
// If the boundary bin is larger than the list (heavily repeated values), the
// kernel falls back to two more digit passes over the row and a bitmap of the
// elements equal to the threshold value.
//
// Few long rows (decode): one workgroup per row would leave most of the chip
// idle, so the two passes over the row are split over many workgroups
// (topk_hist_kernel, topk_partition_kernel) that leave the histogram and the
// compacted lists in the workspace; topk_kernel<true> then finishes each row
// from those lists.
#include "kernels.h"
#include "radix.h"

namespace misa {

constexpr int kCap = 7000;          // boundary list capacity (entries); sized so two workgroups share a CU
constexpr int kChunk = 8192;        // row elements per workgroup in the split passes
constexpr int kPreHeader = kBins + 64;  // hist, then n_certain, n_boundary, padding

// Visits elements lo..hi-1 of a row with all threads of the block.  Eight
// coalesced loads per thread are in flight before the first one is used.  f is
// called by every thread of every wavefront in each round (in == false past
// the end), so it may contain wavefront-wide operations.
template <typename F>
__device__ __forceinline__ void scan_row(const float* __restrict__ s, int lo, int hi, F f) {
  constexpr int U = 8;
  for (int base = lo; base < hi; base += kTopkThreads * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * kTopkThreads + (int)threadIdx.x;
      v[u] = i < hi ? s[i] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = base + u * kTopkThreads + (int)threadIdx.x;
      f(i, v[u], i < hi);
    }
  }
}

__device__ __forceinline__ int pre_stride(int k) { return (kPreHeader + k + 2 * kCap + 63) & ~63; }

// ---------------------------------------------------------------- split pass 1
__global__ __launch_bounds__(kTopkThreads) void topk_hist_kernel(Prob p, const float* __restrict__ S,
                                                                 int k, int* __restrict__ pre) {
  __shared__ int hist[kBins];
  const int chunk = blockIdx.x, t = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const int n = visible(p, seq, t);
  const int lo = chunk * kChunk, hi = min(lo + kChunk, n);
  if (lo >= hi) return;
  zero_hist(hist);
  const float* s = S + row * p.L;
  scan_row(s, lo, hi, [&](int, float v, bool in) {
    if (in) atomicAdd(&hist[order_key(v) >> 21], 1);
  });
  __syncthreads();
  int* g = pre + row * pre_stride(k);
  for (int i = tid; i < kBins; i += kTopkThreads)
    if (hist[i]) atomicAdd(&g[i], hist[i]);
}

// ---------------------------------------------------------------- split pass 2
// Each workgroup first compacts its chunk into LDS (certain indices from the
// front, boundary entries from the back of one 8192-entry array: together they
// never exceed the chunk), then reserves room in the row's global lists with
// one atomic per list and copies the entries out with coalesced stores.
__global__ __launch_bounds__(kTopkThreads) void topk_partition_kernel(Prob p,
                                                                      const float* __restrict__ S,
                                                                      int k, int* __restrict__ pre) {
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ int cnt[2];    // certain, boundary entries of this chunk
  __shared__ int base[2];   // their first slots in the row's lists
  __shared__ int ent_idx[kChunk];
  __shared__ uint32_t ent_key[kChunk];
  const int chunk = blockIdx.x, t = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const int n = visible(p, seq, t);
  const int lo = chunk * kChunk, hi = min(lo + kChunk, n);
  const int k_eff = min(k, n);
  if (lo >= hi || k_eff == n) return;  // k_eff == n: everything is selected, nothing to partition
  int* g = pre + row * pre_stride(k);
  if (tid < 2) cnt[tid] = 0;
  find_threshold_bin(g, k_eff, scan_scratch, thr);
  const uint32_t d1 = thr[0];
  const bool listed = thr[2] <= kCap;
  int* certain = g + kPreHeader;
  int* bkey = certain + k;
  int* bidx = bkey + kCap;
  const float* s = S + row * p.L;
  scan_row(s, lo, hi, [&](int i, float v, bool in) {
    const uint32_t key = order_key(v), a = key >> 21;
    const int c = wave_append(in && a > d1, &cnt[0]);
    if (c >= 0) ent_idx[c] = i;
    if (listed) {
      const int b = wave_append(in && a == d1, &cnt[1]);
      if (b >= 0) { ent_idx[kChunk - 1 - b] = i; ent_key[kChunk - 1 - b] = key; }
    }
  });
  __syncthreads();
  const int nc = cnt[0], nb = cnt[1];
  if (tid == 0) base[0] = nc ? atomicAdd(&g[kBins], nc) : 0;
  if (tid == 64) base[1] = nb ? atomicAdd(&g[kBins + 1], nb) : 0;
  __syncthreads();
  for (int i = tid; i < nc; i += kTopkThreads) certain[base[0] + i] = ent_idx[i];
  for (int i = tid; i < nb; i += kTopkThreads) {
    bkey[base[1] + i] = (int)ent_key[kChunk - 1 - i];
    bidx[base[1] + i] = ent_idx[kChunk - 1 - i];
  }
}

// ---------------------------------------------------------------- per-row kernel
template <bool PRE>
__device__ __forceinline__ void topk_row(const Prob& p, const float* __restrict__ S, int row_len,
                                         int k, const int* __restrict__ map, int* __restrict__ idx,
                                         float* __restrict__ val, const int* __restrict__ pre, int t,
                                         int seq, uint32_t* dyn, bool all_slots = false) {
  // dyn: sel bitmap, then eq bitmap OR boundary list (keys, idx)
  __shared__ int hist[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ int list_len;

  const int tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const float* s = S + row * row_len;
  const int n = (map || all_slots) ? row_len : visible(p, seq, t);
  const int nwords_max = (row_len + 31) / 32;
  uint32_t* sel = dyn;
  uint32_t* eq = dyn + nwords_max;       // fallback path
  uint32_t* lkey = dyn + nwords_max;     // list path (aliases eq)
  int* lidx = reinterpret_cast<int*>(lkey + kCap);
  const int nwords = (n + 31) / 32;
  int* out_idx = idx + row * k;
  float* out_val = val ? val + row * k : nullptr;
  const int* g = PRE ? pre + row * pre_stride(k) : nullptr;

  for (int i = tid; i < nwords; i += kTopkThreads) sel[i] = 0;
  if (tid == 0) list_len = 0;
  if (PRE) {
    for (int i = tid; i < kBins; i += kTopkThreads) hist[i] = g[i];
    __syncthreads();
  } else {
    zero_hist(hist);
    // ---- pass 1: histogram of the top 11 bits
    scan_row(s, 0, n, [&](int, float v, bool in) {
      if (in) atomicAdd(&hist[order_key(v) >> 21], 1);
    });
    __syncthreads();
  }

  int selectable = n;
  if (map || all_slots) {  // never select -inf slots (skipped candidates): they live in bins <= 3
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
    const bool listed = thr[2] <= kCap;
    __syncthreads();
    zero_hist(hist);

    if (listed) {
      // ---- pass 2: mark digit1 > d1, compact digit1 == d1 into the LDS list
      int len;
      if (PRE) {
        const int nc = g[kBins];
        len = g[kBins + 1];
        const int* certain = g + kPreHeader;
        const int* bkey = certain + k;
        const int* bidx = bkey + kCap;
        for (int i = tid; i < nc; i += kTopkThreads) {
          const int e = certain[i];
          atomicOr(&sel[e >> 5], 1u << (e & 31));
        }
        for (int i = tid; i < len; i += kTopkThreads) { lkey[i] = (uint32_t)bkey[i]; lidx[i] = bidx[i]; }
        __syncthreads();
      } else {
        scan_row(s, 0, n, [&](int i, float v, bool in) {
          const uint32_t key = order_key(v), a = key >> 21;
          if (in && a > d1) atomicOr(&sel[i >> 5], 1u << (i & 31));
          const int b = wave_append(in && a == d1, &list_len);
          if (b >= 0) { lkey[b] = key; lidx[b] = i; }
        });
        __syncthreads();
        len = list_len;
      }
      // ---- digits 2 and 3 on the list
      for (int i = tid; i < len; i += kTopkThreads) atomicAdd(&hist[(lkey[i] >> 10) & 0x7FF], 1);
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t d2 = thr[0];
      need = thr[1];
      __syncthreads();
      zero_hist(hist);
      for (int i = tid; i < len; i += kTopkThreads) {
        const uint32_t key = lkey[i];
        const uint32_t b = (key >> 10) & 0x7FF;
        if (b > d2) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
        else if (b == d2) atomicAdd(&hist[key & 0x3FF], 1);
      }
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t low21 = (d2 << 10) | (uint32_t)thr[0];
      need = thr[1];
      const int ties = thr[2];
      __syncthreads();
      zero_hist(hist);
      if (ties == need) {
        for (int i = tid; i < len; i += kTopkThreads) {
          const uint32_t l = lkey[i] & 0x1FFFFFu;
          if ((l >> 10) == d2 && l >= low21) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
        }
      } else {
        // More ties than places: take the `need` lowest indices among them, by the
        // same digit search on (high, low) halves of the index, inverted so that a
        // lower index ranks higher.  Indices are distinct, so this is exact.
        for (int i = tid; i < len; i += kTopkThreads) {
          const uint32_t l = lkey[i] & 0x1FFFFFu;
          if ((l >> 10) == d2 && l > low21) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
          else if (l == low21) atomicAdd(&hist[kBins - 1 - (lidx[i] >> 10)], 1);
        }
        __syncthreads();
        find_threshold_bin(hist, need, scan_scratch, thr);
        const int hi_digit = kBins - 1 - thr[0];
        need = thr[1];
        __syncthreads();
        zero_hist(hist);
        for (int i = tid; i < len; i += kTopkThreads) {
          if ((lkey[i] & 0x1FFFFFu) != low21) continue;
          const int e = lidx[i];
          if ((e >> 10) < hi_digit) atomicOr(&sel[e >> 5], 1u << (e & 31));
          else if ((e >> 10) == hi_digit) atomicAdd(&hist[kBins - 1 - (e & 0x3FF)], 1);
        }
        __syncthreads();
        find_threshold_bin(hist, need, scan_scratch, thr);
        const int lo_digit = kBins - 1 - thr[0];
        for (int i = tid; i < len; i += kTopkThreads) {
          if ((lkey[i] & 0x1FFFFFu) != low21) continue;
          const int e = lidx[i];
          if ((e >> 10) == hi_digit && (e & 0x3FF) <= lo_digit) atomicOr(&sel[e >> 5], 1u << (e & 31));
        }
      }
      __syncthreads();
    } else {
      // ---- fallback: two more digit passes over the row, ties through a bitmap
      for (int i = tid; i < nwords; i += kTopkThreads) eq[i] = 0;
      __syncthreads();
      scan_row(s, 0, n, [&](int i, float v, bool in) {
        const uint32_t key = order_key(v), a = key >> 21;
        if (!in) return;
        if (a > d1) atomicOr(&sel[i >> 5], 1u << (i & 31));
        else if (a == d1) atomicAdd(&hist[(key >> 10) & 0x7FF], 1);
      });
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t d2 = thr[0];
      need = thr[1];
      __syncthreads();
      zero_hist(hist);
      const uint32_t pre22 = (d1 << 11) | d2;
      scan_row(s, 0, n, [&](int i, float v, bool in) {
        const uint32_t key = order_key(v);
        if (!in || (key >> 21) != d1) return;
        const uint32_t b = (key >> 10) & 0x7FF;
        if (b > d2) atomicOr(&sel[i >> 5], 1u << (i & 31));
        else if (b == d2) atomicAdd(&hist[key & 0x3FF], 1);
      });
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t tkey = (pre22 << 10) | (uint32_t)thr[0];
      need = thr[1];  // how many elements equal to the threshold value are taken
      __syncthreads();
      scan_row(s, 0, n, [&](int i, float v, bool in) {
        const uint32_t key = order_key(v);
        if (!in || (key >> 10) != pre22) return;
        if (key > tkey) atomicOr(&sel[i >> 5], 1u << (i & 31));
        else if (key == tkey) atomicOr(&eq[i >> 5], 1u << (i & 31));
      });
      __syncthreads();
      // take the `need` lowest-index elements among the ties
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

template <bool PRE>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(Prob p, const float* __restrict__ S,
                                                            int row_len, int k,
                                                            const int* __restrict__ map,
                                                            int* __restrict__ idx,
                                                            float* __restrict__ val,
                                                            const int* __restrict__ pre,
                                                            bool all_slots) {
  extern __shared__ uint32_t dyn[];
  topk_row<PRE>(p, S, row_len, k, map, idx, val, pre, blockIdx.x, blockIdx.y, dyn, all_slots);
}

// Only the rows r with only[r] != 0 (rows another path could not finish).  Normally
// there is none, so a small grid strides over the rows.
__global__ __launch_bounds__(kTopkThreads) void topk_only_kernel(Prob p, const float* __restrict__ S,
                                                                 int k, int* __restrict__ idx,
                                                                 float* __restrict__ val,
                                                                 const int* __restrict__ only) {
  extern __shared__ uint32_t dyn[];
  const int rows = p.n_seq * p.n_q;
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    if (!only[r]) continue;
    topk_row<false>(p, S, p.L, k, nullptr, idx, val, nullptr, r % p.n_q, r / p.n_q, dyn);
    __syncthreads();
  }
}

__global__ void zero_ints_kernel(int* __restrict__ pre, int stride, int count) {
  // clears the histogram and the two list counters of one row per blockIdx.y
  int* g = pre + (size_t)blockIdx.y * stride;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) g[i] = 0;
}

// Rows are split over several workgroups when there are too few of them to fill the chip.
static bool use_split(const Prob& p) {
  return (long long)p.n_seq * p.n_q < 256 && p.L >= 4 * kChunk;
}

size_t topk_ws_bytes(const Prob& p, int k) {
  if (!use_split(p) || k < 1) return 0;
  const size_t stride = (size_t)((kPreHeader + k + 2 * kCap + 63) & ~63);
  return (size_t)p.n_seq * p.n_q * stride * sizeof(int);
}

template <int WHICH>  // 0: topk_kernel<false>, 1: topk_kernel<true>, 2: topk_only_kernel
static hipError_t set_lds_limit(size_t lds) {
  static size_t attr_bytes = 48 * 1024;  // default dynamic LDS limit
  if (lds > attr_bytes) {
    const void* f = WHICH == 0 ? reinterpret_cast<const void*>(topk_kernel<false>)
                  : WHICH == 1 ? reinterpret_cast<const void*>(topk_kernel<true>)
                               : reinterpret_cast<const void*>(topk_only_kernel);
    hipError_t e = hipFuncSetAttribute(f,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  return hipSuccess;
}

hipError_t launch_topk(const Prob& p, const float* S, int row_len, int k, const int* map, int* idx,
                       float* val, void* ws, hipStream_t st, const int* only, bool all_slots) {
  const size_t nwords = (size_t)(row_len + 31) / 32;
  const size_t second = nwords * 4 > (size_t)kCap * 8 ? nwords * 4 : (size_t)kCap * 8;
  const size_t lds = nwords * 4 + second;
  const dim3 grid(p.n_q, p.n_seq);
  if (only) {
    hipError_t e = set_lds_limit<2>(lds);
    if (e != hipSuccess) return e;
    const int rows = p.n_seq * p.n_q;
    topk_only_kernel<<<rows < 256 ? rows : 256, kTopkThreads, lds, st>>>(p, S, k, idx, val, only);
    return hipGetLastError();
  }
  if (!map && !all_slots && use_split(p)) {
    int* pre = static_cast<int*>(ws);
    const int stride = (kPreHeader + k + 2 * kCap + 63) & ~63;
    const int rows = p.n_seq * p.n_q;
    zero_ints_kernel<<<dim3(2, rows), 1024, 0, st>>>(pre, stride, kPreHeader);
    const dim3 g2((p.L + kChunk - 1) / kChunk, p.n_q, p.n_seq);
    topk_hist_kernel<<<g2, kTopkThreads, 0, st>>>(p, S, k, pre);
    topk_partition_kernel<<<g2, kTopkThreads, 0, st>>>(p, S, k, pre);
    hipError_t e = set_lds_limit<1>(lds);
    if (e != hipSuccess) return e;
    topk_kernel<true><<<grid, kTopkThreads, lds, st>>>(p, S, row_len, k, map, idx, val, pre, false);
    return hipGetLastError();
  }
  hipError_t e = set_lds_limit<0>(lds);
  if (e != hipSuccess) return e;
  topk_kernel<false><<<grid, kTopkThreads, lds, st>>>(p, S, row_len, k, map, idx, val, nullptr, all_slots);
  return hipGetLastError();
}

}  // namespace misa
