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
// idle.  There topk_prefilter_kernel runs first, up to 16 workgroups per row:
// each derives the same score threshold from a small sample of the row (so
// that a few thousand elements pass, at least k of them but for a negligible
// chance) and hands the elements of its key range that pass to topk_kernel<true>,
// which selects exactly among them.  A row whose hand-over is not usable (fewer
// than k passed, too many for the list, or too many tied around the k-th) is
// redone by the same workgroup with the two passes over the row, so the result
// never depends on the sample.
#include "kernels.h"
#include "radix.h"

namespace misa {

constexpr int kCap = 7000;          // boundary list capacity (entries); sized so two workgroups share a CU
constexpr int kFew = 64;             // entries around the k-th largest that are ranked directly
constexpr int kMaxRanges = 16;      // key ranges (workgroups) per row in the prefilter
constexpr int kMinRange = 8192;     // shortest key range
constexpr int kSampleLines = 256;   // sampled 16-element lines per row (at most)
constexpr int kSegInts = 64 + 2 * kCap;  // per (row, range): header (count; threshold and upper key at 8, 9), then (index, key) pairs

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

// Length of the key ranges the prefilter cuts a row of L elements into (at most kMaxRanges).
__host__ __device__ inline int range_len(int L) {
  const int per = (L + kMaxRanges - 1) / kMaxRanges;
  const int r = (per + 1023) & ~1023;
  return r < kMinRange ? kMinRange : r;
}

// ---------------------------------------------------------------- sampled prefilter
// Workgroup (range, t, seq).  Sample: the row's n visible elements form lines of 16; of every
// `ls` consecutive lines one (picked by a multiplicative hash) is read, at most kSampleLines
// lines.  With m samples, the sample element of rank r = k m/n + 6 sqrt(k m/n) + 8 gives the
// threshold: the number of row elements above it is >= k unless the sample is more than six
// standard deviations off.  Only the two upper digits of that element's key are resolved (22
// bits), so a few more elements pass.  Every workgroup of a row computes the same threshold.
__global__ __launch_bounds__(kTopkThreads) void topk_prefilter_kernel(Prob p,
                                                                      const float* __restrict__ S,
                                                                      int k, int rlen,
                                                                      int* __restrict__ pre) {
  __shared__ int hist[kBins];
  __shared__ int hist2[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ int thr_up[3];
  __shared__ int cnt;
  constexpr int SPT = kSampleLines * 16 / kTopkThreads;  // samples per thread
  constexpr int U = 8;
  const int range = blockIdx.x, t = blockIdx.y, seq = blockIdx.z, tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const int n = visible(p, seq, t);
  const int lo = range * rlen, hi = min(lo + rlen, n);
  const int k_eff = min(k, n);
  if (lo >= hi || k_eff == n) return;   // nothing here / every element is selected anyway
  const float* s = S + row * p.L;
  int* seg = pre + (row * gridDim.x + range) * kSegInts;

  // samples and the first round of the range are loaded together
  const int lines = (n + 15) >> 4;
  const int ls = (lines + kSampleLines - 1) / kSampleLines;
  const int groups = lines / ls;       // >= 1
  uint32_t skey[SPT];
  bool sin[SPT];
  float sv[SPT], cv[U];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    const int smp = tid + u * kTopkThreads, g = smp >> 4;
    const int line = g * ls + (int)((((uint32_t)g * 2654435761u) >> 16) % (uint32_t)ls);
    const int i = line * 16 + (smp & 15);
    sin[u] = g < groups && i < n;
    sv[u] = sin[u] ? s[i] : 0.f;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int i = lo + u * kTopkThreads + tid;
    cv[u] = i < hi ? s[i] : 0.f;
  }
  if (tid == 0) cnt = 0;
  for (int i = tid; i < kBins; i += kTopkThreads) hist2[i] = 0;
  zero_hist(hist);
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    skey[u] = order_key(sv[u]);
    if (sin[u]) atomicAdd(&hist[skey[u] >> 21], 1);
  }
  // number of samples: 16 per sampled line, less what the row's last line lacks if it is one
  int m = 16 * groups;
  {
    const int last = lines - 1, g = last / ls;
    if (g < groups && g * ls + (int)((((uint32_t)g * 2654435761u) >> 16) % (uint32_t)ls) == last)
      m -= 16 * lines - n;
  }
  __syncthreads();
  const float kf = (float)k_eff * (float)m / (float)n;
  const int r = (int)ceilf(kf + 6.f * sqrtf(kf) + 8.f);
  uint32_t tau = 0;                    // r > m: everything passes
  uint32_t upper = 0xFFFFFFFFu;        // top of the digit that holds the sample element of rank r/4
  if (r <= m) {
    find_threshold_bin(hist, r, scan_scratch, thr, max(r / 4, 1), thr_up);
    const uint32_t d1 = thr[0];
    const int need = thr[1];
    upper = ((uint32_t)thr_up[0] << 21) | 0x1FFFFFu;
#pragma unroll
    for (int u = 0; u < SPT; ++u)
      if (sin[u] && (skey[u] >> 21) == d1) atomicAdd(&hist2[(skey[u] >> 10) & 0x7FF], 1);
    __syncthreads();
    find_threshold_bin(hist2, need, scan_scratch, thr);
    tau = (d1 << 21) | ((uint32_t)thr[0] << 10);
  }

  // elements of the range at or above the threshold -> the segment; the count goes on past
  // the capacity so that the reader sees the overflow
  int2* ent = reinterpret_cast<int2*>(seg + 64);
  for (int base = lo; base < hi; base += kTopkThreads * U) {
    if (base > lo) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * kTopkThreads + tid;
        cv[u] = i < hi ? s[i] : 0.f;
      }
    }
    // one counter update per wavefront and round: the slots of its passing elements follow
    // each other in (u, lane) order
    uint32_t key[U];
    unsigned long long mask[U];
    int total = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      key[u] = order_key(cv[u]);
      mask[u] = __ballot(base + u * kTopkThreads + tid < hi && key[u] >= tau);
      total += __popcll(mask[u]);
    }
    if (total) {   // wavefront-uniform
      const int lane = tid & 63;
      int slot = 0;
      if (lane == 0) slot = atomicAdd(&cnt, total);
      slot = __builtin_amdgcn_readfirstlane(slot);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if ((mask[u] >> lane) & 1) {
          const int c = slot + __popcll(mask[u] & ((1ull << lane) - 1ull));
          if (c < kCap) ent[c] = make_int2(base + u * kTopkThreads + tid, (int)key[u]);
        }
        slot += __popcll(mask[u]);
      }
    }
  }
  __syncthreads();
  if (tid == 0) { seg[0] = cnt; seg[8] = (int)tau; seg[9] = (int)upper; }
}

// ---------------------------------------------------------------- per-row kernel
// Candidate mode (CAND): the elements at or above the sampled threshold were left in `pre` by
// topk_prefilter_kernel, in ranges of rlen elements.  They become the list.  One digit is
// taken of key - threshold, scaled so that the interval [threshold, upper key] of the
// hand-over fills the 2047 lower values of the digit (larger keys share digit 2047); entries
// above the digit of the k-th largest are selected, the few entries in it are ranked against
// each other.  Returns false, with nothing selected, if the hand-over is unusable (fewer than
// k entries, more than the list holds) or more than 64 entries share that digit.
__device__ __forceinline__ bool topk_from_candidates(const int* __restrict__ segs, int ranges, int k,
                                                     uint32_t* sel, uint32_t* lkey, int* lidx,
                                                     int* hist, int* scan_scratch, int* thr,
                                                     int* list_len) {
  __shared__ int seg_base[kMaxRanges + 1];
  __shared__ int seg_cnt[kMaxRanges];
  __shared__ int seg_max;
  __shared__ uint32_t bkey[64];
  __shared__ int bidx[64];
  __shared__ uint32_t key_lo, key_span;
  __shared__ int cand_ok;
  const int tid = threadIdx.x;
  if (tid < 64) {   // lane c looks after range c
    const bool live = tid < ranges;
    const int cnt = live ? segs[(size_t)tid * kSegInts] : 0;
    const uint32_t lo_key = (uint32_t)segs[8], up_key = (uint32_t)segs[9];
    const bool bad = live && (cnt < 0 || cnt > kCap);
    const int inc = wave_inclusive_scan(bad ? 0 : cnt);
    int mx = cnt;
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) mx = max(mx, __shfl_xor(mx, o));   // kMaxRanges = 16 lanes matter
    const int tot = __builtin_amdgcn_readlane(inc, 63);
    const bool any_bad = __ballot(bad) != 0;
    if (live) { seg_cnt[tid] = cnt; seg_base[tid] = inc - cnt; }
    if (tid == 0) {
      seg_base[ranges] = tot;
      seg_max = mx;
      key_lo = lo_key;
      key_span = up_key > lo_key ? up_key - lo_key : 1u;
      cand_ok = !any_bad && tot <= kCap && tot >= k;
    }
  }
  __syncthreads();
  if (!cand_ok) return false;

  const int len = seg_base[ranges];
  const uint32_t klo = key_lo, span = key_span;
  const int sh = __clz(span);
  auto digit = [&](uint32_t key) {
    const uint32_t x = key - klo;
    return x > span ? (uint32_t)(kBins - 1) : (x << sh) >> 21;
  };
  // one entry of every range per thread and round.  The loads are unconditional (clamped to
  // the range's last entry and the row's last range), so all of a round are in flight together.
  int cnt_c[kMaxRanges], base_c[kMaxRanges];
#pragma unroll
  for (int c = 0; c < kMaxRanges; ++c) {
    cnt_c[c] = c < ranges ? seg_cnt[c] : 0;
    base_c[c] = seg_base[min(c, ranges)];
  }
  for (int off = tid; off < seg_max; off += kTopkThreads) {
    int2 e[kMaxRanges];
#pragma unroll
    for (int c = 0; c < kMaxRanges; ++c) {
      const int2* ent = reinterpret_cast<const int2*>(segs + (size_t)min(c, ranges - 1) * kSegInts + 64);
      e[c] = ent[min(off, max(cnt_c[c] - 1, 0))];
    }
#pragma unroll
    for (int c = 0; c < kMaxRanges; ++c)
      if (off < cnt_c[c]) {
        const int j = base_c[c] + off;
        lidx[j] = e[c].x;
        lkey[j] = (uint32_t)e[c].y;
        atomicAdd(&hist[digit((uint32_t)e[c].y)], 1);
      }
  }
  __syncthreads();
  find_threshold_bin(hist, k, scan_scratch, thr);
  const uint32_t d1 = thr[0];
  const int need = thr[1], nb = thr[2];
  if (nb > 64 || d1 == kBins - 1) {   // block-uniform
    __syncthreads();
    zero_hist(hist);
    return false;
  }
  for (int i = tid; i < len; i += kTopkThreads) {
    const uint32_t key = lkey[i], a = digit(key);
    if (a > d1) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
    const int b = wave_append(a == d1, list_len);
    if (b >= 0) { bkey[b] = key; bidx[b] = lidx[i]; }
  }
  __syncthreads();
  if (tid < nb) {
    const uint32_t key = bkey[tid];
    const int e = bidx[tid];
    int rank = 0;
    for (int j = 0; j < nb; ++j) {
      const uint32_t kj = bkey[j];
      rank += (kj > key || (kj == key && bidx[j] < e)) ? 1 : 0;
    }
    if (rank < need) atomicOr(&sel[e >> 5], 1u << (e & 31));
  }
  __syncthreads();
  return true;
}

template <bool CAND>
__device__ __forceinline__ void topk_row(const Prob& p, const float* __restrict__ S, int row_len,
                                         int k, const int* __restrict__ map, int* __restrict__ idx,
                                         float* __restrict__ val, const int* __restrict__ pre,
                                         int rlen, int t, int seq, uint32_t* dyn,
                                         bool all_slots = false) {
  // dyn: sel bitmap, then eq bitmap OR list (keys, idx)
  __shared__ int hist[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ int list_len;
  __shared__ int few_len;
  __shared__ uint32_t fkey[kFew];
  __shared__ int fidx[kFew];

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

  for (int i = tid; i < nwords; i += kTopkThreads) sel[i] = 0;
  if (tid == 0) { list_len = 0; few_len = 0; }
  zero_hist(hist);

  bool done = false;
  if (CAND && k < n) {   // never with map / all_slots; k >= n: every element is selected below
    const int ranges_row = (row_len + rlen - 1) / rlen;
    done = topk_from_candidates(pre + row * ranges_row * kSegInts, (n + rlen - 1) / rlen, k, sel,
                                lkey, lidx, hist, scan_scratch, thr, &list_len);
  }

  if (!done) {
  if (!(CAND && k >= n)) {
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
      scan_row(s, 0, n, [&](int i, float v, bool in) {
        const uint32_t key = order_key(v), a = key >> 21;
        if (in && a > d1) atomicOr(&sel[i >> 5], 1u << (i & 31));
        const int b = wave_append(in && a == d1, &list_len);
        if (b >= 0) { lkey[b] = key; lidx[b] = i; }
      });
      __syncthreads();
      const int len = list_len;
      // ---- digits 2 and 3 on the list
      for (int i = tid; i < len; i += kTopkThreads) atomicAdd(&hist[(lkey[i] >> 10) & 0x7FF], 1);
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t p22 = (d1 << 11) | (uint32_t)thr[0];
      need = thr[1];
      const int nb = thr[2];
      if (nb <= kFew) {
        // ---- few list entries share the second threshold digit (the usual case): they are
        //      ranked against each other by score, then index, instead of a third digit pass
        for (int i = tid; i < len; i += kTopkThreads) {
          const uint32_t key = lkey[i], kp = key >> 10;
          if (kp > p22) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
          const int b = wave_append(kp == p22, &few_len);
          if (b >= 0) { fkey[b] = key; fidx[b] = lidx[i]; }
        }
        __syncthreads();
        if (tid < nb) {
          const uint32_t key = fkey[tid];
          const int e = fidx[tid];
          int rank = 0;
          for (int j = 0; j < nb; ++j) {
            const uint32_t kj = fkey[j];
            rank += (kj > key || (kj == key && fidx[j] < e)) ? 1 : 0;
          }
          if (rank < need) atomicOr(&sel[e >> 5], 1u << (e & 31));
        }
      } else {
      __syncthreads();
      zero_hist(hist);
      for (int i = tid; i < len; i += kTopkThreads) {
        const uint32_t key = lkey[i], kp = key >> 10;
        if (kp > p22) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
        else if (kp == p22) atomicAdd(&hist[key & 0x3FF], 1);
      }
      __syncthreads();
      find_threshold_bin(hist, need, scan_scratch, thr);
      const uint32_t tkey = (p22 << 10) | (uint32_t)thr[0];
      need = thr[1];
      const int ties = thr[2];
      __syncthreads();
      zero_hist(hist);
      if (ties == need) {
        for (int i = tid; i < len; i += kTopkThreads)
          if (lkey[i] >= tkey) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
      } else {
        // More ties than places: take the `need` lowest indices among them, by the
        // same digit search on (high, low) halves of the index, inverted so that a
        // lower index ranks higher.  Indices are distinct, so this is exact.
        for (int i = tid; i < len; i += kTopkThreads) {
          const uint32_t key = lkey[i];
          if (key > tkey) atomicOr(&sel[lidx[i] >> 5], 1u << (lidx[i] & 31));
          else if (key == tkey) atomicAdd(&hist[kBins - 1 - (lidx[i] >> 10)], 1);
        }
        __syncthreads();
        find_threshold_bin(hist, need, scan_scratch, thr);
        const int hi_digit = kBins - 1 - thr[0];
        need = thr[1];
        __syncthreads();
        zero_hist(hist);
        for (int i = tid; i < len; i += kTopkThreads) {
          if (lkey[i] != tkey) continue;
          const int e = lidx[i];
          if ((e >> 10) < hi_digit) atomicOr(&sel[e >> 5], 1u << (e & 31));
          else if ((e >> 10) == hi_digit) atomicAdd(&hist[kBins - 1 - (e & 0x3FF)], 1);
        }
        __syncthreads();
        find_threshold_bin(hist, need, scan_scratch, thr);
        const int lo_digit = kBins - 1 - thr[0];
        for (int i = tid; i < len; i += kTopkThreads) {
          if (lkey[i] != tkey) continue;
          const int e = lidx[i];
          if ((e >> 10) == hi_digit && (e & 0x3FF) <= lo_digit) atomicOr(&sel[e >> 5], 1u << (e & 31));
        }
      }
      }  // more than kFew entries in the second digit
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

  }  // !done

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

template <bool CAND>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(Prob p, const float* __restrict__ S,
                                                            int row_len, int k,
                                                            const int* __restrict__ map,
                                                            int* __restrict__ idx,
                                                            float* __restrict__ val,
                                                            const int* __restrict__ pre, int rlen,
                                                            bool all_slots) {
  extern __shared__ uint32_t dyn[];
  // queries in descending order: under a causal mask the late ones have the longest rows, and
  // the workgroups with the most work should start first
  topk_row<CAND>(p, S, row_len, k, map, idx, val, pre, rlen, gridDim.x - 1 - blockIdx.x, blockIdx.y, dyn, all_slots);
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
    topk_row<false>(p, S, p.L, k, nullptr, idx, val, nullptr, 0, r % p.n_q, r / p.n_q, dyn);
    __syncthreads();
  }
}

// Rows are split over several workgroups when there are too few of them to fill the chip.
static bool use_split(const Prob& p) {
  return (long long)p.n_seq * p.n_q < 256 && p.L >= 4 * kMinRange;
}

size_t topk_ws_bytes(const Prob& p, int k) {
  if (!use_split(p) || k < 1) return 0;
  const int rlen = range_len(p.L);
  const size_t ranges = (size_t)(p.L + rlen - 1) / rlen;
  return (size_t)p.n_seq * p.n_q * ranges * kSegInts * sizeof(int);
}

template <int WHICH>  // 0: topk_kernel<false>, 1: topk_kernel<true>, 2: topk_only_kernel
static hipError_t set_lds_limit(size_t lds) {
  static LdsSeen seen;
  const void* f = WHICH == 0 ? reinterpret_cast<const void*>(topk_kernel<false>)
                : WHICH == 1 ? reinterpret_cast<const void*>(topk_kernel<true>)
                             : reinterpret_cast<const void*>(topk_only_kernel);
  return ensure_dynamic_lds(f, lds, seen);
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
    const int rlen = range_len(p.L);
    const dim3 g2((p.L + rlen - 1) / rlen, p.n_q, p.n_seq);
    hipError_t e = set_lds_limit<1>(lds);   // before the first launch: a failure leaves nothing enqueued
    if (e != hipSuccess) return e;
    topk_prefilter_kernel<<<g2, kTopkThreads, 0, st>>>(p, S, k, rlen, pre);
    topk_kernel<true><<<grid, kTopkThreads, lds, st>>>(p, S, row_len, k, map, idx, val, pre, rlen, false);
    return hipGetLastError();
  }
  hipError_t e = set_lds_limit<0>(lds);
  if (e != hipSuccess) return e;
  topk_kernel<false><<<grid, kTopkThreads, lds, st>>>(p, S, row_len, k, map, idx, val, nullptr, 0, all_slots);
  return hipGetLastError();
}

}  // namespace misa
