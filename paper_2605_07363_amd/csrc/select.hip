// Stages 3 + 4 in one call for many-query (prefill) problems: the indices of the
// k best-scoring visible keys of every query (Eq. misa_score followed by Eq.
// misa_topk; with all heads Eq. dsa_score / Eq. dsa_topk) without writing the
// [rows, L] score matrix to memory and reading it back.
//
//   1. sample    The tile scoring kernel scores one key of every group of 16
//                (1/16 of the work) into a small matrix.
//   2. threshold Per row, the r-th largest sampled score tau is found (radix
//                select, rounded down).  r is a little above k/16, so that with
//                overwhelming probability at least k of all scores reach tau
//                while only about 16 r do.  Rows with few visible keys get
//                tau = -inf (everything is a candidate).
//   3. filter    The tile scoring kernel runs over all keys and writes the
//                (key, score) pairs with score >= tau to per-row lists.  A row's
//                list is cut into one segment per key range of that launch,
//                sized in step 2 from the range's own sampled scores, so every
//                segment has exactly one writer and needs no atomics.
//   4. select    Per row, the exact top-k of the list (ties: lower index) is
//                chosen by radix select in LDS and written in ascending index
//                order.  Since every score >= tau is in the list, the result
//                equals the top-k of the full row whenever the list holds at
//                least k entries and did not overflow.
//   5. repair    Rows for which that does not hold are flagged; the plain path
//                (dense scores of their query tiles, then the row top-k) runs
//                for them only.  Without flagged rows these two launches exit
//                at once.  The result is therefore always exact; the sampling
//                only decides how much work it takes.
//
// Everything is stream-ordered device work: no host read-back, so the call can
// be captured in a HIP graph.
#include <algorithm>
#include <cmath>

#include "kernels.h"
#include "radix.h"

namespace misa {

constexpr int kFusedMaxK = 8192;          // the candidate list of a row is held in registers
constexpr int kFusedMinL = 4096;

// Rank of the sampled threshold: mean k/16 sampled scores lie among the top k; the
// margin covers the sampling noise of that count (more than five standard deviations).
static int sample_rank(int k) {
  const double mu = (double)k / kSampleStride;
  return (int)std::ceil(mu + 6.0 * std::sqrt(mu) + 8.0);
}

// Length of the list segment of a key range in which c sampled scores reached the threshold.
// Exactly one key of every group of 16 is sampled, so with n keys of the range at or above
// the threshold the count of sampled ones has mean n / 16 and variance below n / 16; the
// segment holds 16 c plus six standard deviations of 16 (c - n / 16) at n = 16 (c + 1), plus
// room for a range none of whose ~200 hits was sampled (probability (15/16)^200 < 3e-6) and
// for the unsampled tail group.  Device and host use the same integer formula.
__host__ __device__ inline int segment_length(int c) {
  int root = 0;                                     // ceil(sqrt(c + 1))
  while (root * root < c + 1) ++root;
  return kSampleStride * c + 6 * kSampleStride * root + 128;
}

// At most this many sampled scores may reach the threshold of a row (r do by construction,
// more only through ties at the threshold value); rows with more are left to the repair pass.
static int max_sample_hits(int k) { return sample_rank(k) + sample_rank(k) / 4 + 16; }

// List capacity of a row: the segment lengths add up to at most this (the square roots are
// largest when the sampled hits are spread evenly over the ranges), in units of 256.
static int list_capacity(int k, int ranges) {
  const int hits = max_sample_hits(k);
  const int per = (hits + ranges - 1) / ranges;
  long long c = 0;
  for (int r = 0; r < ranges; ++r) c += segment_length(per) + 6 * kSampleStride;   // (+ one more root: the roots are rounded up)
  return (int)((c + 255) / 256 * 256);
}

static size_t select_lds_bytes(const Prob& p) {
  const size_t nwords = ((size_t)p.L + 31) / 32;
  return nwords * 8;  // selection bitmap and per-word prefix counts
}

// With one or two active heads a quarter or half of all keys score exactly 0 (every active head
// negative); the k-th largest then often lies on that plateau of ties, whose rows the threshold
// filter has to hand to the repair pass, and the two calls are faster (measured with h = 2 on the
// 131072-key prefill: 1.89 ms against 0.97 ms).
static bool fused(const Prob& p, int k_dtype, int q_dtype, int k) {
  return tile_path(p, k_dtype, q_dtype) && k <= kFusedMaxK && p.L >= kFusedMinL && p.h > 2;
}

__device__ __forceinline__ float key_to_float(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

// ---------------------------------------------------------------- threshold
// One workgroup of 256 threads per row: tau[row] = a value at or just below the r-th largest of
// the row's visible sampled scores (the lower edge of its 22-bit radix bin, i.e. within 2^-13
// relative), so at least r samples reach it.  upper[row]: the top key of the first radix digit
// that holds the sampled score of rank r / 4, a robust upper end of the interval in which the
// k-th largest score lies (select_rows_kernel spreads its first digit over [tau, upper]).  The
// first 16 samples of every thread (4096 per row) stay in registers for both digit passes, all
// their loads in flight together; longer rows read the rest again in the second pass.  Also
// clears the row's repair flags and lays out the row's candidate list: seg[row][r] is the offset
// of the segment of key range r (seg[row][ranges] the total), its length segment_length(samples
// of the range that reach tau), cut to the visible keys of the range.  A row whose sampled hits
// exceed max_hits (ties at the threshold value) gets empty segments and so falls to the repair
// pass.  A row all of whose visible keys fit the list keeps every key (tau = -inf, segments =
// the visible keys of each range).
constexpr int kThrThreads = 256;
constexpr int kThrHeld = 16;
__global__ __launch_bounds__(kThrThreads) void select_threshold_kernel(
    Prob p, const float* __restrict__ Ss, int m, int r, int cap, int keep_all, int qwg, int q_tiles, int ranges,
    int keys_per_range, int max_hits, float* __restrict__ tau, uint32_t* __restrict__ upper,
    int* __restrict__ seg, int* __restrict__ row_flag, int* __restrict__ tile_flag) {
  __shared__ int hist[kBins];
  __shared__ int range_hits[64];
  __shared__ int hist2[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ int thr_up[3];
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const int seq = row / p.n_q, t = row % p.n_q;
  const int n = visible(p, seq, t);
  if (tid == 0) {
    row_flag[row] = 0;
    if (t % qwg == 0) tile_flag[seq * q_tiles + t / qwg] = 0;
  }
  int* row_seg = seg + (size_t)row * (ranges + 1);
  if (n <= keep_all) {  // every visible key fits into the list (and into the registers of the row
                        // selection): a range's segment holds its visible keys
    if (tid == 0) { tau[row] = -INFINITY; upper[row] = 0xFFFFFFFFu; }
    if (tid <= ranges) row_seg[tid] = (int)min((long long)n, (long long)tid * keys_per_range);
    return;
  }
  const int ns = n / kSampleStride;  // visible samples; ns > keep_all / 16 >= r
  const float* s = Ss + (size_t)row * m;
  float held[kThrHeld];
#pragma unroll
  for (int u = 0; u < kThrHeld; ++u) {
    const int i = u * kThrThreads + tid;
    held[u] = i < ns ? s[i] : 0.f;
  }
  for (int i = tid; i < kBins; i += kThrThreads) { hist[i] = 0; hist2[i] = 0; }
  __syncthreads();
  auto scan = [&](auto f) {
#pragma unroll
    for (int u = 0; u < kThrHeld; ++u)
      if (u * kThrThreads + tid < ns) f(order_key(held[u]));
    for (int base = kThrHeld * kThrThreads; base < ns; base += 8 * kThrThreads) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * kThrThreads + tid;
        v[u] = i < ns ? s[i] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (base + u * kThrThreads + tid < ns) f(order_key(v[u]));
    }
  };
  scan([&](uint32_t key) { atomicAdd(&hist[key >> 21], 1); });
  __syncthreads();
  find_threshold_bin_n<kThrThreads>(hist, r, scan_scratch, thr, max(r / 4, 1), thr_up);
  const uint32_t d1 = (uint32_t)thr[0];
  const int need = thr[1];
  scan([&](uint32_t key) {
    if ((key >> 21) == d1) atomicAdd(&hist2[(key >> 10) & 0x7FF], 1);
  });
  __syncthreads();
  find_threshold_bin_n<kThrThreads>(hist2, need, scan_scratch, thr);
  const float tau_row = key_to_float((d1 << 21) | ((uint32_t)thr[0] << 10));
  if (tid == 0) {
    tau[row] = tau_row;
    upper[row] = ((uint32_t)thr_up[0] << 21) | 0x1FFFFFu;
  }
  // sampled scores of every key range that reach the threshold (sample i stands for the keys
  // 16 i .. 16 i + 15, and a range is a whole number of such groups)
  if (tid < 64) range_hits[tid] = 0;
  __syncthreads();
  const int groups_per_range = keys_per_range / kSampleStride;
  auto tally = [&](float v, int i) {
    if (v >= tau_row) atomicAdd(&range_hits[i / groups_per_range], 1);
  };
#pragma unroll
  for (int u = 0; u < kThrHeld; ++u)
    if (u * kThrThreads + tid < ns) tally(held[u], u * kThrThreads + tid);
  for (int i = kThrHeld * kThrThreads + tid; i < ns; i += kThrThreads) tally(s[i], i);
  __syncthreads();
  if (tid < 64) {  // one wavefront: segment lengths, their prefix sums
    const int hits = tid < ranges ? range_hits[tid] : 0;
    int total_hits = hits;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) total_hits += __shfl_xor(total_hits, o);
    const long long first_key = (long long)tid * keys_per_range;
    const int visible_here = (int)max(0ll, min((long long)n - first_key, (long long)keys_per_range));
    int len = tid < ranges ? min(segment_length(hits), visible_here) : 0;
    if (total_hits > max_hits) len = 0;          // ties at the threshold: the repair pass takes the row
    int end = wave_inclusive_scan(len);
    if (__shfl(end, 63) > cap) { len = 0; end = 0; }   // cannot happen below max_hits; never lay out past the list
    if (tid < ranges) row_seg[tid] = end - len;
    if (tid == ranges - 1) row_seg[ranges] = end;
  }
}

// ---------------------------------------------------------------- select
// One workgroup of NT threads per row: exact top-k of the row's candidate list.
// Thread t owns list entries t, t + NT, ... (at most EPT of them) and keeps them in
// registers for all passes, so LDS only holds the histogram and the row bitmaps and
// several rows share a compute unit.
template <int NT, int EPT>
__global__ __launch_bounds__(NT) void select_rows_kernel(
    Prob p, const int2* __restrict__ cand, const int* __restrict__ seg, const int* __restrict__ seg_count,
    int ranges, const float* __restrict__ tau, const uint32_t* __restrict__ upper, int cap, int k, int qwg,
    int q_tiles, int* __restrict__ idx, float* __restrict__ val, int* __restrict__ row_flag,
    int* __restrict__ tile_flag) {
  extern __shared__ uint32_t dyn[];  // selection bitmap, then the prefix count of every bitmap word
  __shared__ int hist[kBins];
  __shared__ int scan_scratch[32];
  __shared__ int thr[3];
  __shared__ uint32_t bkey[64];
  __shared__ int bidx[64];
  __shared__ int b_len;
  __shared__ int brank[64];       // entries of the boundary list that rank before an entry
  __shared__ int seg_first[65];   // offset of a range's segment in the row's list
  __shared__ int seg_pre[65];     // entries of the ranges before it (compact numbering of the row's entries)
  __shared__ int seg_bad;
  const int t = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const size_t row = (size_t)seq * p.n_q + t;
  const int n = visible(p, seq, t);
  const int k_eff = min(k, n);
  int* out_idx = idx + row * k;
  float* out_val = val ? val + row * k : nullptr;
  for (int i = k_eff + tid; i < k; i += NT) {
    out_idx[i] = -1;
    if (out_val) out_val[i] = -INFINITY;
  }
  if (k_eff == 0) return;
  // the row's entries: range r holds seg_count[r] of them from seg[r] on; a count above the
  // segment's length means that hits were dropped
  if (tid < 64) {
    int cnt = 0, len = 0, first = 0;
    if (tid < ranges) {
      first = seg[row * (ranges + 1) + tid];
      len = seg[row * (ranges + 1) + tid + 1] - first;
      cnt = seg_count[row * ranges + tid];
    }
    const unsigned long long bad = __ballot(cnt > len);
    const int end = wave_inclusive_scan(cnt);
    seg_first[tid] = first;
    seg_pre[tid] = end - cnt;
    if (tid == 63) { seg_pre[64] = end; seg_bad = bad != 0; }
  }
  __syncthreads();
  const int c = seg_pre[64];
  if (seg_bad || c > NT * EPT || c < k_eff) {  // a segment overflowed, more entries than this kernel holds, or threshold too high: leave the row to the repair pass
    if (tid == 0) {
      row_flag[row] = 1;
      tile_flag[seq * q_tiles + t / qwg] = 1;
    }
    return;
  }
  const int nwords = (n + 31) / 32;
  uint32_t* sel = dyn;
  int* wpre = reinterpret_cast<int*>(dyn + (p.L + 31) / 32);
  // this thread's entries: index (-1 = none) and order-preserving key of the score
  int ei[EPT];
  uint32_t ek[EPT];
  float ev[EPT];
  const int2* src = cand + row * (size_t)cap;
  int rg = 0, rg_begin = 0, rg_end = seg_pre[1];   // the range whose entries [rg_begin, rg_end) hold entry i
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const int i = tid + u * NT;                    // (increasing with u: the range only moves forward)
    int2 e = make_int2(-1, 0);
    if (i < c) {
      while (rg_end <= i) {                        // ends at the latest at range 63: seg_pre[64] = c > i
        ++rg;
        rg_begin = rg_end;
        rg_end = seg_pre[rg + 1];
      }
      e = src[seg_first[rg] + (i - rg_begin)];
    }
    ei[u] = e.x;
    ev[u] = __int_as_float(e.y);
    ek[u] = order_key(ev[u]);
  }
  for (int i = tid; i < nwords; i += NT) sel[i] = 0;
  if (tid == 0) b_len = 0;
  if (tid < 64) brank[tid] = 0;
  zero_hist_n<NT>(hist);  // ends with a barrier
  auto mark = [&](int e) { atomicOr(&sel[e >> 5], 1u << (e & 31)); };

  // Short way: one digit of key - key(tau), scaled so that [tau, upper] fills the 2047 lower
  // values of the digit (larger keys share 2047).  The list entries then spread over the whole
  // histogram instead of piling up in the few bins a raw key prefix gives them; entries above
  // the digit of the k-th largest are selected and the few inside it ranked against each other
  // (score descending, index ascending).  More than 64 entries in that digit, or the catch-all
  // digit: the three raw key digits below decide instead.
  bool done = false;
  if (c != k_eff) {
    const uint32_t klo = order_key(tau[row]);
    const uint32_t up = upper[row];
    const uint32_t span = up > klo ? up - klo : 1u;
    const int sh = __clz(span);
    auto digit = [&](uint32_t key) {
      const uint32_t x = key > klo ? key - klo : 0u;
      return x > span ? (uint32_t)(kBins - 1) : (x << sh) >> 21;
    };
#pragma unroll
    for (int u = 0; u < EPT; ++u)
      if (ei[u] >= 0) atomicAdd(&hist[digit(ek[u])], 1);
    __syncthreads();
    find_threshold_bin_n<NT>(hist, k_eff, scan_scratch, thr);
    const uint32_t d1 = thr[0];
    const int need = thr[1], nb = thr[2];
    if (nb <= 64 && d1 != kBins - 1) {   // block-uniform
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const uint32_t a = ei[u] >= 0 ? digit(ek[u]) : 0u;
        if (ei[u] >= 0 && a > d1) mark(ei[u]);
        const int b = wave_append(ei[u] >= 0 && a == d1, &b_len);
        if (b >= 0) { bkey[b] = ek[u]; bidx[b] = ei[u]; }
      }
      __syncthreads();
      {
        // all pairs of the (at most 64) boundary entries, spread over the block: thread t compares
        // entry t % 64 with its share of the others
        constexpr int JP = 64 / (NT / 64);
        const int i = tid & 63, j0 = (tid >> 6) * JP;
        if (i < nb && j0 < nb) {
          const uint32_t key = bkey[i];
          const int e = bidx[i];
          int part = 0;
#pragma unroll
          for (int j = j0; j < j0 + JP; ++j)
            part += (j < nb && (bkey[j] > key || (bkey[j] == key && bidx[j] < e))) ? 1 : 0;
          if (part) atomicAdd(&brank[i], part);
        }
      }
      __syncthreads();
      if (tid < nb && brank[tid] < need) mark(bidx[tid]);
      done = true;
    } else {
      __syncthreads();
      zero_hist_n<NT>(hist);
    }
  }

  if (c == k_eff) {
#pragma unroll
    for (int u = 0; u < EPT; ++u)
      if (ei[u] >= 0) mark(ei[u]);
  } else if (!done) {
    // most significant digit first: 11 + 11 + 10 bits of the key
#pragma unroll
    for (int u = 0; u < EPT; ++u)
      if (ei[u] >= 0) atomicAdd(&hist[ek[u] >> 21], 1);
    __syncthreads();
    find_threshold_bin_n<NT>(hist, k_eff, scan_scratch, thr);
    const uint32_t d1 = thr[0];
    int need = thr[1];
    __syncthreads();
    zero_hist_n<NT>(hist);
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
      if (ei[u] < 0) continue;
      const uint32_t a = ek[u] >> 21;
      if (a > d1) mark(ei[u]);
      else if (a == d1) atomicAdd(&hist[(ek[u] >> 10) & 0x7FF], 1);
    }
    __syncthreads();
    find_threshold_bin_n<NT>(hist, need, scan_scratch, thr);
    const uint32_t pre22 = (d1 << 11) | (uint32_t)thr[0];
    need = thr[1];
    __syncthreads();
    zero_hist_n<NT>(hist);
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
      if (ei[u] < 0 || (ek[u] >> 21) != d1) continue;
      if ((ek[u] >> 10) > pre22) mark(ei[u]);
      else if ((ek[u] >> 10) == pre22) atomicAdd(&hist[ek[u] & 0x3FF], 1);
    }
    __syncthreads();
    find_threshold_bin_n<NT>(hist, need, scan_scratch, thr);
    const uint32_t tkey = (pre22 << 10) | (uint32_t)thr[0];
    need = thr[1];
    const int ties = thr[2];
    __syncthreads();
    if (ties == need) {
#pragma unroll
      for (int u = 0; u < EPT; ++u)
        if (ei[u] >= 0 && (ek[u] >> 10) == pre22 && ek[u] >= tkey) mark(ei[u]);
    } else {
      // More entries equal to the threshold value than places: the `need` lowest
      // indices among them win, found by the same digit search on the (high, low)
      // halves of the index with the bin order inverted.
      zero_hist_n<NT>(hist);
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        if (ei[u] < 0) continue;
        if ((ek[u] >> 10) == pre22 && ek[u] > tkey) mark(ei[u]);
        else if (ek[u] == tkey) atomicAdd(&hist[kBins - 1 - (ei[u] >> 10)], 1);
      }
      __syncthreads();
      find_threshold_bin_n<NT>(hist, need, scan_scratch, thr);
      const int hi_digit = kBins - 1 - thr[0];
      need = thr[1];
      __syncthreads();
      zero_hist_n<NT>(hist);
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        if (ei[u] < 0 || ek[u] != tkey) continue;
        if ((ei[u] >> 10) < hi_digit) mark(ei[u]);
        else if ((ei[u] >> 10) == hi_digit) atomicAdd(&hist[kBins - 1 - (ei[u] & 0x3FF)], 1);
      }
      __syncthreads();
      find_threshold_bin_n<NT>(hist, need, scan_scratch, thr);
      const int lo_digit = kBins - 1 - thr[0];
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        if (ei[u] < 0 || ek[u] != tkey) continue;
        if ((ei[u] >> 10) == hi_digit && (ei[u] & 0x3FF) <= lo_digit) mark(ei[u]);
      }
    }
  }
  __syncthreads();

  // Output slot of a selected index = number of selected indices below it.
  const int wpt = (nwords + NT - 1) / NT;
  const int w_lo = min(tid * wpt, nwords), w_hi = min(w_lo + wpt, nwords);
  int cnt = 0;
  for (int w = w_lo; w < w_hi; ++w) cnt += __popc(sel[w]);
  int total;
  int pos = block_exclusive_scan(cnt, scan_scratch, &total);
  for (int w = w_lo; w < w_hi; ++w) {
    wpre[w] = pos;
    pos += __popc(sel[w]);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const int e = ei[u];
    if (e < 0) continue;
    const uint32_t bits = sel[e >> 5], bit = 1u << (e & 31);
    if (!(bits & bit)) continue;
    const int slot = wpre[e >> 5] + __popc(bits & (bit - 1u));
    if (slot < k) {  // always true when the selection is consistent
      out_idx[slot] = e;
      if (out_val) out_val[slot] = ev[u];
    }
  }
}

// ---------------------------------------------------------------- host side
namespace {

struct Layout {
  size_t S, sample, tau, upper, row_flag, tile_flag, seg, seg_count, cand, total;
  int m, cap, qwg, q_tiles, ranges, keys_per_range;
};

size_t up(size_t x) { return (x + 255) & ~(size_t)255; }

Layout layout(const Prob& p, bool routed, int k, bool q8 = false) {
  Layout l;
  const size_t rows = (size_t)p.n_seq * p.n_q;
  l.m = p.L / kSampleStride;
  l.ranges = tile_key_ranges(p, routed, q8, kTileFilter, &l.keys_per_range);
  l.cap = list_capacity(k, l.ranges);
  l.qwg = tile_queries_per_wg(p, routed, q8);
  l.q_tiles = (p.n_q + l.qwg - 1) / l.qwg;
  size_t o = 0;
  l.S = o;         o += up(rows * p.L * sizeof(float));
  l.sample = o;    o += up(rows * l.m * sizeof(float));
  l.tau = o;       o += up(rows * sizeof(float));
  l.upper = o;     o += up(rows * sizeof(uint32_t));
  l.row_flag = o;  o += up(rows * sizeof(int));
  l.tile_flag = o; o += up((size_t)p.n_seq * l.q_tiles * sizeof(int));
  l.seg = o;       o += up(rows * (l.ranges + 1) * sizeof(int));
  l.seg_count = o; o += up(rows * l.ranges * sizeof(int));
  l.cand = o;      o += up(rows * l.cap * sizeof(int2));
  l.total = o;
  return l;
}

}  // namespace

size_t select_ws_bytes(const Prob& p, int k_dtype, int q_dtype, int k) {
  if (k < 1) return 0;
  const size_t dense = up((size_t)p.n_seq * p.n_q * p.L * sizeof(float));
  if (!fused(p, k_dtype, q_dtype, k)) return dense + up(topk_ws_bytes(p, k));
  // the number of key ranges, hence the list capacity, and the number of query tiles depend
  // on the head count of the call: room for either kind
  return std::max(layout(p, false, k).total, layout(p, true, k).total);
}

long long select_row_flags_offset(const Prob& p, int k_dtype, int q_dtype, bool routed, int k) {
  if (k < 1 || !fused(p, k_dtype, q_dtype, k)) return -1;
  return (long long)layout(p, routed, k).row_flag;
}

hipError_t launch_select(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                         const int* heads, const void* K, const float* kscale, int k, int* idx,
                         float* val, void* ws, hipStream_t st) {
  char* base = static_cast<char*>(ws);
  if (!fused(p, k_dtype, q_dtype, k)) {
    float* S = reinterpret_cast<float*>(base);
    const size_t dense = up((size_t)p.n_seq * p.n_q * p.L * sizeof(float));
    hipError_t e = launch_score(p, k_dtype, q_dtype, Q, W, heads, K, kscale, nullptr, 0, S, st);
    if (e != hipSuccess) return e;
    return launch_topk(p, S, p.L, k, nullptr, idx, val, base + dense, st);
  }
  const Layout l = layout(p, heads != nullptr, k, q_dtype == MISA_FP8_E4M3);
  float* S = reinterpret_cast<float*>(base + l.S);
  float* Ss = reinterpret_cast<float*>(base + l.sample);
  float* tau = reinterpret_cast<float*>(base + l.tau);
  uint32_t* upper = reinterpret_cast<uint32_t*>(base + l.upper);
  int* seg = reinterpret_cast<int*>(base + l.seg);
  int* seg_count = reinterpret_cast<int*>(base + l.seg_count);
  int* row_flag = reinterpret_cast<int*>(base + l.row_flag);
  int* tile_flag = reinterpret_cast<int*>(base + l.tile_flag);
  int2* cand = reinterpret_cast<int2*>(base + l.cand);
  const dim3 rows(p.n_q, p.n_seq);

  // the row selection holds a row's entries in registers: 512 threads x 10 for up to 5120
  // expected entries (16 r plus six standard deviations), 1024 x 13 above (measured on MI355X);
  // rows with more entries go to the repair pass
  const double rr = sample_rank(k);
  const bool small_rows = kSampleStride * rr * (1.0 + 6.0 / std::sqrt(rr)) <= 5120.0;
  const int entry_limit = small_rows ? 512 * 10 : 1024 * 13;   // k = kFusedMaxK: 13056 expected

  hipError_t e = launch_tile_mode(p, k_dtype, q_dtype, kTileSample, TileAux{}, Q, W, heads, K, kscale, Ss, st);
  if (e != hipSuccess) return e;
  select_threshold_kernel<<<p.n_seq * p.n_q, kThrThreads, 0, st>>>(
      p, Ss, l.m, sample_rank(k), l.cap, std::min(l.cap, entry_limit), l.qwg, l.q_tiles, l.ranges, l.keys_per_range, max_sample_hits(k), tau,
      upper, seg, row_flag, tile_flag);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  TileAux filter;
  filter.tau = tau;
  filter.cand = cand;
  filter.seg = seg;
  filter.seg_count = seg_count;
  filter.cap = l.cap;
  filter.ranges = l.ranges;
  e = launch_tile_mode(p, k_dtype, q_dtype, kTileFilter, filter, Q, W, heads, K, kscale, nullptr, st);
  if (e != hipSuccess) return e;

  const size_t lds = select_lds_bytes(p);  // at most 128 KB (L <= 524288)
#define GO(NT, EPT)                                                                                 \
  do {                                                                                              \
    static LdsSeen seen;                                                                            \
    e = ensure_dynamic_lds(reinterpret_cast<const void*>(select_rows_kernel<NT, EPT>), lds, seen);  \
    if (e != hipSuccess) return e;                                                                  \
    select_rows_kernel<NT, EPT><<<rows, NT, lds, st>>>(p, cand, seg, seg_count, l.ranges, tau, upper, l.cap, k, \
                                                       l.qwg, l.q_tiles, idx, val, row_flag, tile_flag); \
  } while (0)
  if (small_rows) GO(512, 10);
  else GO(1024, 13);
#undef GO
  if ((e = hipGetLastError()) != hipSuccess) return e;

  // repair pass, a no-op unless rows were flagged
  TileAux repair;
  repair.run = tile_flag;
  e = launch_tile_mode(p, k_dtype, q_dtype, kTileStore, repair, Q, W, heads, K, kscale, S, st);
  if (e != hipSuccess) return e;
  return launch_topk(p, S, p.L, k, nullptr, idx, val, nullptr, st, row_flag);
}

}  // namespace misa
