// Exact top-k of one short row (at most 8192 scores) that already sits in LDS, by the 256
// threads of a workgroup: the tail of the fused re-rank kernel (Eq. misa_final_topk), where the
// dense scores of a query's candidates never leave the workgroup that computed them.
//
// Same result as topk_kernel in map mode, bit for bit: -inf (skipped candidates) is never
// selected, the k largest of the rest are, ties go to the lower position, positions come out in
// ascending order and unused output slots hold -1 / -inf.
//
// Method: thread t owns positions t, t + 256, ... (32 of them) and keeps their keys
// (order-preserving integer images) in registers.  One
// 2047-bin digit, linear in the key over [lo, max] (keys below lo share bin 0 and are counted in
// registers), is counted in LDS; everything above the bin that holds the k-th largest is
// selected, everything below it dropped, and the bin itself is either taken whole, ranked by
// brute force (at most 64 entries), or refined by the next pass over its own key range.  lo
// starts four binades below the row maximum, which is where the k-th largest of a few thousand
// scores normally lies; after two passes that ended in the catch-all bin lo is the row minimum,
// and from there the range shrinks 2048-fold per pass until all live keys are equal (ties: the
// lowest positions win, by a bitmap walk).  The loops over a thread's elements are free of
// branches, so that their LDS reads and atomics are issued back to back.
#pragma once

#include "radix.h"

namespace misa {

constexpr int kSmallTopkThreads = 256;
constexpr int kSmallTopkMax = 8192;                                  // scores per row
constexpr int kSmallTopkEpt = kSmallTopkMax / kSmallTopkThreads;     // 32 per thread
constexpr int kSmallTopkWords = kSmallTopkMax / 32;                  // bitmap words: one per thread
constexpr int kSmallTopkFew = 64;    // brute-force ranking up to here (256 measured 20 us slower on 2048 rows of 8192)

struct SmallTopkLds {
  int hist[kBins];
  uint32_t sel[kSmallTopkWords];
  uint32_t eq[kSmallTopkWords];
  int wpre[kSmallTopkWords];         // selected positions in the bitmap words before a word
  uint2 few[kSmallTopkFew];          // (key, position) of the entries of the threshold bin
  int few_rank[kSmallTopkFew];       // entries of that list that rank before an entry
  int scan[32];
  int thr[4];
  uint32_t red[3 * 4];
  int few_len;
};

// sc[0 .. n): the bit patterns of the row's scores in LDS (complete: the caller has passed a
// barrier); n <= 8192.
// map[0 .. n): global; out_idx[j] = map[position] for the selected positions in ascending order.
// All 256 threads call this; it contains barriers.
__device__ __forceinline__ void small_row_topk(const int* sc, int n, int k, const int* __restrict__ map,
                                               int* __restrict__ out_idx, float* __restrict__ out_val,
                                               SmallTopkLds& L) {
  constexpr int NT = kSmallTopkThreads, EPT = kSmallTopkEpt;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  uint32_t key[EPT];
  uint32_t act = 0;        // bit u: element tid + NT u can still be selected and is undecided
  uint32_t kmax = 0, kmin = 0xFFFFFFFFu;
#pragma unroll
  for (int u = 0; u < EPT; ++u) key[u] = order_key(__int_as_float(sc[min(tid + NT * u, n - 1)]));
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const bool ok = tid + NT * u < n && key[u] > kKeyNegInf;
    act |= ok ? 1u << u : 0u;
    kmax = max(kmax, ok ? key[u] : 0u);
    kmin = min(kmin, ok ? key[u] : 0xFFFFFFFFu);
  }
  int selectable = __popc(act);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    selectable += __shfl_xor(selectable, off);
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
  }
  if (lane == 0) { L.red[wave] = (uint32_t)selectable; L.red[4 + wave] = kmax; L.red[8 + wave] = kmin; }
  if (tid == 0) L.few_len = 0;
  if (tid < kSmallTopkFew) {
    L.few[tid] = make_uint2(0u, 0u);   // padding of the brute-force list: key 0 ranks below every live key
    L.few_rank[tid] = 0;
  }
  __syncthreads();
  selectable = (int)(L.red[0] + L.red[1] + L.red[2] + L.red[3]);
  kmax = max(max(L.red[4], L.red[5]), max(L.red[6], L.red[7]));
  kmin = min(min(L.red[8], L.red[9]), min(L.red[10], L.red[11]));

  const int k_eff = min(k, selectable);
  for (int i = k_eff + tid; i < k; i += NT) {
    out_idx[i] = -1;
    if (out_val) out_val[i] = -INFINITY;
  }
  if (k_eff == 0) return;

  enum { kDone, kBrute, kTies };
  int mode = kDone;
  int need = k_eff, nb = selectable;   // nb: live elements
  uint32_t chosen = 0;
  if (k_eff == selectable) {
    chosen = act;
  } else {
    for (int pass = 0;; ++pass) {      // every quantity that steers the loop is uniform over the block
      if (nb <= kSmallTopkFew) { mode = kBrute; break; }
      if (kmax == kmin) { mode = kTies; break; }               // all live keys are equal
      const uint32_t lo = (pass < 2 && kmax - kmin > (1u << 25)) ? kmax - (1u << 25) : kmin;
      const uint32_t span = kmax - lo;
      int shift = max(0, 32 - __clz((int)span) - 11);
      if ((span >> shift) > (uint32_t)(kBins - 2)) ++shift;      // bins 1 .. 2047 cover [lo, kmax]
      zero_hist_n<NT>(L.hist);
      int below = 0;                   // live elements under lo: counted in registers, not by LDS atomics
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const bool live = (act >> u) & 1u;
        const bool in = live && key[u] >= lo;
        below += (int)live - (int)in;
        if (in) atomicAdd(&L.hist[(int)((key[u] - lo) >> shift) + 1], 1);
      }
      below = wave_inclusive_scan(below);
      if (lane == 63 && below) atomicAdd(&L.hist[0], below);
      __syncthreads();
      find_threshold_bin_n<NT>(L.hist, need, L.scan, L.thr);
      const int b = L.thr[0];
      need = L.thr[1];
      nb = L.thr[2];
#pragma unroll
      for (int u = 0; u < EPT; ++u) {
        const int d = key[u] < lo ? 0 : (int)((key[u] - lo) >> shift) + 1;
        const uint32_t bit = act & (1u << u);
        chosen |= d > b ? bit : 0u;
        act &= d == b ? ~0u : ~bit;
      }
      if (nb == need) { chosen |= act; break; }
      if (b > 0) {
        kmin = lo + ((uint32_t)(b - 1) << shift);
        kmax = min(kmax, kmin + ((1u << shift) - 1u));
      } else {
        kmax = lo - 1u;                                         // (lo > kmin here: bin 0 was not empty)
      }
      __syncthreads();                                          // thr is rewritten by the next pass
    }
  }

  // ---- the selected positions as a bitmap: element tid + NT u is bit (tid & 31) of word 2 wave + 8 u (+ 1)
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const unsigned long long m = __ballot((chosen >> u) & 1u);
    if (lane == 0) {
      L.sel[2 * wave + 8 * u] = (uint32_t)m;
      L.sel[2 * wave + 8 * u + 1] = (uint32_t)(m >> 32);
    }
    if (mode == kTies) {
      const unsigned long long e = __ballot((act >> u) & 1u);
      if (lane == 0) {
        L.eq[2 * wave + 8 * u] = (uint32_t)e;
        L.eq[2 * wave + 8 * u + 1] = (uint32_t)(e >> 32);
      }
    }
  }
  if (mode == kBrute) {
    // the (at most 64) live entries, listed by the few threads that own one
    for (uint32_t a = act; a; a &= a - 1) {
      const int i = tid + NT * (__ffs(a) - 1);
      const int slot = atomicAdd(&L.few_len, 1);
      if (slot < kSmallTopkFew) L.few[slot] = make_uint2(order_key(__int_as_float(sc[i])), (uint32_t)i);
    }
  }
  __syncthreads();
  if (mode == kBrute) {
    // the nb entries of the threshold bin, ranked by score, then position: all pairs, thread t
    // comparing entry t % 64 with a quarter of the list (padded with entries that rank below all)
    {
      constexpr int JP = kSmallTopkFew / (NT / 64);
      const int i = tid & 63, j0 = (tid >> 6) * JP;
      const uint2 mine = L.few[i];
      int part = 0;
#pragma unroll
      for (int j = j0; j < j0 + JP; ++j) {
        const uint2 o = L.few[j];
        part += (o.x > mine.x || (o.x == mine.x && o.y < mine.y)) ? 1 : 0;
      }
      if (part) atomicAdd(&L.few_rank[i], part);
    }
    __syncthreads();
    if (tid < nb && L.few_rank[tid] < need) {
      const uint32_t e = L.few[tid].y;
      atomicOr(&L.sel[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
  } else if (mode == kTies) {
    // more equal scores than places: the `need` lowest positions among them
    const uint32_t bits0 = L.eq[tid];
    int total;
    int before = block_exclusive_scan(__popc(bits0), L.scan, &total);
    uint32_t bits = bits0, kept = 0;
    while (bits && before < need) {
      const uint32_t low = bits & (0u - bits);
      kept |= low;
      bits ^= low;
      ++before;
    }
    L.sel[tid] |= kept;          // a word is owned by one thread here
    __syncthreads();
  }

  // ---- output in position order: slot of a selected position = selected positions before it
  //      = those of the bitmap words before its word (prefix sums, one word per thread) + the lower
  //      bits of its word.  Every thread goes back to its own positions t, t + 256, ..., so that the
  //      map entries are read coalesced and all at once.
  int mapped[EPT];
#pragma unroll
  for (int u = 0; u < EPT; ++u) mapped[u] = map[min(tid + NT * u, n - 1)];
  {
    int total;
    const int before = block_exclusive_scan(__popc(L.sel[tid]), L.scan, &total);
    L.wpre[tid] = before;
  }
  __syncthreads();
  const uint32_t below = (1u << (tid & 31)) - 1u;
#pragma unroll
  for (int u = 0; u < EPT; ++u) {
    const int w = (tid >> 5) + 8 * u;
    const uint32_t word = L.sel[w];
    const int pos = L.wpre[w] + __popc(word & below);
    if (((word >> (tid & 31)) & 1u) && pos < k) {   // pos < k: always true when the selection is consistent
      out_idx[pos] = mapped[u];
      if (out_val) out_val[pos] = __int_as_float(sc[tid + NT * u]);
    }
  }
}

}  // namespace misa
