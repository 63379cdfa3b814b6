// Building blocks of the radix select shared by the top-k kernels: 2048-bin
// LDS histograms scanned from the top by a block of 1024 threads, and
// wavefront-aggregated list appends.
#pragma once

#include "common.h"

namespace misa {

constexpr int kTopkThreads = 1024;
constexpr int kBins = 2048;

// Finds the digit d (scanning from the top) with count(digit > d) < need <= count(digit >= d).
// A block of NT threads, the histogram complete; thread i owns the 2048 / NT bins from
// 2047 - i * 2048 / NT downwards.  Writes {d, need - count(digit > d), hist[d]} to out
// (nothing if need exceeds the total).  Uses scan_scratch[16..31] (block_exclusive_scan uses
// the lower half); two barriers, the second at the end.
// need2 > 0: the digit for a second count is searched in the same scan and written to out2.
template <int NT>
__device__ __forceinline__ void find_threshold_bin_n(const int* hist, int need, int* scan_scratch,
                                                     int* out, int need2 = 0, int* out2 = nullptr) {
  constexpr int BPT = kBins / NT, NW = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int top = kBins - 1 - BPT * (int)threadIdx.x;
  int* wave_total = scan_scratch + 16;
  int h[BPT], sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) { h[i] = hist[top - i]; sum += h[i]; }
  const int inc = wave_inclusive_scan(sum);
  if (lane == 63) wave_total[wave] = inc;
  __syncthreads();
  int total;
  int above = waves_before(wave_total, NW, &total) + inc - sum;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    if (above < need && need <= above + h[i]) {
      out[0] = top - i; out[1] = need - above; out[2] = h[i];
    }
    if (need2 > 0 && above < need2 && need2 <= above + h[i]) {
      out2[0] = top - i; out2[1] = need2 - above; out2[2] = h[i];
    }
    above += h[i];
  }
  __syncthreads();
}

__device__ __forceinline__ void find_threshold_bin(const int* hist, int need, int* scan_scratch,
                                                   int* out, int need2 = 0, int* out2 = nullptr) {
  find_threshold_bin_n<kTopkThreads>(hist, need, scan_scratch, out, need2, out2);
}

template <int NT>
__device__ __forceinline__ void zero_hist_n(int* hist) {
  for (int i = threadIdx.x; i < kBins; i += NT) hist[i] = 0;
  __syncthreads();
}

__device__ __forceinline__ void zero_hist(int* hist) { zero_hist_n<kTopkThreads>(hist); }

// Appends the flagged lanes' values to a list whose length counter lives at *counter
// (LDS or global); one atomic per wavefront.  Returns the slot of this lane (or -1).
__device__ __forceinline__ int wave_append(bool flag, int* counter) {
  const unsigned long long mask = __ballot(flag);
  if (mask == 0) return -1;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((long long)mask) - 1;
  int base = 0;
  if (lane == leader) base = atomicAdd(counter, __popcll(mask));
  base = __shfl(base, leader);
  return flag ? base + __popcll(mask & ((1ull << lane) - 1ull)) : -1;
}

}  // namespace misa
