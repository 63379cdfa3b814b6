// Host-side launchers of the MISA kernels.  Each returns the hipError_t of its
// launches; arguments were validated by the C ABI layer before.
#pragma once

#include <algorithm>
#include <atomic>

#include "common.h"

namespace misa {

size_t pool_ws_bytes(const Prob& p);
// from_token != nullptr: only the blocks from the one holding token from_token[seq] to the end
// of each sequence are recomputed (at most max_blocks of them).
hipError_t launch_pool(const Prob& p, int k_dtype, const void* K, const float* kscale, float* Kp,
                       void* ws, hipStream_t st, const int* from_token = nullptr, int max_blocks = 0);

int route_splits(const Prob& p);
size_t route_ws_bytes(const Prob& p);
hipError_t launch_route(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const float* Kp, const void* K, const float* kscale, int* heads, float* E,
                        void* ws, hipStream_t st);

hipError_t launch_route_proxy(const Prob& p, int q_dtype, int kind, const void* Q, const float* W,
                              int* heads, float* E, hipStream_t st);

// Scores of all L keys (cand == nullptr, out = S [n_seq, n_q, L]) or of the
// k_cand listed candidates (out = [n_seq, n_q, k_cand]).
hipError_t launch_score(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const int* heads, const void* K, const float* kscale, const int* cand,
                        int k_cand, float* out, hipStream_t st);

// The whole re-rank of a query (dense scores of its k_cand candidates, Eq. dsa_score, and their
// top-k, Eq. misa_final_topk) in one workgroup, no score matrix: taken when rerank_fused_path says
// so (at least kRerankFusedMinRows queries, k_cand <= 8192, matrix-core types); the results equal
// launch_score + launch_topk(map = cand) bit for bit.
constexpr int kRerankFusedMinRows = 1024;
bool rerank_fused_path(const Prob& p, int k_dtype, int q_dtype, int k_cand);
hipError_t launch_rerank_fused(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                               const void* K, const float* kscale, const int* cand, int k_cand, int k,
                               int* idx, float* val, hipStream_t st);

// The prefill (matrix-core tile) scoring kernel in its three modes; see score.hip.
enum { kTileStore = 0, kTileSample = 1, kTileFilter = 2 };
constexpr int kSampleStride = 16;
struct TileAux {
  const int* run = nullptr;     // store mode: per query tile, 0 = skip the tile (nullptr: run all)
  const float* tau = nullptr;   // filter mode: per-row score threshold
  int2* cand = nullptr;         // filter mode: [rows, cap] (key index, score bits), cut into segments
  const int* seg = nullptr;     // filter mode: [rows, ranges + 1] segment offsets inside a row's list
  int* seg_count = nullptr;     // filter mode: [rows, ranges] hits of a key range (may exceed its segment: overflow)
  int cap = 0;                  // filter mode: list entries per row
  int ranges = 0;               // filter mode: key ranges = workgroups along x of the launch
};
// Key ranges (workgroups along x) and keys per range of the tile kernel's launch in a mode.
int tile_key_ranges(const Prob& p, bool routed, bool q8, int mode, int* keys_per_wg);
bool tile_path(const Prob& p, int k_dtype, int q_dtype);  // launch_score uses the tile kernel
int tile_queries_per_wg(const Prob& p, bool routed, bool q8);  // q8: fp8 query codes (fp8 matrix instruction)
// q_dtype: MISA_BF16, or MISA_FP8_E4M3 (codes, with fp8 keys only: contracted on the fp8 matrix instruction)
hipError_t launch_tile_mode(const Prob& p, int k_dtype, int q_dtype, int mode, const TileAux& aux,
                            const void* Q, const float* W, const int* heads, const void* K,
                            const float* kscale, float* S, hipStream_t st);

// Fused scoring + top-k (scores are not materialised on the common path).
size_t select_ws_bytes(const Prob& p, int k_dtype, int q_dtype, int k);
// Byte offset in the workspace of the per-row int flags (1 = the row was repaired by the
// two-call path) that the last launch_select left, or -1 when the problem is not fused.
long long select_row_flags_offset(const Prob& p, int k_dtype, int q_dtype, bool routed, int k);
hipError_t launch_select(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                         const int* heads, const void* K, const float* kscale, int k, int* idx,
                         float* val, void* ws, hipStream_t st);

// Top-k of rows of length row_len.  map == nullptr: row r scans its visible
// prefix and reports positions.  map != nullptr (re-rank): row r scans all
// row_len slots, never selects -inf slots and reports map[slot].
constexpr int kMaxTopK = 16384;
constexpr int kMaxRowLen = 524288;
size_t topk_ws_bytes(const Prob& p, int k);
// only != nullptr: rows r with only[r] == 0 are left untouched (ws is not needed then).
// all_slots (with map == nullptr): row r scans all row_len slots, never selects -inf slots
// and reports positions.
hipError_t launch_topk(const Prob& p, const float* S, int row_len, int k, const int* map, int* idx,
                       float* val, void* ws, hipStream_t st, const int* only = nullptr,
                       bool all_slots = false);

// HISA and Block-Sparse comparison indexers (hisa.hip); k == 0 selects Block-Sparse.
size_t hisa_ws_bytes(const Prob& p, int m);
hipError_t launch_hisa(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                       const float* Kp, const void* K, const float* kscale, int m, int k, int* blocks,
                       int* idx, float* val, void* ws, hipStream_t st);

// Raises a kernel's dynamic-LDS limit when a launch needs more than any launch before it on the
// current device.  `seen` is the caller's per-kernel record, one entry per device (the only state
// the library keeps besides its error text: atomics, so host threads may call concurrently; a
// lost update only repeats the cheap attribute call).  Devices past the 64th get the attribute
// set on every launch.
using LdsSeen = std::atomic<size_t>[64];
inline hipError_t ensure_dynamic_lds(const void* func, size_t lds, LdsSeen& seen) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && lds <= seen[dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e == hipSuccess && tracked) {
    size_t cur = seen[dev].load(std::memory_order_relaxed);
    while (cur < lds && !seen[dev].compare_exchange_weak(cur, lds, std::memory_order_release)) {}
  }
  return e;
}

// fp8 query codes -> bf16 (convert.hip); n_elems a multiple of 128.
hipError_t launch_widen_queries(const void* q8, void* q16, size_t n_elems, hipStream_t st);

// Probes for the roofline report (peaks.hip).
constexpr int kProbeMfmaFlopsPerWaveIter = 4 * 2 * 32 * 32 * 16;
hipError_t launch_probe_read(const void* buf, size_t bytes, void* sink, hipStream_t st);
// operands: nullptr (constant operands) or 2048 bytes on the device: fragment a, then fragment b, of the 64 lanes
hipError_t launch_probe_mfma(int workgroups, int iters, const void* operands, float* sink, hipStream_t st);

}  // namespace misa
