// Host-side launchers of the MISA kernels.  Each returns the hipError_t of its
// launches; arguments were validated by the C ABI layer before.
#pragma once

#include "common.h"

namespace misa {

size_t pool_ws_bytes(const Prob& p);
hipError_t launch_pool(const Prob& p, int k_dtype, const void* K, const float* kscale, float* Kp,
                       void* ws, hipStream_t st);

int route_splits(const Prob& p);
size_t route_ws_bytes(const Prob& p);
hipError_t launch_route(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const float* Kp, const void* K, const float* kscale, int* heads, float* E,
                        void* ws, hipStream_t st);

// Scores of all L keys (cand == nullptr, out = S [n_seq, n_q, L]) or of the
// k_cand listed candidates (out = [n_seq, n_q, k_cand]).
hipError_t launch_score(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const int* heads, const void* K, const float* kscale, const int* cand,
                        int k_cand, float* out, hipStream_t st);

// Top-k of rows of length row_len.  map == nullptr: row r scans its visible
// prefix and reports positions.  map != nullptr (re-rank): row r scans all
// row_len slots, never selects -inf slots and reports map[slot].
constexpr int kMaxTopK = 16384;
constexpr int kMaxRowLen = 524288;
size_t topk_ws_bytes(const Prob& p, int k);
hipError_t launch_topk(const Prob& p, const float* S, int row_len, int k, const int* map, int* idx,
                       float* val, void* ws, hipStream_t st);

}  // namespace misa
