// Stage 2: block-pooled head router (Eq. misa_route_score, Eq. misa_route).
//
// route_tile_kernel (bf16 queries): the [queries x heads, 128] x [128, blocks]
// product runs on the matrix core.  Query-head rows are the stationary operand
// (registers); the fp32 pooled keys stream through LDS as two bf16 tiles, the
// bf16 nearest to each value and the bf16 nearest to the exact remainder, and
// both are multiplied, so the products carry the pooled key to 2^-17 relative.  ReLU, the causal
// block mask and the sum over blocks stay in accumulator lanes until the end
// of the block range, when one wavefront reduction per row writes the partial
// sum to the workspace.
// route_partial_kernel (fp32 queries): lane = head.  Each lane keeps its query head in
// registers; the pooled key of the block being visited is the same for the
// whole wavefront, so it is fetched with wave-uniform (scalar) loads and every
// FMA takes one scalar and one vector operand.  The four wavefronts of a
// workgroup stride over the blocks of one split of the prefix; partial sums of
// ReLU(q.k~) go to the workspace.
// route_finalize_kernel: adds the causal tail block (mean of the raw keys of
// the last, partial block of a query that does not sit at the end of the
// cache), scales by |w| / M_n and selects the top-h heads by rank counting.
#include <algorithm>

#include "kernels.h"

namespace misa {

template <int QDT>
__device__ __forceinline__ void load_query_head(const void* Q, size_t head_index, float* qv) {
  using V = Vec16<QDT>;
  const char* src = static_cast<const char*>(Q) + head_index * V::ROW_BYTES;
#pragma unroll
  for (int c = 0; c < kD / V::N; ++c) V::load(src + c * 16, qv + c * V::N);
}

// Two fp32 values -> two packed bf16 pairs whose sums represent them to 2^-17 relative: hi is
// the bf16 nearest to the value, lo the bf16 nearest to the (exactly computed) remainder.
// Element 0 sits in the low half of each word.
typedef __bf16 bf16x2_r __attribute__((ext_vector_type(2)));
typedef float f32x2_r __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  union { bf16x2_r b; uint32_t u; } h, l;
  const f32x2_r v = {x0, x1};
  h.b = __builtin_convertvector(v, bf16x2_r);
  const f32x2_r r = {x0 - __uint_as_float(h.u << 16), x1 - __uint_as_float(h.u & 0xFFFF0000u)};
  l.b = __builtin_convertvector(r, bf16x2_r);
  hi = h.u;
  lo = l.u;
}

// Blocks whose pooled key in Kp is valid for a query with prefix n: all
// ceil(n/B) when the query sits at the end of the cache (the partial block in
// Kp then holds exactly its tokens), else only the complete ones.
__device__ __forceinline__ int pooled_blocks(int n, int len, int B) {
  const int full = n / B;
  return full + ((n == len && full * B != n) ? 1 : 0);
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

constexpr int kRouteKT = 32;  // pooled blocks per LDS tile

union RFrag {
  bf16x8 v;
  uint4 u;
};

// RG wavefronts of a workgroup own different 64-row groups; the other 4 / RG
// "phases" take every (4 / RG)-th block tile of the same rows.
template <int RG>
__global__ __launch_bounds__(256) void route_tile_kernel(Prob p, int splits,
                                                         const uint16_t* __restrict__ Q,
                                                         const float* __restrict__ Kp,
                                                         float* __restrict__ part) {
  constexpr int CP = 4 / RG;
  __shared__ uint2 tile[2][2][kRouteKT * 32];  // [buffer][hi | lo][block row * 32 + 8-byte slot]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, hf = lane >> 5;
  const int split = blockIdx.x, seq = blockIdx.z;
  const int rg = wave % RG, phase = wave / RG;
  const int rows_per_seq = p.n_q * p.H;
  const int row0 = (blockIdx.y * RG + rg) * 64;  // first (query, head) row of this wavefront
  const int len = seq_length(p, seq);

  const int per = (p.M + splits - 1) / splits;
  const int b_lo = split * per, b_hi = min(b_lo + per, p.M);

  // stationary operand
  RFrag a[2][8];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int row = row0 + rt * 32 + col;
    const uint16_t* src = Q + ((size_t)seq * rows_per_seq + min(row, rows_per_seq - 1)) * kD + hf * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + ks * 16);
      a[rt][ks].u = row < rows_per_seq ? v : make_uint4(0, 0, 0, 0);
    }
  }
  // per row of the wavefront, the number of pooled blocks it may use (its own prefix, cut at
  // the end of this split); kept in LDS because only tiles on the causal edge need it
  __shared__ int s_nb[4][64];
  int nb_lane = 0;
  {
    const int rr = row0 + lane;
    if (rr < rows_per_seq) nb_lane = min(pooled_blocks(visible(p, seq, rr / p.H), len, p.B), b_hi);
    s_nb[wave][lane] = nb_lane;
  }
  int nb_max = nb_lane, nb_min = nb_lane;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    nb_max = max(nb_max, __shfl_xor(nb_max, o));
    nb_min = min(nb_min, __shfl_xor(nb_min, o));
  }
  // tiles that end at or before this limit are visible in full to every row of the wavefront
  const int b_full = __builtin_amdgcn_readfirstlane(nb_min);
  // the block range this workgroup must visit: up to the largest count of any of its rows
  __shared__ int s_stop;
  if (tid == 0) s_stop = 0;
  __syncthreads();
  if (lane == 0) atomicMax(&s_stop, nb_max);
  __syncthreads();
  const int b_stop = s_stop;

  const float* kp_seq = Kp + (size_t)seq * p.M * kD;
  float4 stage[2][4];  // two sets: with CP == 1 tiles are requested two iterations ahead
  auto load_tile = [&](int b0, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + 256 * i;               // float4 index inside the 32 x 128 tile
      const int row = e >> 5;
      stage[SET][i] = *reinterpret_cast<const float4*>(kp_seq + (size_t)min(b0 + row, p.M - 1) * kD + (e & 31) * 4);
    }
  };
  auto store_tile = [&](int buf, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + 256 * i;
      const int row = e >> 5, c4 = e & 31;        // c4: group of 4 components
      const float x[4] = {stage[SET][i].x, stage[SET][i].y, stage[SET][i].z, stage[SET][i].w};
      uint32_t hi[2], lo[2];
      split_pair(x[0], x[1], hi[0], lo[0]);
      split_pair(x[2], x[3], hi[1], lo[1]);
      // 16-byte chunk c4 / 2 of the row, XOR-swizzled by the row; 8-byte half c4 & 1
      const int slot = row * 32 + (((c4 >> 1) ^ (row & 15)) << 1) + (c4 & 1);
      tile[buf][0][slot] = make_uint2(hi[0], hi[1]);
      tile[buf][1][slot] = make_uint2(lo[0], lo[1]);
    }
  };

  float sum[2][16];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum[rt][r] = 0.f;

  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;
  int buf = 0;
  if (b_lo < b_stop) {
    load_tile(b_lo, Set1{});
    store_tile(0, Set1{});
    if (CP == 1) load_tile(b_lo + kRouteKT, Set0{});  // staged during the first iteration
  }
  __builtin_amdgcn_s_waitcnt(0);  // prologue loads have landed; in-loop waits concern only loop loads
  __syncthreads();
  int it = 0;
  // One iteration.  CP == 1: the set named by set_tag holds the next tile (requested an iteration
  // ago) and is staged between the matrix instructions, the tile after it is requested into the
  // other set.  Otherwise one set is loaded at the top and staged at the bottom.  Tiles past the
  // last are requested and staged too, with clamped addresses (never read): the body stays one
  // scheduling region.
  auto iteration = [&](int b0, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
    if (CP == 1) load_tile(b0 + 2 * kRouteKT, std::integral_constant<int, SET ^ 1>{});
    else load_tile(b0 + kRouteKT, Set0{});
    if (it % CP == phase) {
      f32x16 acc[2];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rt][r] = 0.f;
      const uint4* hi_t = reinterpret_cast<const uint4*>(tile[buf][0]);
      const uint4* lo_t = reinterpret_cast<const uint4*>(tile[buf][1]);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        RFrag bh, bl;
        const int idx = col * 16 + ((ks * 2 + hf) ^ (col & 15));
        bh.u = hi_t[idx];
        bl.u = lo_t[idx];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, bh.v, acc[rt], 0, 0, 0);
          acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, bl.v, acc[rt], 0, 0, 0);
        }
      }
      if (CP == 1) {
        // staging the next tile (split into pieces, LDS writes) needs nothing from these matrix
        // instructions and its data arrived an iteration ago: it sits in the same scheduling
        // region, ahead of the sums that have to wait for them
        store_tile(buf ^ 1, set_tag);
      }
      if (b0 + kRouteKT <= b_full) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int r = 0; r < 16; ++r) sum[rt][r] += relu(acc[rt][r]);
      } else {
        const int b = b0 + col;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int4 nb = *reinterpret_cast<const int4*>(&s_nb[wave][rt * 32 + 8 * g + 4 * hf]);
            sum[rt][4 * g + 0] += b < nb.x ? relu(acc[rt][4 * g + 0]) : 0.f;
            sum[rt][4 * g + 1] += b < nb.y ? relu(acc[rt][4 * g + 1]) : 0.f;
            sum[rt][4 * g + 2] += b < nb.z ? relu(acc[rt][4 * g + 2]) : 0.f;
            sum[rt][4 * g + 3] += b < nb.w ? relu(acc[rt][4 * g + 3]) : 0.f;
          }
      }
    }
    if (CP != 1) store_tile(buf ^ 1, Set0{});
    __syncthreads();
    buf ^= 1;
    ++it;
  };
  for (int b0 = b_lo; b0 < b_stop;) {
    iteration(b0, Set0{});
    b0 += kRouteKT;
    if (b0 >= b_stop) break;
    if (CP == 1) iteration(b0, Set1{}); else iteration(b0, Set0{});
    b0 += kRouteKT;
  }

  // sum over the 32 block columns of each half-wave, then one lane per row writes
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = sum[rt][r];
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) v += __shfl_xor(v, o);
      const int rr = row0 + rt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      if (col == 0 && rr < rows_per_seq) {
        const int t = rr / p.H, j = rr % p.H;
        part[(((size_t)seq * p.n_q + t) * (splits * CP) + split * CP + phase) * kWave + j] = v;
      }
    }
}

// Few query-head rows (decode: n_q * H <= 64): every wavefront works alone on its own tiles
// of 32 pooled blocks, which it loads straight into matrix fragments (a lane reads 32
// contiguous bytes of one pooled key per k-step) and splits into bf16 hi/lo pieces in
// registers: no LDS, no barrier, one round of loads per tile.  RT = 32-row tiles in use.
template <int RT>
__global__ __launch_bounds__(256) void route_wave_kernel(Prob p, int tiles_per_wave, int n_parts,
                                                         const uint16_t* __restrict__ Q,
                                                         const float* __restrict__ Kp,
                                                         float* __restrict__ part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hf = lane >> 5;
  const int seq = blockIdx.y;
  const int pi = blockIdx.x * 4 + wave;  // partial-sum slot of this wavefront
  if (pi >= n_parts) return;
  const int rows_per_seq = p.n_q * p.H;
  const int len = seq_length(p, seq);
  // row / H for rows < 64 by one multiplication: exact because row * (H * inv - 65536) < 65536
  const uint32_t inv = (65536u + (uint32_t)p.H - 1u) / (uint32_t)p.H;

  RFrag a[RT][8];
  int nb[RT][16];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int row = rt * 32 + col;
    const uint16_t* src = Q + ((size_t)seq * rows_per_seq + min(row, rows_per_seq - 1)) * kD + hf * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + ks * 16);
      a[rt][ks].u = row < rows_per_seq ? v : make_uint4(0, 0, 0, 0);
    }
    int t_prev = -1, nb_prev = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rr = rt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      int v = 0;
      if (rr < rows_per_seq) {
        const int t = (int)(((uint32_t)rr * inv) >> 16);
        if (t != t_prev) { nb_prev = pooled_blocks(visible(p, seq, t), len, p.B); t_prev = t; }
        v = nb_prev;
      }
      nb[rt][r] = v;
    }
  }
  float sum[RT][16];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum[rt][r] = 0.f;

  const float* kp_seq = Kp + (size_t)seq * p.M * kD;
  for (int tl = 0; tl < tiles_per_wave; ++tl) {
    const int b0 = (pi * tiles_per_wave + tl) * kRouteKT;
    if (b0 >= p.M) break;
    const float* src = kp_seq + (size_t)min(b0 + col, p.M - 1) * kD + hf * 8;
    float4 x[8][2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      x[ks][0] = *reinterpret_cast<const float4*>(src + ks * 16);
      x[ks][1] = *reinterpret_cast<const float4*>(src + ks * 16 + 4);
    }
    f32x16 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[rt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const float v[8] = {x[ks][0].x, x[ks][0].y, x[ks][0].z, x[ks][0].w,
                          x[ks][1].x, x[ks][1].y, x[ks][1].z, x[ks][1].w};
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) split_pair(v[2 * j], v[2 * j + 1], hi[j], lo[j]);
      RFrag bh, bl;
      bh.u = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      bl.u = make_uint4(lo[0], lo[1], lo[2], lo[3]);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, bh.v, acc[rt], 0, 0, 0);
        acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt][ks].v, bl.v, acc[rt], 0, 0, 0);
      }
    }
    const int b = b0 + col;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[rt][r] += (b < nb[rt][r] && b < p.M) ? relu(acc[rt][r]) : 0.f;
  }

  // sum over the 32 block columns of each half-wave, then one lane per row writes
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = sum[rt][r];
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) v += __shfl_xor(v, o);
      const int rr = rt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      if (col == 0 && rr < rows_per_seq) {
        const int t = (int)(((uint32_t)rr * inv) >> 16), j = rr - t * p.H;
        part[(((size_t)seq * p.n_q + t) * n_parts + pi) * kWave + j] = v;
      }
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
  __shared__ float sred[4][kMaxH];
  __shared__ float sdot[kMaxH];
  using KV = Vec16<KDT>;
  const int t = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int n = visible(p, seq, t), len = seq_length(p, seq);
  const int nfull = n / p.B, r = n - nfull * p.B;
  const int Mn = nfull + (r > 0 ? 1 : 0);
  const bool tail = r > 0 && n < len;

  if (tail) {  // mean of keys nfull*B .. n-1, component tid
    const char* base = static_cast<const char*>(K);
    auto key_component = [&](int row) {
      const size_t slot = key_slot(p, seq, row);
      const char* src = base + slot * KV::ROW_BYTES;
      if (KDT == MISA_F32) return reinterpret_cast<const float*>(src)[tid];
      if (KDT == MISA_BF16) return bf16_bits_to_float(reinterpret_cast<const uint16_t*>(src)[tid]);
      const uint32_t w = reinterpret_cast<const uint32_t*>(src)[tid >> 2];
      const f32x2 pr = __builtin_amdgcn_cvt_pk_f32_fp8(w >> ((tid & 2) * 8), false);
      return pr[tid & 1] * kscale[slot];
    };
    // rows are added in order; 32 loads are in flight at a time (the workgroup's run time is the
    // latency of these rounds, and a block of 64 has at most two of them)
    float s = 0.f;
    for (int row = nfull * p.B; row < n; row += 32) {
      float v[32];
#pragma unroll
      for (int u = 0; u < 32; ++u) v[u] = key_component(min(row + u, n - 1));
#pragma unroll
      for (int u = 0; u < 32; ++u) s += row + u < n ? v[u] : 0.f;
    }
    tailk[tid] = s / (float)r;
  }
  // Partial sums of the block tiles: the 128 threads form 4 (H <= 32) or 2 groups of one thread
  // per head; group g adds the slots g, g + G, ... in order, eight loads in flight at a time,
  // and the groups' sums are added in group order below.
  {
    const int hp = p.H <= 32 ? 32 : 64, G = 128 / hp, g = tid / hp, j = tid % hp;
    float s = 0.f;
    if (j < p.H) {
      const float* ps = part + ((size_t)seq * p.n_q + t) * splits * kWave + j;
      for (int sp = g; sp < splits; sp += 8 * G) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = sp + u * G < splits ? ps[(size_t)(sp + u * G) * kWave] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
      }
    }
    sred[g][j] = s;
  }
  __syncthreads();

  if (tail) {
    // q_j . (tail mean) for all heads: the query's H rows are one contiguous piece, read in
    // 16-byte chunks in thread order; the CPH consecutive lanes that hold a head's chunks add
    // their partial products with a butterfly, and the first of them keeps the sum.
    using QV = Vec16<QDT>;
    constexpr int CPH = kD / QV::N;  // chunks per head row: 32 (fp32) or 16 (bf16)
    const char* qrow = static_cast<const char*>(Q) + ((size_t)seq * p.n_q + t) * p.H * QV::ROW_BYTES;
    const int total = p.H * CPH, part_of = tid % CPH;
    for (int base = 0; base < total; base += 128) {
      const int c = base + tid;
      float v[QV::N], d = 0.f;
      if (c < total) {
        QV::load(qrow + (size_t)c * 16, v);
#pragma unroll
        for (int e = 0; e < QV::N; ++e) d = fmaf(v[e], tailk[part_of * QV::N + e], d);
      }
#pragma unroll
      for (int o = CPH / 2; o >= 1; o >>= 1) d += __shfl_xor(d, o);
      if (part_of == 0 && c < total) sdot[c / CPH] = d;
    }
    __syncthreads();
  }

  if (tid < p.H) {
    const size_t qi = ((size_t)seq * p.n_q + t) * p.H + tid;
    float s = sred[0][tid] + sred[1][tid];
    if (p.H <= 32) s += sred[2][tid] + sred[3][tid];
    if (tail) s += fmaxf(sdot[tid], 0.f);
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

// Content-free router scores of the routing-score ablation (appendix "Ablation: routing
// score"): kind 1: E_j = w_j, the gate itself; kind 2: E_j = ||q_j||_2.  Same top-h rule.
// One wavefront per query, lane = head.
template <int QDT>
__global__ __launch_bounds__(64) void route_proxy_kernel(Prob p, int kind, const void* __restrict__ Q,
                                                         const float* __restrict__ W,
                                                         int* __restrict__ heads,
                                                         float* __restrict__ E) {
  __shared__ float Es[kWave];
  __shared__ int sel[kWave];
  const int t = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const size_t qi = ((size_t)seq * p.n_q + t) * p.H + tid;
  float e = -INFINITY;
  if (tid < p.H) {
    if (kind == MISA_ROUTER_GATE) {
      e = W[qi];
    } else {
      float qv[kD];
      load_query_head<QDT>(Q, qi, qv);
      float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
      for (int c = 0; c < kD; c += 4) {
        s0 = fmaf(qv[c], qv[c], s0);
        s1 = fmaf(qv[c + 1], qv[c + 1], s1);
        s2 = fmaf(qv[c + 2], qv[c + 2], s2);
        s3 = fmaf(qv[c + 3], qv[c + 3], s3);
      }
      e = sqrtf((s0 + s1) + (s2 + s3));
    }
    if (E) E[qi] = e;
  }
  if (e == 0.f) e = 0.f;  // -0.0 ties with +0.0
  Es[tid] = e;
  __syncthreads();
  int rank = 0;
  for (int i = 0; i < p.H; ++i) {
    const float o = Es[i];
    rank += (o > e || (o == e && i < tid)) ? 1 : 0;
  }
  sel[tid] = (tid < p.H && rank < p.h) ? 1 : 0;
  __syncthreads();
  if (sel[tid]) {
    int pos = 0;
    for (int i = 0; i < tid; ++i) pos += sel[i];
    heads[((size_t)seq * p.n_q + t) * p.h + pos] = tid;
  }
}

hipError_t launch_route_proxy(const Prob& p, int q_dtype, int kind, const void* Q, const float* W,
                              int* heads, float* E, hipStream_t st) {
  const dim3 grid(p.n_q, p.n_seq);
  if (q_dtype == MISA_F32) route_proxy_kernel<MISA_F32><<<grid, 64, 0, st>>>(p, kind, Q, W, heads, E);
  else if (q_dtype == MISA_BF16) route_proxy_kernel<MISA_BF16><<<grid, 64, 0, st>>>(p, kind, Q, W, heads, E);
  else route_proxy_kernel<MISA_FP8_E4M3><<<grid, 64, 0, st>>>(p, kind, Q, W, heads, E);
  return hipGetLastError();
}

// Row groups (of 64 query-head rows) per workgroup of the tiled kernel.
static int route_row_groups(const Prob& p) {
  const long long groups = ((long long)p.n_q * p.H + 63) / 64;
  return groups >= 4 ? 4 : (groups >= 2 ? 2 : 1);
}

int route_splits(const Prob& p) {
  // Enough workgroups to cover the chip, but at least 4 block tiles (128 blocks) per split.
  const long long wgs = (long long)p.n_seq * (((long long)p.n_q * p.H + 255) / 256);
  long long s = (512 + wgs - 1) / wgs;
  const long long cap = (p.M + 127) / 128;
  if (s > cap) s = cap;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return (int)s;
}

// The per-wavefront kernel is used when all (query, head) rows of a sequence fit one wavefront.
static bool route_by_wave(const Prob& p) { return (long long)p.n_q * p.H <= 64; }

// Tiles per wavefront and partial sums per query of the per-wavefront kernel: one tile each
// up to 64 partial sums, more tiles per wavefront beyond.
static void route_wave_shape(const Prob& p, int* tiles_per_wave, int* n_parts) {
  const int tiles = (p.M + kRouteKT - 1) / kRouteKT;
  *tiles_per_wave = (tiles + 63) / 64;
  *n_parts = (tiles + *tiles_per_wave - 1) / *tiles_per_wave;
}

size_t route_ws_bytes(const Prob& p) {
  // partial sums [n_seq, n_q, parts, 64]; the tiled kernel needs room for every column phase
  // (splits * 4), the per-wavefront kernel for its (at most 64) parts
  size_t parts = (size_t)route_splits(p) * 4;
  if (route_by_wave(p)) parts = std::max<size_t>(parts, 64);
  return (size_t)p.n_seq * p.n_q * parts * kWave * sizeof(float);
}

hipError_t launch_route(const Prob& p, int k_dtype, int q_dtype, const void* Q, const float* W,
                        const float* Kp, const void* K, const float* kscale, int* heads, float* E,
                        void* ws, hipStream_t st) {
  const int splits = route_splits(p);
  float* part = static_cast<float*>(ws);
  int total_splits = splits;
  if (q_dtype == MISA_BF16 && route_by_wave(p)) {
    int tpw, parts;
    route_wave_shape(p, &tpw, &parts);
    total_splits = parts;
    const dim3 g1((parts + 3) / 4, p.n_seq);
    const uint16_t* q = static_cast<const uint16_t*>(Q);
    if (p.n_q * p.H <= 32) route_wave_kernel<1><<<g1, 256, 0, st>>>(p, tpw, parts, q, Kp, part);
    else route_wave_kernel<2><<<g1, 256, 0, st>>>(p, tpw, parts, q, Kp, part);
  } else if (q_dtype == MISA_BF16) {
    const int rg = route_row_groups(p);
    total_splits = splits * (4 / rg);
    const int rows = p.n_q * p.H;
    const dim3 g1(splits, (rows + 64 * rg - 1) / (64 * rg), p.n_seq);
    const uint16_t* q = static_cast<const uint16_t*>(Q);
    if (rg == 4) route_tile_kernel<4><<<g1, 256, 0, st>>>(p, splits, q, Kp, part);
    else if (rg == 2) route_tile_kernel<2><<<g1, 256, 0, st>>>(p, splits, q, Kp, part);
    else route_tile_kernel<1><<<g1, 256, 0, st>>>(p, splits, q, Kp, part);
  } else {
    const dim3 g1(splits, p.n_q, p.n_seq);
    route_partial_kernel<MISA_F32><<<g1, 256, 0, st>>>(p, splits, Q, Kp, part);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 g2(p.n_q, p.n_seq);
#define FIN(KD, QD) \
  route_finalize_kernel<KD, QD><<<g2, 128, 0, st>>>(p, total_splits, Q, W, K, kscale, part, heads, E)
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
