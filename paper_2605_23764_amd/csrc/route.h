// Routing and Dispatch bookkeeping kernels (paper Section 2.2: routing and
// Dispatch; Section 5.1: tile offsets derived from the routing result at run time).
//
// Three steps, each a device function so that the serialized launches and the
// persistent scheduler run the same code:
//   route_chunk  top-k + softmax for the 64 tokens of a chunk, per-chunk expert histogram
//   scan_all     prefix sums over chunks and experts, counts/offsets, M-tile map
//   rank_chunk   stable row of every local slot, inverse maps
// The permutation is a stable counting sort keyed by expert: rows of one expert
// ascend in token id, so every index is a pure function of the routing result
// (no atomics decide an order).
#pragma once
#include "common.h"

namespace moe {

struct RouteParams {
  const float* logits;   // [T,E]
  int32_t* topk_idx;     // [T,k]
  float* topk_w;         // [T,k]
  int32_t* counts;       // [E_local]
  int32_t* offsets;      // [E_local+1]
  int32_t* row_of;       // [T,k]
  int32_t* token_of;     // [R_max]
  int32_t* slot_of;      // [R_max]
  int32_t* chunk_cnt;    // [n_chunks, E_local]  histogram, then exclusive offsets
  TileMap tiles;
  int T, E, E_local, expert_base, k, n_chunks;
  int BM;        // M-tile row capacity
  int granule;   // an expert's tiles are equal multiples of this (last one takes the remainder)
};

// Monotone map float -> uint32 (larger float = larger key); -0.0 and NaN are
// canonicalised first (-0.0 ties with +0.0, NaN ranks as -inf).
__device__ __forceinline__ uint32_t float_order_key(float v) {
  if (v != v) v = -__builtin_huge_valf();
  if (v == 0.0f) v = 0.0f;
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_from_order_key(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __builtin_bit_cast(float, u);
}

// Wave-wide unsigned maximum through DPP row operations (no LDS traffic): row_shr
// 1/2/4/8 leave each 16-lane row's maximum in its last lane, row_bcast 15 and 31
// carry it across rows, lane 63 ends up with the wave maximum.  0 is the identity.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#define MOE_DPP_MAX(ctrl, row_mask)                                                                          \
  {                                                                                                          \
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, row_mask, 0xf, false);         \
    v = o > v ? o : v;                                                                                       \
  }
  MOE_DPP_MAX(0x111, 0xf)   // row_shr:1
  MOE_DPP_MAX(0x112, 0xf)   // row_shr:2
  MOE_DPP_MAX(0x114, 0xf)   // row_shr:4
  MOE_DPP_MAX(0x118, 0xf)   // row_shr:8
  MOE_DPP_MAX(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
  MOE_DPP_MAX(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef MOE_DPP_MAX
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

constexpr int kRouteTokensPerWave = 4;   // tokens a wave routes at once (independent reduction chains overlap)

// Top-k of kRouteTokensPerWave tokens by one wave.  Lane l holds the logits of
// experts l, l+64, l+128, l+192 as order-preserving 32-bit keys (0 = taken or
// absent).  Each round takes the wave maximum and, among the lanes that hold it,
// the lowest expert id: ids grow with the register index first, then with the
// lane, so the first register whose ballot is non-empty and its lowest set lane
// win.  Lane j < k ends up holding slot j.
__device__ __forceinline__ void route_tokens(const RouteParams& p, int t_first, int lane, int32_t* s_idx_first) {
  constexpr int Q = kRouteTokensPerWave, PL = kMaxE / kWave;
  uint32_t key[Q][PL];
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int t = min(t_first + q, p.T - 1);   // tokens past the end repeat the last one; results are not stored
    const float* row = p.logits + (size_t)t * p.E;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      const int e = lane + i * kWave;
      key[q][i] = e < p.E ? float_order_key(row[e]) : 0u;
    }
  }
  float my_val[Q];
  int my_idx[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) { my_val[q] = 0.f; my_idx[q] = 0; }
  for (int j = 0; j < p.k; ++j) {
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      uint32_t local = key[q][0];
#pragma unroll
      for (int i = 1; i < PL; ++i) local = key[q][i] > local ? key[q][i] : local;
      const uint32_t best = wave_max_u32(local);
      int win_i = -1, win_lane = 0;
#pragma unroll
      for (int i = PL - 1; i >= 0; --i) {
        const uint64_t b = __ballot(key[q][i] == best);
        if (b != 0) { win_i = i; win_lane = __builtin_ctzll(b); }
      }
#pragma unroll
      for (int i = 0; i < PL; ++i)
        if (i == win_i && lane == win_lane) key[q][i] = 0;
      if (lane == j) {
        my_val[q] = float_from_order_key(best);
        my_idx[q] = win_lane + win_i * kWave;
      }
    }
  }
  // softmax over the k selected logits; slot 0 holds the maximum
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int t = t_first + q;
    const float m = __shfl(my_val[q], 0, kWave);
    const float pj = lane < p.k ? expf(my_val[q] - m) : 0.f;
    float sum = pj;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, kWave);   // k <= 16 lanes hold mass
    sum = __shfl(sum, 0, kWave);
    if (t < p.T && lane < p.k) {
      p.topk_idx[(size_t)t * p.k + lane] = my_idx[q];
      p.topk_w[(size_t)t * p.k + lane] = pj / sum;
      s_idx_first[q * kMaxK + lane] = my_idx[q];
    }
  }
}

// Bitmask of the local experts a token selected, from its k indices.
__device__ __forceinline__ void local_mask(const int32_t* idx, int k, int base, int E_local,
                                           uint64_t mask[kMaskWords]) {
#pragma unroll
  for (int w = 0; w < kMaskWords; ++w) mask[w] = 0;
  for (int j = 0; j < k; ++j) {
    int le = idx[j] - base;
    if (le >= 0 && le < E_local) {
      uint64_t bit = 1ull << (le & 63);
#pragma unroll
      for (int w = 0; w < kMaskWords; ++w)
        if ((le >> 6) == w) mask[w] |= bit;
    }
  }
}

// One chunk of kChunk tokens by a workgroup (16 waves x 4 tokens at 1024 threads),
// then wave 0 (lane = token) builds the chunk's histogram with ballots.
// s_idx: kChunk*kMaxK int32 of LDS.
__device__ __forceinline__ void route_chunk(const RouteParams& p, int chunk, int32_t* s_idx) {
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const int n_waves = blockDim.x / kWave;
  const int t0 = chunk * kChunk;
  for (int i = wave * kRouteTokensPerWave; i < kChunk; i += n_waves * kRouteTokensPerWave)
    if (t0 + i < p.T) route_tokens(p, t0 + i, lane, s_idx + i * kMaxK);
  __syncthreads();
  if (wave == 0) {
    uint64_t mask[kMaskWords];
    int t = t0 + lane;
    local_mask(s_idx + lane * kMaxK, t < p.T ? p.k : 0, p.expert_base, p.E_local, mask);
    int32_t* out = p.chunk_cnt + (size_t)chunk * p.E_local;
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) {
      if (w * 64 >= p.E_local) break;
      int n = min(64, p.E_local - w * 64);
      int cnt = 0;
      for (int b = 0; b < n; ++b) {
        uint64_t bal = __ballot((mask[w] >> b) & 1);
        if (lane == b) cnt = __popcll(bal);
      }
      if (lane < n) out[w * 64 + lane] = cnt;
    }
  }
  __syncthreads();
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

// Rows per expert -> counts, offsets (both optional outputs) and the M-tile map, by
// ONE wave.  cnt may live in LDS or in global memory.
//
// Order of the map: an expert with nt tiles contributes nt/2 sibling pairs; pair j
// sits at entries 2j, 2j+1.  The left-over single tiles of experts with an odd
// count follow, in expert order, and pair up with each other.  Consumers deal pair
// j to XCD j % 8 and run its two tiles side by side on neighbouring CUs, so the
// weight panel both siblings stream is fetched from HBM once and hits in that
// XCD's L2 for the second reader.
__device__ __forceinline__ void build_tile_map(int E_local, const int32_t* cnt, int BM, int granule,
                                               int32_t* counts, int32_t* offsets, const TileMap& tiles) {
  const int lane = lane_id();
  int total_pairs = 0;
  for (int e0 = 0; e0 < E_local; e0 += kWave) {
    const int e = e0 + lane;
    const int c = e < E_local ? cnt[e] : 0;
    const int np_incl = wave_incl_scan(((c + BM - 1) / BM) >> 1, lane);
    total_pairs += __shfl(np_incl, kWave - 1, kWave);
  }
  int row_run = 0, pair_run = 0, single_run = 0;
  for (int e0 = 0; e0 < E_local; e0 += kWave) {
    const int e = e0 + lane;
    const int c = e < E_local ? cnt[e] : 0;
    const int nt = (c + BM - 1) / BM;
    const int np = nt >> 1, ns = nt & 1;
    const int row_incl = wave_incl_scan(c, lane);
    const int pair_incl = wave_incl_scan(np, lane);
    const int single_incl = wave_incl_scan(ns, lane);
    const int off = row_run + row_incl - c;
    const int pbase = pair_run + pair_incl - np;
    const int sbase = single_run + single_incl - ns;
    if (e < E_local) {
      if (counts) counts[e] = c;
      if (offsets) offsets[e] = off;
      // equal split: sibling tiles of an expert take the same time, so they
      // stream the expert's weights in step
      const int per = nt ? (((c + nt - 1) / nt + granule - 1) / granule) * granule : 0;
      for (int i = 0; i < nt; ++i) {
        const int idx = i < 2 * np ? 2 * pbase + i : 2 * total_pairs + sbase;
        tiles.expert[idx] = e;
        tiles.row0[idx] = off + i * per;
        tiles.rows[idx] = min(per, c - i * per);
      }
    }
    row_run += __shfl(row_incl, kWave - 1, kWave);
    pair_run += __shfl(pair_incl, kWave - 1, kWave);
    single_run += __shfl(single_incl, kWave - 1, kWave);
  }
  if (lane == 0) {
    if (offsets) offsets[E_local] = row_run;
    tiles.meta[kMetaMTiles] = 2 * total_pairs + single_run;
    tiles.meta[kMetaRows] = row_run;
    tiles.meta[kMetaStatus] = 0;
  }
}

// Whole-problem scan by ONE workgroup: chunk histograms -> exclusive chunk
// offsets (in place), counts, offsets, M-tile map.  s_cnt: (kMaxE + 2) int32 of LDS.
__device__ __forceinline__ void scan_all(const RouteParams& p, int32_t* s_cnt) {
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const int n_waves = blockDim.x / kWave;
  for (int e = wave; e < p.E_local; e += n_waves) {
    int running = 0;
    for (int c0 = 0; c0 < p.n_chunks; c0 += kWave) {
      int c = c0 + lane;
      int v = c < p.n_chunks ? p.chunk_cnt[(size_t)c * p.E_local + e] : 0;
      int incl = wave_incl_scan(v, lane);
      if (c < p.n_chunks) p.chunk_cnt[(size_t)c * p.E_local + e] = running + incl - v;
      running += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) s_cnt[e] = running;
  }
  __syncthreads();
  if (wave == 0) build_tile_map(p.E_local, s_cnt, p.BM, p.granule, p.counts, p.offsets, p.tiles);
}

// Rows of the local slots of one chunk, by one wave (lane = token):
// row = offsets[e] + (tokens of earlier chunks selecting e) + (earlier lanes selecting e).
__device__ __forceinline__ void rank_chunk(const RouteParams& p, int chunk) {
  const int lane = lane_id();
  const int t = chunk * kChunk + lane;
  const bool live = t < p.T;
  int32_t idx[kMaxK], row[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    idx[j] = (live && j < p.k) ? p.topk_idx[(size_t)t * p.k + j] : -1;
    row[j] = -1;
  }
  uint64_t mask[kMaskWords];
#pragma unroll
  for (int w = 0; w < kMaskWords; ++w) mask[w] = 0;
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    int le = idx[j] - p.expert_base;
    if (idx[j] >= 0 && le >= 0 && le < p.E_local) {
#pragma unroll
      for (int w = 0; w < kMaskWords; ++w)
        if ((le >> 6) == w) mask[w] |= 1ull << (le & 63);
    }
  }
  const int32_t* coff = p.chunk_cnt + (size_t)chunk * p.E_local;
  const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int w = 0; w < kMaskWords; ++w) {
    if (w * 64 >= p.E_local) break;
    const int n = min(64, p.E_local - w * 64);
    // first row of expert w*64+lane for this chunk, fetched once (one coalesced load
    // instead of a dependent load per expert inside the loop)
    const int my_base = lane < n ? p.offsets[w * 64 + lane] + coff[w * 64 + lane] : 0;
    for (int b = 0; b < n; ++b) {
      const bool sel = (mask[w] >> b) & 1;
      const uint64_t bal = __ballot(sel);
      if (bal == 0) continue;
      const int base_row = __builtin_amdgcn_readlane(my_base, b);
      if (sel) {
        const int r = base_row + __popcll(bal & lt);
        const int ge = w * 64 + b + p.expert_base;
        int slot = 0;
#pragma unroll
        for (int j = 0; j < kMaxK; ++j)
          if (idx[j] == ge) { row[j] = r; slot = j; }
        p.token_of[r] = t;
        p.slot_of[r] = slot;
      }
    }
  }
  if (live) {
#pragma unroll
    for (int j = 0; j < kMaxK; ++j)
      if (j < p.k) p.row_of[(size_t)t * p.k + j] = row[j];
  }
}

__global__ __launch_bounds__(1024) void route_kernel(RouteParams p) {
  __shared__ int32_t s_idx[kChunk * kMaxK];
  route_chunk(p, blockIdx.x, s_idx);
}

__global__ __launch_bounds__(1024) void scan_kernel(RouteParams p) {
  __shared__ int32_t s_cnt[kMaxE + 2];
  scan_all(p, s_cnt);
}

__global__ __launch_bounds__(256) void rank_kernel(RouteParams p) {
  int chunk = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (chunk < p.n_chunks) rank_chunk(p, chunk);
}

// M-tile map from the rows per expert alone (the backward rebuilds it from the
// saved counts instead of keeping the forward's workspace alive).
__global__ __launch_bounds__(kWave) void tile_map_kernel(const int32_t* counts, int E_local, int BM, int granule,
                                                         TileMap tiles) {
  build_tile_map(E_local, counts, BM, granule, nullptr, nullptr, tiles);
}

}  // namespace moe
