// Routing and Dispatch bookkeeping kernels (paper Section 2.2: routing and
// Dispatch; Section 5.1: tile offsets derived from the routing result at run time).
//
// Three steps, each a device function:
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
  int32_t* chunk_cnt;    // [n_sub, E_local]  histogram of every 32-token sub-chunk
  TileMap tiles;
  int T, E, E_local, expert_base, k;
  int n_sub;     // ceil(T / kSub) histogram rows
  int n_groups;  // ceil(T / kChunk) rank groups
  int BM;        // M-tile row capacity of the plain wide shape
  int wide_max;  // rows a single wide M tile can take (>= BM: the bf16 kernels feed one more row block per wave row from registers)
  int tall;      // row capacity of a tall M tile (0 = the kernels have no tall shape)
  int granule;   // an expert's rows are dealt to its tiles in units of this many rows
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

// Reductions over the 16 lanes of a DPP row (butterfly: every lane ends up with the
// result): quad_perm [1,0,3,2] and [2,3,0,1], then the 8-lane and 16-lane mirrors.
#define MOE_DPP_ROW_STEPS(OP)  \
  OP(0xB1) OP(0x4E) OP(0x141) OP(0x140)
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v) {
#define MOE_STEP(ctrl)                                                                               \
  {                                                                                                  \
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, 0xf, 0xf, false);      \
    v = o > v ? o : v;                                                                               \
  }
  MOE_DPP_ROW_STEPS(MOE_STEP)
#undef MOE_STEP
  return v;
}
__device__ __forceinline__ float row_sum_f32(float v) {
#define MOE_STEP(ctrl) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, false));
  MOE_DPP_ROW_STEPS(MOE_STEP)
#undef MOE_STEP
  return v;
}
#undef MOE_DPP_ROW_STEPS

constexpr int kHistBatch = 16;             // histogram rows fetched per round trip
constexpr int kRouteTokensPerWave = 4;    // one token per 16-lane row
constexpr int kRouteKeys = kMaxE / 16;    // experts per lane

// Logits of the wave's four tokens as order-preserving keys: lane s of row r holds
// experts 16s .. 16s+15 of token t_first + r (0 = absent).
__device__ __forceinline__ void route_load(const RouteParams& p, int t_first, int lane, uint32_t (&key)[kRouteKeys]) {
  const int t = min(t_first + (lane >> 4), p.T - 1);   // tokens past the end repeat the last one; results are not stored
  const float* row = p.logits + (size_t)t * p.E;
  const int e0 = (lane & 15) * kRouteKeys;
  if ((p.E & 3) == 0) {
#pragma unroll
    for (int i = 0; i < kRouteKeys; i += 4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      const bool in = e0 + i < p.E;
      if (in) v = *reinterpret_cast<const float4*>(row + e0 + i);
      key[i + 0] = in ? float_order_key(v.x) : 0u;
      key[i + 1] = in ? float_order_key(v.y) : 0u;
      key[i + 2] = in ? float_order_key(v.z) : 0u;
      key[i + 3] = in ? float_order_key(v.w) : 0u;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kRouteKeys; ++i) key[i] = e0 + i < p.E ? float_order_key(row[e0 + i]) : 0u;
  }
}

// Top-k of four tokens by one wave, one token per 16-lane row, so every reduction
// step serves four tokens.  Each round: a lane's best remaining key (lowest
// position among equals), the row maximum, the lowest lane of the row that holds
// it (expert ids grow with the lane, then with the position), and that lane
// retires the key and files (id, logit) as slot j in LDS.  Afterwards lane s < k of
// a row picks up slot s and the row computes the softmax over the k selected logits.
// s_idx / s_val: [4][kMaxK] words of LDS for this wave.
__device__ __forceinline__ void route_select(const RouteParams& p, int t_first, int lane, uint32_t (&key)[kRouteKeys],
                                             int32_t* s_idx, float* s_val) {
  const int row = lane >> 4, s = lane & 15;
  for (int j = 0; j < p.k; ++j) {
    uint32_t local = key[0];
    int li = 0;
#pragma unroll
    for (int i = 1; i < kRouteKeys; ++i)
      if (key[i] > local) { local = key[i]; li = i; }
    const uint32_t best = row_max_u32(local);
    const uint64_t bal = __ballot(local == best);
    const uint32_t in_row = (uint32_t)(bal >> (row * 16)) & 0xFFFFu;
    const bool winner = s == __builtin_ctz(in_row);   // in_row != 0: the row maximum is some lane's local maximum
#pragma unroll
    for (int i = 0; i < kRouteKeys; ++i)
      if (winner && i == li) key[i] = 0u;
    if (winner) {
      s_idx[row * kMaxK + j] = s * kRouteKeys + li;
      s_val[row * kMaxK + j] = float_from_order_key(best);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // softmax over the k selected logits; slot 0 holds the maximum
  const int t = t_first + row;
  const bool slot = s < p.k;
  const float val = slot ? s_val[row * kMaxK + s] : 0.f;
  const int idx = slot ? s_idx[row * kMaxK + s] : 0;
  const float m = s_val[row * kMaxK];
  const float pj = slot ? expf(val - m) : 0.f;
  const float sum = row_sum_f32(pj);
  if (t < p.T && slot) {
    p.topk_idx[(size_t)t * p.k + s] = idx;
    p.topk_w[(size_t)t * p.k + s] = pj / sum;
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

// One sub-chunk of kSub tokens by a workgroup (a wave routes four tokens per pass;
// the logits of the next pass are fetched while the current one is selected), then
// wave 0 (lane = token) builds the sub-chunk's histogram row with ballots.
// s_idx, s_val: kSub*kMaxK words of LDS each.
__device__ __forceinline__ void route_chunk(const RouteParams& p, int sub, int32_t* s_idx, float* s_val) {
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const int n_waves = blockDim.x / kWave;
  const int t0 = sub * kSub;
  const int step = n_waves * kRouteTokensPerWave;
  uint32_t key[kRouteKeys], key_next[kRouteKeys];
  int i = wave * kRouteTokensPerWave;
  if (i < kSub && t0 + i < p.T) route_load(p, t0 + i, lane, key);
  for (; i < kSub && t0 + i < p.T; i += step) {
    const bool more = i + step < kSub && t0 + i + step < p.T;
    if (more) route_load(p, t0 + i + step, lane, key_next);
    route_select(p, t0 + i, lane, key, s_idx + i * kMaxK, s_val + i * kMaxK);
#pragma unroll
    for (int q = 0; q < kRouteKeys; ++q) key[q] = key_next[q];
  }
  __syncthreads();
  if (wave == 0) {
    uint64_t mask[kMaskWords];
    const int t = t0 + lane;
    local_mask(s_idx + (lane & (kSub - 1)) * kMaxK, (lane < kSub && t < p.T) ? p.k : 0, p.expert_base, p.E_local, mask);
    int32_t* out = p.chunk_cnt + (size_t)sub * p.E_local;
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

// Inclusive scan across a wave.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

// Tiling of one expert with c rows.  A wide tile holds up to wide_max rows; an expert with
// wide_max < c <= tall rows (tall = 0: never) is covered by ONE tall tile, so its weights are fetched once
// instead of once per wide tile.  Larger experts are split into the fewest wide tiles, n = ceil(c / wide_max),
// and the expert's rows are dealt to them in units of `granule` rows as evenly as possible (the first `extra`
// tiles take one unit more; the last tile takes what is left).  The granule of the bf16 kernels is 64: both
// wave rows of a tile then get the same number of 32-row MFMA blocks.  With many rows per expert the kernel is
// MFMA-bound and the wide shape moves fewer operand bytes per MFMA (measured: tall tiles for 1000-row
// experts cost 15-20 %).
struct ExpertTiling { int n, base, extra, granule; bool is_tall; };
__device__ __forceinline__ ExpertTiling expert_tiling(int c, int wide_max, int granule, int tall) {
  ExpertTiling t;
  t.is_tall = c > wide_max && c <= tall;
  t.n = t.is_tall ? 1 : (c + wide_max - 1) / wide_max;
  const int units = (c + granule - 1) / granule;
  t.base = t.n ? units / t.n : 0;
  t.extra = t.n ? units % t.n : 0;
  t.granule = granule;
  return t;
}
// First row (relative to the expert's segment) and rows of tile i.
__device__ __forceinline__ int tile_first_row(const ExpertTiling& t, int i) { return t.granule * (i * t.base + min(i, t.extra)); }
__device__ __forceinline__ int tile_row_count(const ExpertTiling& t, int i, int c) {
  return min(t.granule * (t.base + (i < t.extra ? 1 : 0)), c - tile_first_row(t, i));
}

// Rows per expert -> counts, offsets (both optional outputs) and the M-tile map, by
// ONE wave.  cnt may live in LDS or in global memory.
//
// Order of the map: it is a list of pair slots, slot j = entries 2j, 2j+1.  A tall
// tile owns a slot (its second entry has 0 rows); wide sibling tiles of one expert
// share a slot; the left-over single wide tiles follow and pair up with each other.
// Consumers deal slot j to XCD j % 8 and run its two tiles side by side on neighbouring CUs.
//
// Singles decide how even the XCDs' shares are.  With balance (the kernels that use it accept
// empty entries anywhere in the map):
//   * the pair slots of the last, incomplete round of 8 are broken up, their tiles join the
//     left-over singles (so that no XCD ends up a whole pair ahead of the others: with 27 pair
//     slots three XCDs would hold 8 tiles and five of them 6 or 7);
//   * all singles are ranked by cost (tiles of 257..320 rows cost a fifth more than tiles of up
//     to 256) and dealt to the XCDs boustrophedon, continuing the round-robin of the slots before
//     them; inside an XCD consecutive singles share a slot, and every other slot swaps its
//     halves, so that the CUs that always take a slot's first tile do not always take the
//     costlier one.  Slots and halves that stay empty are marked with 0 rows.
// Without balance: expert order, no gaps.
constexpr int kMapSlack = 34;      // map entries beyond 2 * tiles that the gaps can take
constexpr int kMaxBrokenTiles = 14;   // tiles of at most 7 broken pair slots
__device__ __forceinline__ int single_cost_of_rows(int rows) {
  return max((rows + 63) & ~63, 128);   // small tiles still stream the expert's whole weight panel
}
__device__ __forceinline__ void build_tile_map(int E_local, const int32_t* cnt, int wide_max, int granule, int tall,
                                               int32_t* counts, int32_t* offsets, const TileMap& tiles) {
  __shared__ int32_t s_broken[3][16];   // expert, first row, rows of the tiles of broken pair slots
  const int lane = lane_id();
  const bool balance = tall > 0;
  constexpr int kPasses = kMaxE / kWave;
  // ---- per expert (lane = expert, kPasses passes): rows before it, tall slots and pair slots before it ----
  int off[kPasses], tall_ex[kPasses], pair_ex[kPasses], single_ex[kPasses];
  int cost[kPasses];     // cost of the expert's left-over single tile, 0 = none
  int n_rows = 0, n_tall = 0, n_pair = 0, n_left = 0, max_rows = 0;
#pragma unroll
  for (int p = 0; p < kPasses; ++p) {
    off[p] = tall_ex[p] = pair_ex[p] = single_ex[p] = cost[p] = 0;
    if (p * kWave >= E_local) continue;
    const int e = p * kWave + lane;
    const int c = e < E_local ? cnt[e] : 0;
    max_rows = max(max_rows, c);
    const ExpertTiling t = expert_tiling(c, wide_max, granule, tall);
    const int nt = t.is_tall ? t.n : 0, np = t.is_tall ? 0 : (t.n >> 1), n1 = t.is_tall ? 0 : (t.n & 1);
    if (n1) cost[p] = single_cost_of_rows(tile_row_count(t, t.n - 1, c));
    const int row_incl = wave_incl_scan(c, lane), tall_incl = wave_incl_scan(nt, lane);
    const int pair_incl = wave_incl_scan(np, lane), single_incl = wave_incl_scan(n1, lane);
    off[p] = n_rows + row_incl - c;
    tall_ex[p] = n_tall + tall_incl - nt;
    pair_ex[p] = n_pair + pair_incl - np;
    single_ex[p] = n_left + single_incl - n1;
    n_rows += __shfl(row_incl, kWave - 1, kWave);
    n_tall += __shfl(tall_incl, kWave - 1, kWave);
    n_pair += __shfl(pair_incl, kWave - 1, kWave);
    n_left += __shfl(single_incl, kWave - 1, kWave);
  }
  // pair slots of the last incomplete round of 8 are broken up (the globally last ones, in expert order)
  const int n_broken = balance ? min((n_tall + n_pair) & 7, n_pair) : 0;
  const int pairs_kept = n_pair - n_broken;
  const int total_slots = n_tall + pairs_kept;   // slots that are not made of singles
  const int n_extra = 2 * n_broken;
  const int n_single = n_left + n_extra;
  if (n_broken) {
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      if (p * kWave >= E_local) break;
      const int e = p * kWave + lane;
      const int c = e < E_local ? cnt[e] : 0;
      const ExpertTiling t = expert_tiling(c, wide_max, granule, tall);
      const int np = t.is_tall ? 0 : (t.n >> 1);
      for (int i = max(pairs_kept - pair_ex[p], 0); i < np; ++i)
        for (int h = 0; h < 2; ++h) {
          const int x = 2 * (pair_ex[p] + i - pairs_kept) + h;
          s_broken[0][x] = e;
          s_broken[1][x] = off[p] + tile_first_row(t, 2 * i + h);
          s_broken[2][x] = tile_row_count(t, 2 * i + h, c);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  // lane x < n_extra holds broken tile x
  const int x_expert = lane < n_extra ? s_broken[0][lane] : 0;
  const int x_row0 = lane < n_extra ? s_broken[1][lane] : 0;
  const int x_rows = lane < n_extra ? s_broken[2][lane] : 0;
  const int x_cost = lane < n_extra ? single_cost_of_rows(x_rows) : 0;
  // rank of each single by (cost descending; left-over singles in expert order, then the broken tiles).  Costs
  // are multiples of 64 between 128 and the wide tile's rows: per cost class one ballot per pass tells every
  // single how many of its class come before it.
  int rank[kPasses], x_rank = 0;
#pragma unroll
  for (int p = 0; p < kPasses; ++p) rank[p] = 0;
  if (balance) {
    const uint64_t lt = (1ull << lane) - 1;
    int run = 0;
    for (int ck = single_cost_of_rows(wide_max); ck >= 128; ck -= 64) {
#pragma unroll
      for (int p = 0; p < kPasses; ++p) {
        if (p * kWave >= E_local) break;
        const uint64_t bal = __ballot(cost[p] == ck);
        if (cost[p] == ck) rank[p] = run + __popcll(bal & lt);
        run += __popcll(bal);
      }
      const uint64_t bal = __ballot(x_cost == ck);
      if (x_cost == ck) x_rank = run + __popcll(bal & lt);
      run += __popcll(bal);
    }
  }
  // singles are dealt to 8 bins (bin b = XCD (total_slots + b) % 8) in rounds of 8, every other round backwards
  const int full = n_single >> 3, rem = n_single & 7;
  auto bin_count = [&](int bin) { return full + (((full & 1) ? 7 - bin : bin) < rem ? 1 : 0); };
  const int bin_slots = ((full + (rem ? 1 : 0)) + 1) >> 1;                     // slots of the fullest bin
  const int n_entries = balance ? 2 * (total_slots + (n_single ? 8 * bin_slots : 0)) : 2 * total_slots + n_single;
  auto single_entry = [&](int r) {
    const int round = r >> 3, pos = r & 7;
    const int bin = (round & 1) ? 7 - pos : pos, j = round, m = j >> 1;
    const bool alone = j == bin_count(bin) - 1 && !(j & 1);
    return 2 * (total_slots + bin + 8 * m) + (alone ? 0 : ((j & 1) ^ (m & 1)));
  };
  if (balance) {
    for (int i = 2 * total_slots + lane; i < n_entries; i += kWave) {           // entries no single will occupy
      const int g = (i >> 1) - total_slots, bin = g & 7, m = g >> 3, half = i & 1;
      const int in_slot = min(max(bin_count(bin) - 2 * m, 0), 2);
      if (half >= in_slot) { tiles.expert[i] = 0; tiles.row0[i] = 0; tiles.rows[i] = 0; }
    }
  }
#pragma unroll
  for (int p = 0; p < kPasses; ++p) {
    if (p * kWave >= E_local) break;
    const int e = p * kWave + lane;
    if (e >= E_local) continue;
    const int c = cnt[e];
    const ExpertTiling t = expert_tiling(c, wide_max, granule, tall);
    if (counts) counts[e] = c;
    if (offsets) offsets[e] = off[p];
    const int sbase = tall_ex[p] + min(pair_ex[p], pairs_kept);   // slots of the experts before this one
    const int kept = t.is_tall ? 0 : max(min(pairs_kept - pair_ex[p], t.n >> 1), 0);
    for (int i = 0; i < t.n; ++i) {
      int idx;
      if (t.is_tall) {
        idx = 2 * (sbase + i);
        tiles.expert[idx + 1] = e; tiles.row0[idx + 1] = off[p]; tiles.rows[idx + 1] = 0;   // the slot's unused half
      } else if (i < 2 * kept) {
        idx = 2 * sbase + i;
      } else if (i < 2 * (t.n >> 1)) {
        continue;                                             // tile of a broken pair slot: written below
      } else if (!balance) {
        idx = 2 * total_slots + single_ex[p];
      } else {
        idx = single_entry(rank[p]);
      }
      tiles.expert[idx] = e;
      tiles.row0[idx] = off[p] + tile_first_row(t, i);
      tiles.rows[idx] = tile_row_count(t, i, c);
    }
  }
  if (lane < n_extra) {
    const int idx = single_entry(x_rank);
    tiles.expert[idx] = x_expert;
    tiles.row0[idx] = x_row0;
    tiles.rows[idx] = x_rows;
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) max_rows = max(max_rows, __shfl_xor(max_rows, o, kWave));
  if (lane == 0) {
    if (offsets) offsets[E_local] = n_rows;
    tiles.meta[kMetaMaxRows] = max_rows;
    tiles.meta[kMetaMTiles] = n_entries;
    tiles.meta[kMetaRows] = n_rows;
    tiles.meta[kMetaStatus] = 0;
  }
}

// Whole-problem step by ONE workgroup: rows per expert (column sums of the
// histogram table) -> counts, offsets, M-tile map.  The table itself is left as it
// is: every rank group derives its own prefix from it.
// s_cnt: (kMaxE + 2) int32 of LDS; s_part: n_waves * kMaxE int32 of LDS.
__device__ __forceinline__ void scan_all(const RouteParams& p, int32_t* s_cnt, int32_t* s_part) {
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const int n_waves = blockDim.x / kWave;
  for (int e0 = 0; e0 < p.E_local; e0 += kWave) {
    const int e = e0 + lane;
    int sum = 0;
    if (e < p.E_local) {
      // batches of independent loads: the table comes from L2, one round trip per batch
      for (int c0 = wave; c0 < p.n_sub; c0 += kHistBatch * n_waves) {
        int v[kHistBatch];
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
          const int c = c0 + u * n_waves;
          v[u] = c < p.n_sub ? p.chunk_cnt[(size_t)c * p.E_local + e] : 0;
        }
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) sum += v[u];
      }
      s_part[wave * kMaxE + e] = sum;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < p.E_local; e += blockDim.x) {
    int sum = 0;
    for (int w = 0; w < n_waves; ++w) sum += s_part[w * kMaxE + e];
    s_cnt[e] = sum;
  }
  __syncthreads();
  if (wave == 0) build_tile_map(p.E_local, s_cnt, p.wide_max, p.granule, p.tall, p.counts, p.offsets, p.tiles);
}

constexpr int kRankLdsWords = 4 * kMaxE;   // LDS words rank_chunk needs per wave

// Rows of the local slots of one group of kChunk tokens, by one wave (lane = token):
// row = (rows of lower experts) + (tokens of earlier sub-chunks selecting e) + (earlier lanes of the
// token's own sub-chunk selecting e).
// The first two terms come straight from the histogram table (lane = expert: one
// pass over its rows gives every expert's total and its count in earlier sub-chunks;
// a wave scan of the totals gives the expert offsets), so a group needs nothing but
// the finished table.  The lanes that selected expert e are collected as a 64-bit
// mask per expert in LDS (an OR, so the result does not depend on the order of the
// updates); a slot's rank inside its sub-chunk is the number of lower lanes of that
// sub-chunk in its expert's mask.
// s_lds: kRankLdsWords int32 of LDS owned by this wave.
__device__ __forceinline__ void rank_chunk(const RouteParams& p, int group, int32_t* s_lds) {
  const int lane = lane_id();
  const int t = group * kChunk + lane;
  const bool live = t < p.T;
  unsigned long long* s_mask = reinterpret_cast<unsigned long long*>(s_lds);   // [E_local]
  int32_t* s_base = s_lds + 2 * kMaxE;                                           // [2][E_local] first row per half
  const int sub0 = group * (kChunk / kSub);
  // The table walk is a chain of round trips to the L2, so it is spread over all 64 lanes: with fewer than 64
  // local experts, `parts` lanes share an expert and take every parts-th batch of rows (E_local = 32: 8 round
  // trips instead of 16 at T = 8192); their partial sums are added with a butterfly.
  const int ew = p.E_local >= kWave ? kWave : (p.E_local <= 1 ? 1 : 1 << (32 - __builtin_clz(p.E_local - 1)));
  const int parts = kWave / ew, part = lane >> __builtin_ctz(ew), el = lane & (ew - 1);
  int run = 0;   // rows of the experts before this block of ew
  for (int e0 = 0; e0 < p.E_local; e0 += ew) {
    const int e = e0 + el;
    int total = 0, before = 0, own0 = 0;
    if (e < p.E_local) {
      for (int c0 = part * kHistBatch; c0 < p.n_sub; c0 += kHistBatch * parts) {
        int v[kHistBatch];
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) v[u] = c0 + u < p.n_sub ? p.chunk_cnt[(size_t)(c0 + u) * p.E_local + e] : 0;
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
          total += v[u];
          before += c0 + u < sub0 ? v[u] : 0;
          own0 = c0 + u == sub0 ? v[u] : own0;
        }
      }
    }
    for (int off = ew; off < kWave; off <<= 1) {   // own0 is non-zero in one part only
      total += __shfl_xor(total, off, kWave);
      before += __shfl_xor(before, off, kWave);
      own0 += __shfl_xor(own0, off, kWave);
    }
    const int incl = wave_incl_scan(part == 0 ? total : 0, lane);   // lanes 0..ew-1: running sum over the experts
    if (part == 0 && e < p.E_local) {
      const int first = run + incl - total + before;
      s_mask[e] = 0ull;
      s_base[e] = first;
      s_base[kMaxE + e] = first + own0;
    }
    run += __shfl(incl, kWave - 1, kWave);
  }
  int32_t le[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    const int idx = (live && j < p.k) ? p.topk_idx[(size_t)t * p.k + j] : -1;
    const int l = idx - p.expert_base;
    le[j] = (idx >= 0 && l >= 0 && l < p.E_local) ? l : -1;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int j = 0; j < kMaxK; ++j)
    if (le[j] >= 0) atomicOr(&s_mask[le[j]], 1ull << lane);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int half = lane / kSub;
  // lower lanes of this lane's own sub-chunk
  const unsigned long long lt = ((1ull << lane) - 1ull) & (half ? ~((1ull << kSub) - 1ull) : ~0ull);
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    if (j >= p.k) break;
    int r = -1;
    if (le[j] >= 0) {
      r = s_base[half * kMaxE + le[j]] + __popcll(s_mask[le[j]] & lt);
      p.token_of[r] = t;
      p.slot_of[r] = j;
    }
    if (live) p.row_of[(size_t)t * p.k + j] = r;
  }
}

__global__ __launch_bounds__(512) void route_kernel(RouteParams p) {
  __shared__ int32_t s_idx[kSub * kMaxK];
  __shared__ float s_val[kSub * kMaxK];
  route_chunk(p, blockIdx.x, s_idx, s_val);
}

// The two steps that need nothing but the finished histogram table run side by side in one launch
// (sched_prepare_kernel): workgroup 0 sums the table into counts, offsets and the M-tile map; every other
// workgroup ranks 4 groups of 64 tokens, one per wave.  Grid: 1 + ceil(n_groups / 4) workgroups of 256 threads.
constexpr int kScanRankWaves = 4;
static_assert(kScanRankWaves * kRankLdsWords >= (kScanRankWaves + 1) * kMaxE + 2 + 64, "LDS of the scan step");

}  // namespace moe
