// Device code of asl_rank's sort pass (see rank.hip for the method), written as a function over an
// explicit shared-state struct so that another kernel can host it beside a second body.
#pragma once
#include "asl_internal.h"

namespace asl {

constexpr int kSortThreads = ASL_SORT_THREADS;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortGroups = kSortThreads / 128;              // thread groups that share the polling
// Elements per thread: kSortRounds normally (tiles of kSortTile elements); kSortRoundsBig for inputs
// whose kSortTile-element tiles would be more workgroups than one launch may have.
constexpr int kSortRounds = kSortTile / kSortThreads;
constexpr int kSortRoundsBig = 4 * kSortRounds;
static_assert(kSortTile % kSortThreads == 0 && kSortThreads % 128 == 0 && kSortThreads >= 256, "sort geometry");
static_assert(kSortThreads * kSortRoundsBig < (1 << kFlagCountBits), "a tile's digit count must fit the packed field");

struct SortShared {
  uint32_t h[kHistWords];
  uint32_t cnt[kSortWaves][256];
  uint32_t start[kSortWaves][256];
  uint32_t part_tot[kSortGroups][256];
  uint32_t part_prev[kSortGroups][256];
  uint32_t digit_off[256];
  uint32_t wave_sum[4];
  int gave_up;
};

struct SortArgs {
  const float* s;                // scores (first pass only)
  const uint32_t* keys_in;       // (key, index) pairs of the previous pass
  const uint32_t* idx_in;
  int T, shift, n_tiles;
  unsigned long long* table;     // [n_tiles][128] tagged digit counts
  unsigned long long* epoch;     // launch counter behind the tags
  uint32_t* fault;
  uint32_t* keys_out;
  uint32_t* idx_out;
  int32_t* rank_out;             // last pass only
};

// Tiles of a sort of T scores: kSortTile elements each, or four times that when T would otherwise
// need more workgroups than `limit`; n_tiles = 0 if even those are too many.
struct SortPlan {
  int n_tiles;
  bool big;
};
SortPlan sort_plan(int T, int limit);
// Arguments of pass `pass` (0..3) of the sort of s[0..T) into rank_out, using ws's sort buffers.
SortArgs sort_pass_args(const Workspace& ws, const float* s, int T, int n_tiles, int32_t* rank_out, int pass);

// One pass for tile `me` (kSortThreads threads, R elements each).
template <int R, bool FIRST, bool LAST>
__device__ __forceinline__ void sort_pass_body(SortShared& sh, const SortArgs& a, int me) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const unsigned long long tag = *a.epoch + 1ull;

  // this wave's elements: issue every load before anything waits on one
  constexpr int kTile = kSortThreads * R, kPerWave = 64 * R;
  uint32_t key[R], idx[R], off[R];
  const int base = me * kTile + wave * kPerWave;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    key[r] = 0;
    idx[r] = 0;
    if (e < a.T) {
      key[r] = FIRST ? order_key(a.s[e]) : a.keys_in[e];
      idx[r] = FIRST ? (uint32_t)e : a.idx_in[e];
    }
  }
  hist_clear(sh.h, tid, kSortThreads);
  if (tid == 0) sh.gave_up = 0;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w)
    if (tid < 256) sh.cnt[w][tid] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r)
    if (base + r * 64 + lane < a.T) hist_add(sh.h, tid, (key[r] >> a.shift) & 255u);
  __syncthreads();
  // publish this tile's counts, two digits per word
  if (tid < 128)
    flag_publish(&a.table[(int64_t)me * 128 + tid], tag, hist_total(sh.h, 2 * tid), hist_total(sh.h, 2 * tid + 1));

  // every tile's counts of digits 2w, 2w+1 (w = tid % 128); the thread groups share the tiles
  {
    const int w = tid & 127, grp = tid >> 7;
    uint32_t tot0 = 0, tot1 = 0, prev0 = 0, prev1 = 0;
    bool failed = false;
    for (int t0 = grp; t0 < a.n_tiles; t0 += kSortGroups * kFlagBatch) {
      unsigned long long v[kFlagBatch];
      failed |= !flag_poll_batch<kSortGroups>(a.table + w, 128, t0, a.n_tiles, tag, v);
#pragma unroll
      for (int u = 0; u < kFlagBatch; ++u) {
        const int t = t0 + u * kSortGroups;
        if (t < a.n_tiles) {
          const uint32_t c0 = flag_count0(v[u]), c1 = flag_count1(v[u]);
          tot0 += c0;
          tot1 += c1;
          prev0 += (t < me) ? c0 : 0u;
          prev1 += (t < me) ? c1 : 0u;
        }
      }
    }
    sh.part_tot[grp][2 * w] = tot0;
    sh.part_tot[grp][2 * w + 1] = tot1;
    sh.part_prev[grp][2 * w] = prev0;
    sh.part_prev[grp][2 * w + 1] = prev1;
    if (failed) {
      sh.gave_up = 1;
      *a.fault = 1u;
    }
  }
  __syncthreads();
  if (sh.gave_up) return;                               // uniform: nothing is scattered by this workgroup
  if (me == 0 && tid == 0) *a.epoch = tag;             // every workgroup has read the old value by now

  // digit `tid` (first 256 threads): total over all tiles, exclusive scan over the digits
  if (tid < 256) {
    uint32_t tot = 0, prev = 0;
#pragma unroll
    for (int g = 0; g < kSortGroups; ++g) {
      tot += sh.part_tot[g][tid];
      prev += sh.part_prev[g][tid];
    }
    const uint32_t incl = wave_prefix_sum(tot);
    if (lane == 63) sh.wave_sum[wave] = incl;
    sh.part_tot[0][tid] = incl - tot;                   // exclusive within the wave (own group row is consumed)
    sh.part_prev[0][tid] = prev;
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t digit_base = sh.part_tot[0][tid];
    for (int w = 0; w < wave; ++w) digit_base += sh.wave_sum[w];
    sh.digit_off[tid] = digit_base + sh.part_prev[0][tid];   // first destination of digit `tid` in this tile
  }

  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    const bool valid = e < a.T;
    const uint32_t d = (key[r] >> a.shift) & 255u;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const uint32_t before = __popcll(peers & lt_mask);
    uint32_t old = 0;
    if (valid) old = sh.cnt[wave][d];
    if (valid && before == 0) sh.cnt[wave][d] = old + (uint32_t)__popcll(peers);
    off[r] = old + before;
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t run = sh.digit_off[tid];
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      sh.start[w][tid] = run;
      run += sh.cnt[w][tid];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    if (e < a.T) {
      const uint32_t d = (key[r] >> a.shift) & 255u;
      const uint32_t dest = sh.start[wave][d] + off[r];
      if (LAST) {
        a.rank_out[idx[r]] = (int32_t)dest;
      } else {
        a.keys_out[dest] = key[r];
        a.idx_out[dest] = idx[r];
      }
    }
  }
}

}  // namespace asl
