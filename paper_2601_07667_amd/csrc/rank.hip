// asl_rank: RankDesc of the all-head score vector (Alg. 1 step 11 of the paper):
// rank[t] = position of t in the order (score descending, token index ascending).
//
// A stable least-significant-digit radix sort of (key, index) pairs on an order-preserving
// 32-bit transform of the fp32 score, 8 bits per pass; the last pass scatters positions to
// rank[index] instead of writing the sorted pairs.  Per pass: a histogram kernel whose last
// workgroup turns the [digit][tile] counts into exclusive offsets, then a scatter kernel that
// ranks equal digits inside a tile with wavefront ballots (stable by construction).
#include "asl_internal.h"

namespace asl {

constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortRounds = kSortTile / kSortThreads;        // elements per thread
constexpr int kSortPerWave = kSortTile / kSortWaves;

// Ascending unsigned order of the result == descending float order; -0 is treated as +0.
__device__ __forceinline__ uint32_t desc_key(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;
}

template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads)
sort_hist_kernel(const float* __restrict__ s, const uint32_t* __restrict__ keys_in, int T, int shift,
                 int n_tiles, uint32_t* tile_hist, uint32_t* ticket) {
  __shared__ uint32_t h[256];
  __shared__ uint32_t tot[256];
  __shared__ int is_last;
  const int tid = threadIdx.x;
  h[tid] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortTile;
#pragma unroll
  for (int i = 0; i < kSortRounds; ++i) {
    int e = base + i * kSortThreads + tid;
    if (e < T) {
      uint32_t key = FIRST ? desc_key(s[e]) : keys_in[e];
      atomicAdd(&h[(key >> shift) & 255u], 1u);
    }
  }
  __syncthreads();
  tile_hist[(int64_t)tid * n_tiles + blockIdx.x] = h[tid];
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    is_last = (t == gridDim.x - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  // exclusive offsets in (digit, tile) order, in place
  uint32_t* row = tile_hist + (int64_t)tid * n_tiles;
  uint32_t sum = 0;
  for (int t = 0; t < n_tiles; ++t) sum += __hip_atomic_load(&row[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  tot[tid] = sum;
  __syncthreads();
  uint32_t run = 0;
  for (int d = 0; d < tid; ++d) run += tot[d];
  for (int t = 0; t < n_tiles; ++t) {
    uint32_t v = __hip_atomic_load(&row[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    row[t] = run;
    run += v;
  }
  if (tid == 0) *ticket = 0;
}

template <bool FIRST, bool LAST>
__global__ void __launch_bounds__(kSortThreads)
sort_scatter_kernel(const float* __restrict__ s, const uint32_t* __restrict__ keys_in,
                    const uint32_t* __restrict__ idx_in, int T, int shift, int n_tiles,
                    const uint32_t* __restrict__ tile_off, uint32_t* __restrict__ keys_out,
                    uint32_t* __restrict__ idx_out, int32_t* __restrict__ rank_out) {
  __shared__ uint32_t cnt[kSortWaves][256];
  __shared__ uint32_t start[kSortWaves][256];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w) cnt[w][tid] = 0;
  __syncthreads();

  constexpr int R = kSortPerWave / 64;
  uint32_t key[R], idx[R], off[R];
  const int base = blockIdx.x * kSortTile + wave * kSortPerWave;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    const bool valid = e < T;
    key[r] = 0;
    idx[r] = 0;
    if (valid) {
      key[r] = FIRST ? desc_key(s[e]) : keys_in[e];
      idx[r] = FIRST ? (uint32_t)e : idx_in[e];
    }
    const uint32_t d = (key[r] >> shift) & 255u;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const uint32_t before = __popcll(peers & lt_mask);
    uint32_t old = 0;
    if (valid) old = cnt[wave][d];
    if (valid && before == 0) cnt[wave][d] = old + (uint32_t)__popcll(peers);
    off[r] = old + before;
  }
  __syncthreads();
  {
    uint32_t run = tile_off[(int64_t)tid * n_tiles + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      start[w][tid] = run;
      run += cnt[w][tid];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    if (e < T) {
      const uint32_t d = (key[r] >> shift) & 255u;
      const uint32_t dest = start[wave][d] + off[r];
      if (LAST) {
        rank_out[idx[r]] = (int32_t)dest;
      } else {
        keys_out[dest] = key[r];
        idx_out[dest] = idx[r];
      }
    }
  }
}

hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st) {
  const int n_tiles = (T + kSortTile - 1) / kSortTile;
  uint32_t* ticket = ws.counters + kCntSortTicket;
  const dim3 grid(n_tiles), block(kSortThreads);
  // pass 0: scores -> buffer 0
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<true>), grid, block, 0, st, s, nullptr, T, 0, n_tiles, ws.tile_hist, ticket);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<true, false>), grid, block, 0, st, s, nullptr, nullptr, T, 0,
                     n_tiles, ws.tile_hist, ws.sort_key[0], ws.sort_idx[0], nullptr);
  // pass 1: 0 -> 1
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[0], T, 8, n_tiles, ws.tile_hist, ticket);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, false>), grid, block, 0, st, nullptr, ws.sort_key[0],
                     ws.sort_idx[0], T, 8, n_tiles, ws.tile_hist, ws.sort_key[1], ws.sort_idx[1], nullptr);
  // pass 2: 1 -> 0
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[1], T, 16, n_tiles, ws.tile_hist, ticket);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, false>), grid, block, 0, st, nullptr, ws.sort_key[1],
                     ws.sort_idx[1], T, 16, n_tiles, ws.tile_hist, ws.sort_key[0], ws.sort_idx[0], nullptr);
  // pass 3: 0 -> rank
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[0], T, 24, n_tiles, ws.tile_hist, ticket);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, true>), grid, block, 0, st, nullptr, ws.sort_key[0],
                     ws.sort_idx[0], T, 24, n_tiles, ws.tile_hist, nullptr, nullptr, rank_out);
  return hipGetLastError();
}

}  // namespace asl
