// asl_select: the k highest-scoring past tokens of each row, ties to the lower index, written in
// ascending token order and followed by the window tokens (Alg. 1 steps 9-10 per KV head;
// Alg. 2 steps 11-12 on the all-head scores).
//
// Radix select on the same order-preserving key transform as the rank kernel: four 8-bit
// histogram passes from the most significant digit narrow down the k-th key, then an order-
// preserving compaction keeps every key below the threshold key and the first k_rem keys equal
// to it.  Integer work throughout: the result does not depend on scheduling.
#include "asl_internal.h"

namespace asl {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelPerWave = kSelTile / kSelWaves;     // 1024
constexpr int kSelRounds = kSelPerWave / 64;          // 16

__device__ __forceinline__ uint32_t sel_key(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;                                        // ascending key == descending score
}

// Workspace layout (all plain stores, no atomics):
//   hist[pass][row][tile][256]  digit histogram of the keys of that tile whose higher digits match
//                               the prefix chosen so far
//   state[pass][row][2]         {prefix of `pass` digits, keys still to take} as known BEFORE pass
//   tile_lt[row][tile]          keys of the tile already known to lie below the threshold key
// Every workgroup of pass p+1 re-derives the digit chosen from the pass-p histograms (a few tens
// of KB of L2 reads), so nothing has to be serialised through atomics or a last workgroup.

struct Pick {
  uint32_t digit;      // digit of the k-th key in this pass
  uint32_t k_rem;      // keys still to take among those equal to the prefix incl. this digit
  uint32_t lt_mine;    // this tile's keys with a smaller digit
  uint32_t lt_prev;    // earlier tiles' keys with a smaller digit
  uint32_t eq_prev;    // earlier tiles' keys with exactly this digit
};

// hp = hist of one (pass,row): [n_tiles][256].  All 256 threads take part.
__device__ __forceinline__ Pick pick_digit(const uint32_t* __restrict__ hp, int n_tiles, int me,
                                           uint32_t k_rem_in, uint32_t* sm /* >= 16 words */) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // column `tid` of the [n_tiles][256] table: all tiles, and the tiles before this one.
  // Loads are independent; unrolled so that many are in flight at once.
  uint32_t tot = 0, prev = 0;
  const uint32_t mine = hp[(int64_t)me * 256 + tid];
  int t = 0;
  for (; t + 16 <= n_tiles; t += 16) {
    uint32_t v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = hp[(int64_t)(t + u) * 256 + tid];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      tot += v[u];
      prev += (t + u < me) ? v[u] : 0u;
    }
  }
  for (; t < n_tiles; ++t) {
    const uint32_t v = hp[(int64_t)t * 256 + tid];
    tot += v;
    prev += (t < me) ? v : 0u;
  }
  uint32_t incl = tot;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();                                     // sm may still be in use by a previous call
  if (lane == 63) sm[wave] = incl;
  if (tid == 0) {                                      // defined result even if no digit qualifies
    sm[4] = 0;                                         // (cannot happen while k <= T)
    sm[5] = 0;
    sm[14] = 0;
  }
  __syncthreads();
  uint32_t excl = incl - tot;
  for (int w = 0; w < wave; ++w) excl += sm[w];
  if (excl < k_rem_in && excl + tot >= k_rem_in) {     // exactly one digit satisfies this
    sm[4] = (uint32_t)tid;
    sm[5] = k_rem_in - excl;
    sm[14] = prev;                                     // earlier tiles' keys with exactly this digit
  }
  __syncthreads();
  Pick p;
  p.digit = sm[4];
  p.k_rem = sm[5];
  p.eq_prev = sm[14];
  uint32_t a = ((uint32_t)tid < p.digit) ? mine : 0u;
  uint32_t b = ((uint32_t)tid < p.digit) ? prev : 0u;
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_down(a, o);
    b += __shfl_down(b, o);
  }
  if (lane == 0) {
    sm[6 + wave] = a;
    sm[10 + wave] = b;
  }
  __syncthreads();
  p.lt_mine = sm[6] + sm[7] + sm[8] + sm[9];
  p.lt_prev = sm[10] + sm[11] + sm[12] + sm[13];
  return p;
}

// Histogram pass `pass` (0..3, most significant digit first).
__global__ void __launch_bounds__(kSelThreads)
select_hist_kernel(const float* __restrict__ scores, int T, int n_tiles, int rows, int pass, int k,
                   uint32_t* __restrict__ hist, uint32_t* __restrict__ state,
                   uint32_t* __restrict__ tile_lt) {
  __shared__ uint32_t h[kHistWords];
  __shared__ uint32_t sm[16];
  const int tid = threadIdx.x, row = blockIdx.y, tile = blockIdx.x;
  const int shift = 24 - 8 * pass;
  const float* sr = scores + (int64_t)row * T;
  const int base = tile * kSelTile;
  constexpr int E = kSelTile / kSelThreads;
  uint32_t key[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {                        // all loads in flight before the first use
    const int e = base + i * kSelThreads + tid;
    key[i] = (e < T) ? sel_key(sr[e]) : 0u;
  }
  uint32_t prefix = 0;
  if (pass > 0) {
    const uint32_t* st_in = state + ((int64_t)(pass - 1) * rows + row) * 2;
    const uint32_t prefix_in = (pass == 1) ? 0u : st_in[0];
    const uint32_t k_rem_in = (pass == 1) ? (uint32_t)k : st_in[1];
    const uint32_t* hp = hist + ((int64_t)(pass - 1) * rows + row) * n_tiles * 256;
    const Pick p = pick_digit(hp, n_tiles, tile, k_rem_in, sm);
    prefix = (prefix_in << 8) | p.digit;
    if (tid == 0) {
      uint32_t* lt = tile_lt + (int64_t)row * n_tiles + tile;
      *lt = (pass == 1 ? 0u : *lt) + p.lt_mine;
      if (tile == 0) {
        uint32_t* st_out = state + ((int64_t)pass * rows + row) * 2;
        st_out[0] = prefix;
        st_out[1] = p.k_rem;
      }
    }
  }
  hist_clear(h, tid, kSelThreads);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int e = base + i * kSelThreads + tid;
    const bool match = (pass == 0) || ((key[i] >> (shift + 8)) == prefix);
    if (e < T && match) hist_add(h, tid, (key[i] >> shift) & 255u);
  }
  __syncthreads();
  hist[(((int64_t)pass * rows + row) * n_tiles + tile) * 256 + tid] = hist_total(h, tid);
}

// Ordered compaction: position of a kept token = (#below before it) + min(#equal before it, k_rem).
__global__ void __launch_bounds__(kSelThreads)
select_write_kernel(const float* __restrict__ scores, int T, int n_tiles, int rows, int k, int W,
                    const uint32_t* __restrict__ hist, const uint32_t* __restrict__ state,
                    const uint32_t* __restrict__ tile_lt, int32_t* __restrict__ idx_out) {
  __shared__ uint32_t sm[16];
  __shared__ uint32_t red[kSelWaves];
  __shared__ uint32_t wave_tot[2][kSelWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, row = blockIdx.y, tile = blockIdx.x;
  const float* sr = scores + (int64_t)row * T;
  // this wave's keys (kSelPerWave consecutive tokens, 64 per round), loaded before anything waits
  const int base = tile * kSelTile + wave * kSelPerWave;
  uint32_t key[kSelRounds];
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    const int e = base + r * 64 + lane;
    key[r] = (e < T) ? sel_key(sr[e]) : 0xffffffffu;
  }
  const uint32_t* st_in = state + ((int64_t)3 * rows + row) * 2;          // 3-digit prefix, written by pass 3
  const uint32_t* h3 = hist + ((int64_t)3 * rows + row) * n_tiles * 256;
  const Pick p = pick_digit(h3, n_tiles, tile, st_in[1], sm);
  const uint32_t thr = (st_in[0] << 8) | p.digit;
  const uint32_t k_rem = p.k_rem;
  int32_t* out = idx_out + (int64_t)row * (k + W);

  // keys below the threshold in the tiles before this one (passes 0-2 from tile_lt, pass 3 from h3)
  uint32_t lt_b = 0;
  for (int t = tid; t < tile; t += kSelThreads) lt_b += tile_lt[(int64_t)row * n_tiles + t];
  for (int o = 32; o > 0; o >>= 1) lt_b += __shfl_down(lt_b, o);
  if (lane == 0) red[wave] = lt_b;

  // this wave's totals
  uint32_t w_lt = 0, w_eq = 0;
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    const int e = base + r * 64 + lane;
    const bool v = e < T;
    w_lt += __popcll(__ballot(v && key[r] < thr));
    w_eq += __popcll(__ballot(v && key[r] == thr));
  }
  if (lane == 0) {
    wave_tot[0][wave] = w_lt;
    wave_tot[1][wave] = w_eq;
  }
  __syncthreads();
  uint32_t lt_run = p.lt_prev, eq_run = p.eq_prev;
  for (int w = 0; w < kSelWaves; ++w) lt_run += red[w];
  for (int w = 0; w < wave; ++w) {
    lt_run += wave_tot[0][w];
    eq_run += wave_tot[1][w];
  }
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    const int e = base + r * 64 + lane;
    const bool v = e < T;
    const bool is_lt = v && key[r] < thr;
    const bool is_eq = v && key[r] == thr;
    const uint64_t b_lt = __ballot(is_lt), b_eq = __ballot(is_eq);
    const uint32_t lt_before = lt_run + (uint32_t)__popcll(b_lt & lt_mask);
    const uint32_t eq_before = eq_run + (uint32_t)__popcll(b_eq & lt_mask);
    if (is_lt || (is_eq && eq_before < k_rem)) {
      const uint32_t pos = lt_before + (eq_before < k_rem ? eq_before : k_rem);
      if (pos < (uint32_t)k) out[pos] = e;             // always true for consistent counts
    }
    lt_run += (uint32_t)__popcll(b_lt);
    eq_run += (uint32_t)__popcll(b_eq);
  }
  // window tokens T .. T+W-1 (Alg. 1 step 10: Concat with I_w)
  if (tile == 0)
    for (int i = tid; i < W; i += kSelThreads) out[k + i] = T + i;
}

hipError_t launch_select(const Workspace& ws, const float* scores, int rows, int T, int k, int W,
                         int32_t* idx_out, hipStream_t st) {
  const int n_tiles = (T + kSelTile - 1) / kSelTile;
  const dim3 grid(n_tiles, rows), block(kSelThreads);
  for (int pass = 0; pass < 4; ++pass)
    ASL_LAUNCH(ws.prof, kKernSelHist, st, select_hist_kernel, grid, block, 0, st, scores, T, n_tiles, rows,
               pass, k, ws.sel_hist, ws.sel_state, ws.sel_tile_cnt);
  ASL_LAUNCH(ws.prof, kKernSelWrite, st, select_write_kernel, grid, block, 0, st, scores, T, n_tiles, rows, k,
             W, ws.sel_hist, ws.sel_state, ws.sel_tile_cnt, idx_out);
  return hipGetLastError();
}

}  // namespace asl
