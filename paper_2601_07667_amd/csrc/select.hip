// asl_select: the k highest-scoring past tokens of each row, ties to the lower index, written in
// ascending token order and followed by the window tokens (Alg. 1 steps 9-10 per KV head;
// Alg. 2 steps 11-12 on the all-head scores).
//
// Radix select on the same order-preserving key transform as the rank kernel: four 8-bit
// histogram passes from the most significant digit narrow down the k-th key (the last workgroup
// of a row picks the digit), then an order-preserving compaction keeps every key below the
// threshold key and the first k_rem keys equal to it.  Integer work throughout: the result does
// not depend on scheduling.
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

// sel_state[row*4 + 0] = key prefix found so far, [row*4 + 1] = how many keys still to take
__global__ void __launch_bounds__(kSelThreads)
select_hist_kernel(const float* __restrict__ scores, int T, int pass, int k, uint32_t* hist,
                   uint32_t* sel_state, uint32_t* tickets) {
  __shared__ uint32_t h[256];
  __shared__ uint32_t scan[256];
  __shared__ int is_last;
  const int tid = threadIdx.x, row = blockIdx.y;
  const int shift = 24 - 8 * pass;
  const uint32_t prefix = (pass == 0) ? 0u : sel_state[row * 4 + 0];
  h[tid] = 0;
  __syncthreads();
  const float* sr = scores + (int64_t)row * T;
  const int base = blockIdx.x * kSelTile;
  for (int i = 0; i < kSelTile / kSelThreads; ++i) {
    int e = base + i * kSelThreads + tid;
    if (e < T) {
      uint32_t key = sel_key(sr[e]);
      bool match = (pass == 0) || ((key >> (shift + 8)) == prefix);
      if (match) atomicAdd(&h[(key >> shift) & 255u], 1u);
    }
  }
  __syncthreads();
  if (h[tid] != 0)
    __hip_atomic_fetch_add(&hist[row * 256 + tid], h[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    uint32_t t = __hip_atomic_fetch_add(&tickets[row], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    is_last = (t == gridDim.x - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  const uint32_t mine = __hip_atomic_load(&hist[row * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint32_t k_rem = (pass == 0) ? (uint32_t)k : sel_state[row * 4 + 1];
  scan[tid] = mine;
  __syncthreads();
  uint32_t excl = 0;
  for (int d = 0; d < tid; ++d) excl += scan[d];
  __syncthreads();
  if (excl < k_rem && excl + mine >= k_rem) {          // exactly one digit satisfies this
    sel_state[row * 4 + 0] = (prefix << 8) | (uint32_t)tid;
    sel_state[row * 4 + 1] = k_rem - excl;
  }
  __hip_atomic_store(&hist[row * 256 + tid], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid == 0) __hip_atomic_store(&tickets[row], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// per (row, tile): how many keys are below / equal to the threshold key
__global__ void __launch_bounds__(kSelThreads)
select_count_kernel(const float* __restrict__ scores, int T, int n_tiles,
                    const uint32_t* __restrict__ sel_state, uint32_t* __restrict__ tile_cnt) {
  __shared__ uint32_t red[2][kSelWaves];
  const int tid = threadIdx.x, row = blockIdx.y;
  const uint32_t thr = sel_state[row * 4 + 0];
  const float* sr = scores + (int64_t)row * T;
  const int base = blockIdx.x * kSelTile;
  uint32_t lt = 0, eq = 0;
  for (int i = 0; i < kSelTile / kSelThreads; ++i) {
    int e = base + i * kSelThreads + tid;
    if (e < T) {
      uint32_t key = sel_key(sr[e]);
      lt += key < thr;
      eq += key == thr;
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    lt += __shfl_down(lt, o);
    eq += __shfl_down(eq, o);
  }
  if ((tid & 63) == 0) {
    red[0][tid >> 6] = lt;
    red[1][tid >> 6] = eq;
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t a = 0, b = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      a += red[0][w];
      b += red[1][w];
    }
    tile_cnt[((int64_t)row * n_tiles + blockIdx.x) * 2 + 0] = a;
    tile_cnt[((int64_t)row * n_tiles + blockIdx.x) * 2 + 1] = b;
  }
}

// ordered compaction: position of a kept token = (#below before it) + min(#equal before it, k_rem)
__global__ void __launch_bounds__(kSelThreads)
select_write_kernel(const float* __restrict__ scores, int T, int n_tiles, int k, int W,
                    const uint32_t* __restrict__ sel_state, const uint32_t* __restrict__ tile_cnt,
                    int32_t* __restrict__ idx_out) {
  __shared__ uint32_t red[2][kSelWaves];
  __shared__ uint32_t wave_tot[2][kSelWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, row = blockIdx.y;
  const uint32_t thr = sel_state[row * 4 + 0];
  const uint32_t k_rem = sel_state[row * 4 + 1];
  const float* sr = scores + (int64_t)row * T;
  int32_t* out = idx_out + (int64_t)row * (k + W);

  // totals of the tiles before this one
  uint32_t lt_b = 0, eq_b = 0;
  for (int t = tid; t < (int)blockIdx.x; t += kSelThreads) {
    lt_b += tile_cnt[((int64_t)row * n_tiles + t) * 2 + 0];
    eq_b += tile_cnt[((int64_t)row * n_tiles + t) * 2 + 1];
  }
  for (int o = 32; o > 0; o >>= 1) {
    lt_b += __shfl_down(lt_b, o);
    eq_b += __shfl_down(eq_b, o);
  }
  if (lane == 0) {
    red[0][wave] = lt_b;
    red[1][wave] = eq_b;
  }

  // this wave's keys (kSelPerWave consecutive tokens, 64 per round) and its totals
  const int base = blockIdx.x * kSelTile + wave * kSelPerWave;
  uint32_t key[kSelRounds];
  uint32_t w_lt = 0, w_eq = 0;
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    const int e = base + r * 64 + lane;
    key[r] = (e < T) ? sel_key(sr[e]) : 0xffffffffu;
    const bool v = e < T;
    w_lt += __popcll(__ballot(v && key[r] < thr));
    w_eq += __popcll(__ballot(v && key[r] == thr));
  }
  if (lane == 0) {
    wave_tot[0][wave] = w_lt;
    wave_tot[1][wave] = w_eq;
  }
  __syncthreads();
  uint32_t lt_run = 0, eq_run = 0;
  for (int w = 0; w < kSelWaves; ++w) {
    lt_run += red[0][w];
    eq_run += red[1][w];
  }
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
      out[pos] = e;
    }
    lt_run += (uint32_t)__popcll(b_lt);
    eq_run += (uint32_t)__popcll(b_eq);
  }
  // window tokens T .. T+W-1 (Alg. 1 step 10: Concat with I_w)
  if (blockIdx.x == 0)
    for (int i = tid; i < W; i += kSelThreads) out[k + i] = T + i;
}

hipError_t launch_select(const Workspace& ws, const float* scores, int rows, int T, int k, int W,
                         int32_t* idx_out, hipStream_t st) {
  const int n_tiles = (T + kSelTile - 1) / kSelTile;
  const dim3 grid(n_tiles, rows), block(kSelThreads);
  uint32_t* tickets = ws.counters + kCntSelTicket;
  for (int pass = 0; pass < 4; ++pass)
    ASL_LAUNCH(ws.prof, kKernSelHist, st, select_hist_kernel, grid, block, 0, st, scores, T, pass, k, ws.sel_hist,
                       ws.sel_state, tickets);
  ASL_LAUNCH(ws.prof, kKernSelCount, st, select_count_kernel, grid, block, 0, st, scores, T, n_tiles, ws.sel_state,
                     ws.sel_tile_cnt);
  ASL_LAUNCH(ws.prof, kKernSelWrite, st, select_write_kernel, grid, block, 0, st, scores, T, n_tiles, k, W, ws.sel_state,
                     ws.sel_tile_cnt, idx_out);
  return hipGetLastError();
}

}  // namespace asl
