// asl_rankvar: the relative rank-variance statistic and the selection-layer decision
// (Alg. 2 steps 4-10 of the paper; Sec. 4.1 top(L), var_top and relative-variance equations).
//
// Ranks are a permutation, so "the k smallest ranks of a row" is rank < k and the union over rows
// is  min_l R[l,t] < k.  Per token the population variance times n^2 is the integer
// n * sum R^2 - (sum R)^2; the sum over the union is accumulated exactly in 64-bit integers
// (per-workgroup partials; integer sums are order-independent); workgroup 0 of the same launch adds
// the partials and performs the single double-precision division, the comparison with tau and the
// state update.  No read-modify-write atomics, no fences.
#include "asl_internal.h"

namespace asl {

constexpr int kVarThreads = 256;

// The ring row of layer_idx continues the rows already held iff layer_idx is the layer after
// state->last_layer, or that layer minus l_obs (a captured trip of l_obs layers round the ring being
// replayed: the same rows are overwritten in the same order).  Any other index restarts the ring.
__device__ __forceinline__ bool continues_ring(const asl_state* state, int layer_idx, int l_obs) {
  const int next = state->last_layer + 1;
  return layer_idx == next || layer_idx == next - l_obs;
}

__global__ void stat_skip_kernel(asl_stat* out, asl_state* state, int layer_idx, int l_obs, int push) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  if (push) {
    int n = state->n_valid_rows;
    if (n > 0 && !continues_ring(state, layer_idx, l_obs)) n = 0;
    state->n_valid_rows = n + 1 < l_obs ? n + 1 : l_obs;
    state->last_layer = layer_idx;
  }
  out->var_top = __builtin_nan("");
  out->rel_var = __builtin_nan("");
  out->numerator = 0;
  out->union_size = 0;
  out->n_rows = 0;
  out->evaluated = 0;
  out->selected = 0;
}

// Rows in use after (optionally) pushing this layer's row: a pure function of the old state, so
// every workgroup derives it on its own; only workgroup 0 writes the state back.
__device__ __forceinline__ int rows_in_use(const asl_state* state, int layer_idx, int l_obs, int push) {
  int n = state->n_valid_rows;
  if (push) {
    if (n > 0 && !continues_ring(state, layer_idx, l_obs)) n = 0;
    n = n + 1 < l_obs ? n + 1 : l_obs;
  }
  return n;
}

// Per-workgroup partial sums over the union (integers, so the order of the later addition does not
// matter), handed to workgroup 0 through tagged words (see asl_internal.h: four words per
// workgroup carry the 64-bit partial numerator in pieces of 28 bits and the partial union count).
// Workgroup 0 waits for all of them, adds them up and performs the single division, the comparison
// with tau and the state update; the other workgroups wait for nobody, so the launch needs no
// particular residency.  Every workgroup reads the old state before it publishes, and workgroup 0
// writes the state only after it has seen every publication.
__global__ void __launch_bounds__(kVarThreads)
rankvar_kernel(const int32_t* __restrict__ ring, int l_obs, int T, int layer_idx, int k, double tau, int push,
               asl_state* state, asl_stat* out, unsigned long long* __restrict__ table,
               unsigned long long* __restrict__ epoch, uint32_t* __restrict__ fault) {
  __shared__ unsigned long long red_num[kVarThreads / 64];
  __shared__ uint32_t red_cnt[kVarThreads / 64];
  __shared__ int gave_up;
  const int tid = threadIdx.x;
  const unsigned long long tag = *epoch + 1ull;
  const int n = rows_in_use(state, layer_idx, l_obs, push);
  unsigned long long num = 0;
  uint32_t cnt = 0;
  if (n >= 2) {
    int row0 = (layer_idx - (n - 1)) % l_obs;            // oldest row in use
    if (row0 < 0) row0 += l_obs;
    for (int t = blockIdx.x * kVarThreads + tid; t < T; t += gridDim.x * kVarThreads) {
      unsigned long long s1 = 0, s2 = 0;
      int mn = 0x7fffffff;
      int row = row0;
#pragma unroll 8
      for (int j = 0; j < n; ++j) {
        const int r = ring[(int64_t)row * T + t];
        row = (row + 1 == l_obs) ? 0 : row + 1;
        s1 += (unsigned long long)r;
        s2 += (unsigned long long)r * (unsigned long long)r;
        mn = r < mn ? r : mn;
      }
      if (mn < k) {
        num += (unsigned long long)n * s2 - s1 * s1;
        cnt += 1;
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    num += __shfl_down(num, o);
    cnt += __shfl_down(cnt, o);
  }
  if ((tid & 63) == 0) {
    red_num[tid >> 6] = num;
    red_cnt[tid >> 6] = cnt;
  }
  if (tid == 0) gave_up = 0;
  __syncthreads();
  if (tid == 0) {
    unsigned long long bn = 0;
    uint32_t bc = 0;
    for (int w = 0; w < kVarThreads / 64; ++w) {
      bn += red_num[w];
      bc += red_cnt[w];
    }
    unsigned long long* mine = table + (int64_t)blockIdx.x * 4;
    const uint32_t m14 = (1u << kFlagCountBits) - 1u;
    flag_publish(mine + 0, tag, (uint32_t)bn & m14, (uint32_t)(bn >> 14) & m14);
    flag_publish(mine + 1, tag, (uint32_t)(bn >> 28) & m14, (uint32_t)(bn >> 42) & m14);
    flag_publish(mine + 2, tag, (uint32_t)(bn >> 56) & m14, 0u);
    flag_publish(mine + 3, tag, bc & m14, (bc >> 14) & m14);
  }
  if (blockIdx.x != 0) return;

  // workgroup 0: gather every workgroup's partials (thread b takes workgroups b, b + 256, ...)
  __syncthreads();                                   // red_* are reused below
  unsigned long long total = 0;
  uint32_t m = 0;
  for (int b = tid; b < (int)gridDim.x; b += kVarThreads) {
    unsigned long long v[kFlagBatch];
    if (!flag_poll_batch<1>(table + (int64_t)b * 4, 1, 0, 4, tag, v)) gave_up = 1;
    const unsigned long long piece0 = (unsigned long long)flag_count0(v[0]) | ((unsigned long long)flag_count1(v[0]) << 14);
    const unsigned long long piece1 = (unsigned long long)flag_count0(v[1]) | ((unsigned long long)flag_count1(v[1]) << 14);
    total += piece0 | (piece1 << 28) | ((unsigned long long)flag_count0(v[2]) << 56);
    m += flag_count0(v[3]) | (flag_count1(v[3]) << 14);
  }
  for (int o = 32; o > 0; o >>= 1) {
    total += __shfl_down(total, o);
    m += __shfl_down(m, o);
  }
  if ((tid & 63) == 0) {
    red_num[tid >> 6] = total;
    red_cnt[tid >> 6] = m;
  }
  __syncthreads();                                   // every thread has read the old state by now
  if (tid != 0) return;
  if (gave_up) {                                     // a peer never reported: no result, state untouched
    *fault = 1u;
    out->var_top = __builtin_nan("");
    out->rel_var = __builtin_nan("");
    out->numerator = 0;
    out->union_size = 0;
    out->n_rows = n;
    out->evaluated = 0;
    out->selected = 0;
    return;
  }
  *epoch = tag;
  total = 0;
  m = 0;
  for (int w = 0; w < kVarThreads / 64; ++w) {
    total += red_num[w];
    m += red_cnt[w];
  }
  if (push) {
    state->n_valid_rows = n;
    state->last_layer = layer_idx;
  }
  if (n < 2) {
    out->var_top = __builtin_nan("");
    out->rel_var = __builtin_nan("");
    out->numerator = 0;
    out->union_size = 0;
    out->n_rows = n;
    out->evaluated = 0;
    out->selected = 0;
    return;
  }
  // var_top = numerator / (n^2 * |union|): one rounding of the integer, one division
  const double den = (double)((unsigned long long)n * (unsigned long long)n * (unsigned long long)m);
  const double var_top = (m > 0) ? (double)total / den : __builtin_nan("");
  double init = state->init_var;
  if (!state->init_set) {
    init = var_top;
    state->init_var = var_top;
    state->init_set = 1;
  }
  const double rel = var_top / init;
  const int selected = (rel < tau) ? 1 : 0;
  out->var_top = var_top;
  out->rel_var = rel;
  out->numerator = total;
  out->union_size = (int32_t)m;
  out->n_rows = n;
  out->evaluated = 1;
  out->selected = selected;
  if (selected) state->n_valid_rows = 0;             // release the rank cache
}

hipError_t launch_stat_skip(Prof* prof, asl_stat* out, asl_state* state, int layer_idx, int l_obs,
                            int push, hipStream_t st) {
  ASL_LAUNCH(prof, kKernRankvarFinal, st, stat_skip_kernel, dim3(1), dim3(64), 0, st, out, state, layer_idx,
             l_obs, push);
  return hipGetLastError();
}

hipError_t launch_rankvar(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx,
                          int k, double tau, int push, asl_state* state, asl_stat* out, hipStream_t st) {
  int blocks = (T + kVarThreads - 1) / kVarThreads;
  if (blocks > kVarMaxBlocks) blocks = kVarMaxBlocks;
  ASL_LAUNCH(ws.prof, kKernRankvar, st, rankvar_kernel, dim3(blocks), dim3(kVarThreads), 0, st, ring, l_obs, T,
             layer_idx, k, tau, push, state, out, ws.var_table, ws.var_epoch, ws.fault);
  return hipGetLastError();
}

}  // namespace asl
