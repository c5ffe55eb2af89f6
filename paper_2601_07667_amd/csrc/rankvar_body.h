// Device code of the rank-variance kernel (see rankvar.hip for the method), written as a function
// over an explicit shared-state struct so that another kernel can host it beside a second body.
#pragma once
#include "asl_internal.h"

namespace asl {

constexpr int kVarThreads = 256;
constexpr int kVarTok = 2;                  // tokens per thread whose ranks are in flight together ...
constexpr int kVarRowBatch = 8;             // ... and ring rows of each

// The ring row of layer_idx continues the rows already held iff layer_idx is the layer after
// state->last_layer, or that layer minus l_obs (a captured trip of l_obs layers round the ring being
// replayed: the same rows are overwritten in the same order).  Any other index restarts the ring.
__device__ __forceinline__ bool continues_ring(const asl_state* state, int layer_idx, int l_obs) {
  const int next = state->last_layer + 1;
  return layer_idx == next || layer_idx == next - l_obs;
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

struct RankvarShared {
  unsigned long long red_num[kVarThreads / 64];
  uint32_t red_cnt[kVarThreads / 64];
  int gave_up;
};

struct RankvarArgs {
  const int32_t* ring;           // [l_obs][T]
  int l_obs, T, layer_idx, k;
  double tau;
  int push;
  asl_state* state;
  asl_stat* out;
  unsigned long long* table;     // [kVarMaxBlocks][4] tagged partial sums
  unsigned long long* epoch;
  uint32_t* fault;
};

// Per-workgroup partial sums over the union (integers, so the order of the later addition does not
// matter), handed to workgroup 0 through tagged words (see asl_internal.h: four words per
// workgroup carry the 64-bit partial numerator in pieces of 28 bits and the partial union count).
// Workgroup 0 waits for all of them, adds them up and performs the single division, the comparison
// with tau and the state update; the other workgroups wait for nobody, so the launch needs no
// particular residency.  Every workgroup reads the old state before it publishes, and workgroup 0
// writes the state only after it has seen every publication.
__device__ __forceinline__ void rankvar_body(RankvarShared& sh, const RankvarArgs& a, int block, int n_blocks) {
  const int tid = threadIdx.x;
  const unsigned long long tag = *a.epoch + 1ull;
  const int n = rows_in_use(a.state, a.layer_idx, a.l_obs, a.push);
  unsigned long long num = 0;
  uint32_t cnt = 0;
  if (n >= 2) {
    int row0 = (a.layer_idx - (n - 1)) % a.l_obs;            // oldest row in use
    if (row0 < 0) row0 += a.l_obs;
    // kVarTok tokens per thread and kVarRowBatch rows of each are read together: the loads of such a
    // step are issued before any is waited for, whatever n is (rows beyond n and tokens beyond T
    // re-read a valid element and are left out of the sums).
    const int stride = n_blocks * kVarThreads;
    for (int t0 = block * kVarThreads + tid; t0 < a.T; t0 += kVarTok * stride) {
      unsigned long long s1[kVarTok], s2[kVarTok];
      int mn[kVarTok];
#pragma unroll
      for (int q = 0; q < kVarTok; ++q) {
        s1[q] = 0;
        s2[q] = 0;
        mn[q] = 0x7fffffff;
      }
      for (int j0 = 0; j0 < n; j0 += kVarRowBatch) {
        int r[kVarTok][kVarRowBatch];
#pragma unroll
        for (int u = 0; u < kVarRowBatch; ++u) {
          int row = row0 + ((j0 + u < n) ? j0 + u : 0);          // < 2 l_obs
          row = (row >= a.l_obs) ? row - a.l_obs : row;
#pragma unroll
          for (int q = 0; q < kVarTok; ++q) {
            const int t = t0 + q * stride;
            r[q][u] = a.ring[(int64_t)row * a.T + (t < a.T ? t : t0)];
          }
        }
#pragma unroll
        for (int u = 0; u < kVarRowBatch; ++u) {
          const int keep = (j0 + u < n) ? -1 : 0;                // all ones or zero, uniform; no branch, so
#pragma unroll                                                   // that every load above stays unconditional
          for (int q = 0; q < kVarTok; ++q) {
            const int v = r[q][u] & keep;                        // ranks are >= 0
            const int vm = r[q][u] | (~keep & 0x7fffffff);
            s1[q] += (unsigned long long)v;
            s2[q] += (unsigned long long)v * (unsigned long long)v;
            mn[q] = vm < mn[q] ? vm : mn[q];
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kVarTok; ++q) {
        if (t0 + q * stride < a.T && mn[q] < a.k) {
          num += (unsigned long long)n * s2[q] - s1[q] * s1[q];
          cnt += 1;
        }
      }
    }
  }
  num = wave_sum(num);
  cnt = wave_sum(cnt);
  if ((tid & 63) == 0) {
    sh.red_num[tid >> 6] = num;
    sh.red_cnt[tid >> 6] = cnt;
  }
  if (tid == 0) sh.gave_up = 0;
  __syncthreads();
  if (tid == 0) {
    unsigned long long bn = 0;
    uint32_t bc = 0;
    for (int w = 0; w < kVarThreads / 64; ++w) {
      bn += sh.red_num[w];
      bc += sh.red_cnt[w];
    }
    unsigned long long* mine = a.table + (int64_t)block * 4;
    const uint32_t m14 = (1u << kFlagCountBits) - 1u;
    flag_publish(mine + 0, tag, (uint32_t)bn & m14, (uint32_t)(bn >> 14) & m14);
    flag_publish(mine + 1, tag, (uint32_t)(bn >> 28) & m14, (uint32_t)(bn >> 42) & m14);
    flag_publish(mine + 2, tag, (uint32_t)(bn >> 56) & m14, 0u);
    flag_publish(mine + 3, tag, bc & m14, (bc >> 14) & m14);
  }
  if (block != 0) return;

  // workgroup 0: gather every workgroup's partials (thread b takes workgroups b, b + 256, ...)
  __syncthreads();                                   // red_* are reused below
  unsigned long long total = 0;
  uint32_t m = 0;
  for (int b = tid; b < n_blocks; b += kVarThreads) {
    unsigned long long v[kFlagBatch];
    if (!flag_poll_batch<1>(a.table + (int64_t)b * 4, 1, 0, 4, tag, v)) sh.gave_up = 1;
    const unsigned long long piece0 = (unsigned long long)flag_count0(v[0]) | ((unsigned long long)flag_count1(v[0]) << 14);
    const unsigned long long piece1 = (unsigned long long)flag_count0(v[1]) | ((unsigned long long)flag_count1(v[1]) << 14);
    total += piece0 | (piece1 << 28) | ((unsigned long long)flag_count0(v[2]) << 56);
    m += flag_count0(v[3]) | (flag_count1(v[3]) << 14);
  }
  total = wave_sum(total);
  m = wave_sum(m);
  if ((tid & 63) == 0) {
    sh.red_num[tid >> 6] = total;
    sh.red_cnt[tid >> 6] = m;
  }
  __syncthreads();                                   // every thread has read the old state by now
  if (tid != 0) return;
  if (sh.gave_up) {                                     // a peer never reported: no result, state untouched
    *a.fault = 1u;
    a.out->var_top = __builtin_nan("");
    a.out->rel_var = __builtin_nan("");
    a.out->numerator = 0;
    a.out->union_size = 0;
    a.out->n_rows = n;
    a.out->evaluated = 0;
    a.out->selected = 0;
    return;
  }
  *a.epoch = tag;
  total = 0;
  m = 0;
  for (int w = 0; w < kVarThreads / 64; ++w) {
    total += sh.red_num[w];
    m += sh.red_cnt[w];
  }
  if (a.push) {
    a.state->n_valid_rows = n;
    a.state->last_layer = a.layer_idx;
  }
  if (n < 2) {
    a.out->var_top = __builtin_nan("");
    a.out->rel_var = __builtin_nan("");
    a.out->numerator = 0;
    a.out->union_size = 0;
    a.out->n_rows = n;
    a.out->evaluated = 0;
    a.out->selected = 0;
    return;
  }
  // var_top = numerator / (n^2 * |union|): one rounding of the integer, one division
  const double den = (double)((unsigned long long)n * (unsigned long long)n * (unsigned long long)m);
  const double var_top = (m > 0) ? (double)total / den : __builtin_nan("");
  double init = a.state->init_var;
  if (!a.state->init_set) {
    init = var_top;
    a.state->init_var = var_top;
    a.state->init_set = 1;
  }
  const double rel = var_top / init;
  const int selected = (rel < a.tau) ? 1 : 0;
  a.out->var_top = var_top;
  a.out->rel_var = rel;
  a.out->numerator = total;
  a.out->union_size = (int32_t)m;
  a.out->n_rows = n;
  a.out->evaluated = 1;
  a.out->selected = selected;
  if (selected) a.state->n_valid_rows = 0;             // release the rank cache
}

// Workgroups of the statistic over T tokens and its argument block.
int rankvar_blocks(int T);
RankvarArgs rankvar_args(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx, int k, double tau,
                         int push, asl_state* state, asl_stat* out);

}  // namespace asl
