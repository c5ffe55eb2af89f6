// asl_rankvar: the relative rank-variance statistic and the selection-layer decision
// (Alg. 2 steps 4-10 of the paper; Sec. 4.1 top(L), var_top and relative-variance equations).
//
// Ranks are a permutation, so "the k smallest ranks of a row" is rank < k and the union over rows
// is  min_l R[l,t] < k.  Per token the population variance times n^2 is the integer
// n * sum R^2 - (sum R)^2; the sum over the union is accumulated exactly in 64-bit integers
// (per-workgroup partials; integer sums are order-independent); workgroup 0 of the same launch adds
// the partials and performs the single double-precision division, the comparison with tau and the
// state update.  No read-modify-write atomics, no fences.
#include "rankvar_body.h"

namespace asl {

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

__global__ void __launch_bounds__(kVarThreads) rankvar_kernel(RankvarArgs a) {
  __shared__ RankvarShared sh;
  rankvar_body(sh, a, (int)blockIdx.x, (int)gridDim.x);
}

hipError_t launch_stat_skip(Prof* prof, asl_stat* out, asl_state* state, int layer_idx, int l_obs,
                            int push, hipStream_t st) {
  ASL_LAUNCH(prof, kKernRankvarFinal, st, stat_skip_kernel, dim3(1), dim3(64), 0, st, out, state, layer_idx,
             l_obs, push);
  return hipGetLastError();
}

int rankvar_blocks(int T) {
  int blocks = (T + kVarThreads - 1) / kVarThreads;
  return blocks > kVarMaxBlocks ? kVarMaxBlocks : blocks;
}

RankvarArgs rankvar_args(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx, int k, double tau,
                         int push, asl_state* state, asl_stat* out) {
  RankvarArgs a = {};
  a.ring = ring;
  a.l_obs = l_obs;
  a.T = T;
  a.layer_idx = layer_idx;
  a.k = k;
  a.tau = tau;
  a.push = push;
  a.state = state;
  a.out = out;
  a.table = ws.var_table;
  a.epoch = ws.var_epoch;
  a.fault = ws.fault;
  return a;
}

hipError_t launch_rankvar(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx,
                          int k, double tau, int push, asl_state* state, asl_stat* out, hipStream_t st) {
  ASL_LAUNCH(ws.prof, kKernRankvar, st, rankvar_kernel, dim3(rankvar_blocks(T)), dim3(kVarThreads), 0, st,
             rankvar_args(ws, ring, l_obs, T, layer_idx, k, tau, push, state, out));
  return hipGetLastError();
}

}  // namespace asl
