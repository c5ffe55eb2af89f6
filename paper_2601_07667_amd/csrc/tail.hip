// The part of a layer step that follows the scoring, in five launches on one stream.
//
// After the scores are pooled two independent chains remain: the ranking sort (four dependent
// passes, Alg. 1 step 11) and the top-k + KV compaction (bound, filter, finish, gather: Alg. 1
// steps 9-10 and 12; Alg. 2 steps 11-12).  Run as separate launches they either serialise (one
// stream) or pay two cross-queue synchronisations per layer (two streams).  Here launch i (0..3)
// hosts pass i of the sort in its first workgroups and stage i of the other chain (bound, filter,
// threshold, index write) in the remaining ones, and a fifth launch hosts the rank-variance
// statistic (Alg. 2 steps 4-10) beside the KV compaction: the two jobs of a launch are independent,
// and every stage depends only on the previous launch, which the launch boundary orders.  The
// bodies are the same device functions the single-call kernels use.
#include "gather_body.h"
#include "rank_body.h"
#include "rankvar_body.h"
#include "select_body.h"

namespace asl {

static_assert(kSortThreads == kFinThreads, "both jobs of a launch use the same workgroup size");
constexpr int kTailThreads = kSortThreads;

union SortGuessShared {
  SortShared sort;
  GuessShared guess;
};
union SortFilterShared {
  SortShared sort;
  FilterShared filter;
};
constexpr size_t kSortFinishLdsBytes = sizeof(SortShared) > kFinishLdsBytes ? sizeof(SortShared) : kFinishLdsBytes;

// launch 0: sort pass 0 | top-k bound (one workgroup per score row)
template <int R>
__global__ void __launch_bounds__(kTailThreads) tail0_kernel(SortArgs sa, SelectArgs se) {
  __shared__ SortGuessShared sh;
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles)
    sort_pass_body<R, true, false>(sh.sort, sa, b);
  else
    select_guess_body(sh.guess, se, b - sa.n_tiles);
}

// launch 1: sort pass 1 | top-k filter (one workgroup per tile of a score row; VEC: 16-byte loads,
// for rows that start on 16-byte boundaries)
template <int R, bool VEC>
__global__ void __launch_bounds__(kTailThreads) tail1_kernel(SortArgs sa, SelectArgs se) {
  __shared__ SortFilterShared sh;
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, false>(sh.sort, sa, b);
  } else {
    const int j = b - sa.n_tiles;
    select_filter_body<kTailThreads, VEC>(sh.filter, se, j / se.n_tiles, j % se.n_tiles);
  }
}

// launch 2: sort pass 2 | top-k threshold (one workgroup per score row); dynamic LDS kSortFinishLdsBytes
template <int R>
__global__ void __launch_bounds__(kTailThreads) tail2_kernel(SortArgs sa, SelectArgs se) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, false>(*reinterpret_cast<SortShared*>(lds_dyn), sa, b);
  } else {
    FinishShared& sh = *reinterpret_cast<FinishShared*>(lds_dyn);
    select_threshold_body(sh, reinterpret_cast<uint32_t*>(lds_dyn + sizeof(FinishShared)), se, b - sa.n_tiles);
  }
}

// launch 3: sort pass 3 (writes the ranks) | top-k index write (one workgroup per score row);
// dynamic LDS kSortFinishLdsBytes
template <int R>
__global__ void __launch_bounds__(kTailThreads) tail3_kernel(SortArgs sa, SelectArgs se) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, true>(*reinterpret_cast<SortShared*>(lds_dyn), sa, b);
  } else {
    FinishShared& sh = *reinterpret_cast<FinishShared*>(lds_dyn);
    select_write_body(sh, reinterpret_cast<uint32_t*>(lds_dyn + sizeof(FinishShared)), se, b - sa.n_tiles);
  }
}

// launch 4: rank-variance statistic over the ring that now holds this layer's ranks (its first
// n_stat workgroups; workgroup 0 waits for the others) | KV compaction with the per-head indices of
// launch 3 (gx blocks per (head, tensor) slab)
template <bool POW2>
__global__ void __launch_bounds__(kVarThreads) tail4_kernel(RankvarArgs ra, int n_stat, GatherArgs ga, int gx, int Hk) {
  __shared__ RankvarShared sh;
  const int b = (int)blockIdx.x;
  if (b < n_stat) {
    rankvar_body(sh, ra, b, n_stat);
  } else {
    const int j = b - n_stat;
    const int bx = j % gx, hw = j / gx;
    gather_body<POW2, kVarThreads>(ga, bx, hw % Hk, hw / Hk, 0);
  }
}

// Sort tiles (workgroups that wait for each other) one of these launches may have on this device.
template <int R>
static int tail_max_tiles() {
  static const int n = [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tail2_kernel<R>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kSortFinishLdsBytes);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tail3_kernel<R>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kSortFinishLdsBytes);
    int m = kSortMaxTiles;
    const int c[] = {coresident_limit(tail0_kernel<R>, kTailThreads), coresident_limit(tail1_kernel<R, false>, kTailThreads),
                     coresident_limit(tail1_kernel<R, true>, kTailThreads),
                     coresident_limit(tail2_kernel<R>, kTailThreads, 1024, kSortFinishLdsBytes),
                     coresident_limit(tail3_kernel<R>, kTailThreads, 1024, kSortFinishLdsBytes)};
    for (int v : c) m = v < m ? v : m;
    return m;
  }();
  return n;
}

template <int R>
static hipError_t launch_tail_r(const Workspace& ws, const float* scores, int rows, int T, int n_tiles, int k, int W,
                                int32_t* rank_row, int32_t* idx_out, const GatherArgs* gather, int Hk, bool have_sample,
                                const RankvarArgs* stat, hipStream_t st) {
  const float* s_all = scores + (int64_t)(rows - 1) * T;       // the all-head row is the last one
  const SelectArgs se = select_args(ws, scores, T, k, W, idx_out, have_sample);
  const dim3 block(kTailThreads);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail0_kernel<R>), dim3(n_tiles + rows), block, 0, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 0), se);
  if (T % 4 == 0 && reinterpret_cast<uintptr_t>(scores) % 16 == 0)
    ASL_LAUNCH(ws.prof, kKernTail, st, (tail1_kernel<R, true>), dim3(n_tiles + rows * se.n_tiles), block, 0, st,
               sort_pass_args(ws, s_all, T, n_tiles, rank_row, 1), se);
  else
    ASL_LAUNCH(ws.prof, kKernTail, st, (tail1_kernel<R, false>), dim3(n_tiles + rows * se.n_tiles), block, 0, st,
               sort_pass_args(ws, s_all, T, n_tiles, rank_row, 1), se);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail2_kernel<R>), dim3(n_tiles + rows), block, kSortFinishLdsBytes, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 2), se);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail3_kernel<R>), dim3(n_tiles + rows), block, kSortFinishLdsBytes, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 3), se);
  // statistic beside the compaction; either may be absent (a layer below L_min, no output tensors)
  if (stat != nullptr && gather != nullptr) {
    GatherArgs ga = *gather;
    const bool pow2 = gather_prepare(ga);
    const int64_t total = (int64_t)ga.n_idx * ga.cpr;
    const int per_block = kVarThreads * kGatherUnroll;
    const int gx = (int)((total + per_block - 1) / per_block);
    const int n_stat = rankvar_blocks(T);
    const dim3 grid4(n_stat + gx * Hk * ga.n_tensors);
    if (gx == 0)
      ASL_LAUNCH(ws.prof, kKernRankvar, st, (tail4_kernel<true>), dim3(n_stat), dim3(kVarThreads), 0, st, *stat, n_stat, ga, 1, Hk);
    else if (pow2)
      ASL_LAUNCH(ws.prof, kKernTail, st, (tail4_kernel<true>), grid4, dim3(kVarThreads), 0, st, *stat, n_stat, ga, gx, Hk);
    else
      ASL_LAUNCH(ws.prof, kKernTail, st, (tail4_kernel<false>), grid4, dim3(kVarThreads), 0, st, *stat, n_stat, ga, gx, Hk);
  } else if (stat != nullptr) {
    const hipError_t e = launch_rankvar(ws, stat->ring, stat->l_obs, stat->T, stat->layer_idx, stat->k, stat->tau,
                                        stat->push, stat->state, stat->out, st);
    if (e != hipSuccess) return e;
  } else if (gather != nullptr) {
    const hipError_t e = launch_gather(ws.prof, *gather, Hk, 1, st);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

bool tail_takes(const Workspace& ws, int rows, int T) {
  if (rows > ws.sel_rows) return false;
  const SortPlan small = sort_plan(T, tail_max_tiles<kSortRounds>());
  if (small.n_tiles > 0 && !small.big) return true;
  const int big_tile = kSortThreads * kSortRoundsBig;
  return (T + big_tile - 1) / big_tile <= tail_max_tiles<kSortRoundsBig>();
}

hipError_t launch_tail(const Workspace& ws, const float* scores, int rows, int T, int k, int W, int32_t* rank_row,
                       int32_t* idx_out, const GatherArgs* gather, int Hk, bool have_sample, const RankvarArgs* stat,
                       hipStream_t st, bool* taken) {
  *taken = false;
  if (rows > ws.sel_rows) return hipSuccess;
  if (gather != nullptr && ((int64_t)gather->n_idx * gather->cpr >= (int64_t(1) << 31))) return hipSuccess;
  const SortPlan small = sort_plan(T, tail_max_tiles<kSortRounds>());
  if (small.n_tiles > 0 && !small.big) {
    *taken = true;
    return launch_tail_r<kSortRounds>(ws, scores, rows, T, small.n_tiles, k, W, rank_row, idx_out, gather, Hk, have_sample, stat, st);
  }
  const int big_tile = kSortThreads * kSortRoundsBig;
  const int n_big = (T + big_tile - 1) / big_tile;
  if (n_big <= tail_max_tiles<kSortRoundsBig>()) {
    *taken = true;
    return launch_tail_r<kSortRoundsBig>(ws, scores, rows, T, n_big, k, W, rank_row, idx_out, gather, Hk, have_sample, stat, st);
  }
  return hipSuccess;
}

}  // namespace asl
