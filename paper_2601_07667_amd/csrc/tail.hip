// The part of a layer step that follows the scoring, in four launches on one stream.
//
// After the scores are pooled two independent chains remain: the ranking sort (four dependent
// passes, Alg. 1 step 11) and the top-k + KV compaction (bound, filter, finish, gather: Alg. 1
// steps 9-10 and 12; Alg. 2 steps 11-12).  Run as separate launches they either serialise (one
// stream) or pay two cross-queue synchronisations per layer (two streams).  Here launch i hosts
// pass i of the sort in its first workgroups and stage i of the other chain in the remaining ones:
// the two jobs of a launch are independent, and stage i depends only on stage i-1, which the
// launch boundary orders.  The bodies are the same device functions the single-call kernels use.
#include "gather_body.h"
#include "rank_body.h"
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

// launch 1: sort pass 1 | top-k filter (one workgroup per tile of a score row)
template <int R>
__global__ void __launch_bounds__(kTailThreads) tail1_kernel(SortArgs sa, SelectArgs se) {
  __shared__ SortFilterShared sh;
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, false>(sh.sort, sa, b);
  } else {
    const int j = b - sa.n_tiles;
    select_filter_body(sh.filter, se, j / se.n_tiles, j % se.n_tiles);
  }
}

// launch 2: sort pass 2 | top-k finish (one workgroup per score row); dynamic LDS kSortFinishLdsBytes
template <int R>
__global__ void __launch_bounds__(kTailThreads) tail2_kernel(SortArgs sa, SelectArgs se) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, false>(*reinterpret_cast<SortShared*>(lds_dyn), sa, b);
  } else {
    FinishShared& sh = *reinterpret_cast<FinishShared*>(lds_dyn);
    select_finish_body(sh, reinterpret_cast<uint32_t*>(lds_dyn + sizeof(FinishShared)), se, b - sa.n_tiles);
  }
}

// launch 3: sort pass 3 (writes the ranks) | KV compaction with the per-head indices of launch 2
// (gx blocks per (head, tensor) slab; absent when gx == 0)
template <int R, bool POW2>
__global__ void __launch_bounds__(kTailThreads) tail3_kernel(SortArgs sa, GatherArgs ga, int gx, int Hk) {
  __shared__ SortShared sh;
  const int b = (int)blockIdx.x;
  if (b < sa.n_tiles) {
    sort_pass_body<R, false, true>(sh, sa, b);
  } else {
    const int j = b - sa.n_tiles;
    const int bx = j % gx, hw = j / gx;
    gather_body<POW2, kTailThreads>(ga, bx, hw % Hk, hw / Hk, 0);
  }
}

// Sort tiles (workgroups that wait for each other) one of these launches may have on this device.
template <int R>
static int tail_max_tiles() {
  static const int n = [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tail2_kernel<R>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kSortFinishLdsBytes);
    int m = kSortMaxTiles;
    const int c[] = {coresident_limit(tail0_kernel<R>, kTailThreads), coresident_limit(tail1_kernel<R>, kTailThreads),
                     coresident_limit(tail2_kernel<R>, kTailThreads, 1024, kSortFinishLdsBytes),
                     coresident_limit(tail3_kernel<R, true>, kTailThreads),
                     coresident_limit(tail3_kernel<R, false>, kTailThreads)};
    for (int v : c) m = v < m ? v : m;
    return m;
  }();
  return n;
}

template <int R>
static hipError_t launch_tail_r(const Workspace& ws, const float* scores, int rows, int T, int n_tiles, int k, int W,
                                int32_t* rank_row, int32_t* idx_out, const GatherArgs* gather, int Hk, bool have_sample,
                                hipStream_t st) {
  const float* s_all = scores + (int64_t)(rows - 1) * T;       // the all-head row is the last one
  const SelectArgs se = select_args(ws, scores, T, k, W, idx_out, have_sample);
  const dim3 block(kTailThreads);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail0_kernel<R>), dim3(n_tiles + rows), block, 0, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 0), se);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail1_kernel<R>), dim3(n_tiles + rows * se.n_tiles), block, 0, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 1), se);
  ASL_LAUNCH(ws.prof, kKernTail, st, (tail2_kernel<R>), dim3(n_tiles + rows), block, kSortFinishLdsBytes, st,
             sort_pass_args(ws, s_all, T, n_tiles, rank_row, 2), se);
  GatherArgs ga = {};
  int gx = 0;
  bool pow2 = true;
  if (gather != nullptr) {
    ga = *gather;
    pow2 = gather_prepare(ga);
    const int64_t total = (int64_t)ga.n_idx * ga.cpr;
    const int per_block = kTailThreads * kGatherUnroll;
    gx = (int)((total + per_block - 1) / per_block);
  }
  const dim3 grid3(n_tiles + gx * Hk * (gather ? ga.n_tensors : 0));
  if (pow2)
    ASL_LAUNCH(ws.prof, kKernTail, st, (tail3_kernel<R, true>), grid3, block, 0, st,
               sort_pass_args(ws, s_all, T, n_tiles, rank_row, 3), ga, gx, Hk);
  else
    ASL_LAUNCH(ws.prof, kKernTail, st, (tail3_kernel<R, false>), grid3, block, 0, st,
               sort_pass_args(ws, s_all, T, n_tiles, rank_row, 3), ga, gx, Hk);
  return hipGetLastError();
}

// Ranks scores' last row into rank_row, selects the top-k of all `rows` rows into idx_out and, if
// `gather` is given, compacts K/V with the first Hk index rows.  *taken = false (and nothing is
// launched) when the sizes do not fit these launches; the caller then issues the single calls.
bool tail_takes(const Workspace& ws, int rows, int T) {
  if (rows > ws.sel_rows) return false;
  const SortPlan small = sort_plan(T, tail_max_tiles<kSortRounds>());
  if (small.n_tiles > 0 && !small.big) return true;
  const int big_tile = kSortThreads * kSortRoundsBig;
  return (T + big_tile - 1) / big_tile <= tail_max_tiles<kSortRoundsBig>();
}

hipError_t launch_tail(const Workspace& ws, const float* scores, int rows, int T, int k, int W, int32_t* rank_row,
                       int32_t* idx_out, const GatherArgs* gather, int Hk, bool have_sample, hipStream_t st,
                       bool* taken) {
  *taken = false;
  if (rows > ws.sel_rows) return hipSuccess;
  if (gather != nullptr && ((int64_t)gather->n_idx * gather->cpr >= (int64_t(1) << 31))) return hipSuccess;
  const SortPlan small = sort_plan(T, tail_max_tiles<kSortRounds>());
  if (small.n_tiles > 0 && !small.big) {
    *taken = true;
    return launch_tail_r<kSortRounds>(ws, scores, rows, T, small.n_tiles, k, W, rank_row, idx_out, gather, Hk, have_sample, st);
  }
  const int big_tile = kSortThreads * kSortRoundsBig;
  const int n_big = (T + big_tile - 1) / big_tile;
  if (n_big <= tail_max_tiles<kSortRoundsBig>()) {
    *taken = true;
    return launch_tail_r<kSortRoundsBig>(ws, scores, rows, T, n_big, k, W, rank_row, idx_out, gather, Hk, have_sample, st);
  }
  return hipSuccess;
}

}  // namespace asl
