// asl_select: the k highest-scoring past tokens of each row, ties to the lower index, written in
// ascending token order and followed by the window tokens (Alg. 1 steps 9-10 per KV head;
// Alg. 2 steps 11-12 on the all-head scores).
//
// Exact selection in three small launches that read the scores once and never wait for each other:
//  1. guess    one workgroup per row looks at an evenly strided sample of the row (read from the
//              scores, or left behind in compact form by the pooling kernel that produced them)
//              and takes the sample's m-th smallest key (keys are an order-preserving transform of the scores,
//              ascending key = descending score) as a bound that, with m a few standard deviations
//              above the expected number of top-k members in the sample, admits at least k keys
//              of the row and not many more;
//  2. filter   one workgroup per tile of 4096 tokens keeps the tile's keys <= the bound, in token
//              order, in the tile's own segment of a candidate buffer (no offsets to agree on);
//  3. finish   one workgroup per row loads the row's candidates (a few thousand) into LDS, finds
//              the k-th smallest key among them by radix select, and writes the kept tokens in
//              order.
// The bound is only a guess: if fewer than k keys passed it, or a tile's or the row's candidates
// do not fit their buffers, step 3 runs the same selection over the whole row straight from the
// scores instead (slower, same result).  The result therefore never depends on the sample.
// Integer work throughout: nothing depends on scheduling.
#include "select_body.h"

namespace asl {

__global__ void __launch_bounds__(kFinThreads) select_guess_kernel(SelectArgs a) {
  __shared__ GuessShared sh;
  select_guess_body(sh, a, (int)blockIdx.x);
}

// grid: x = tile, y = row.  Small workgroups when there are enough tiles to fill the device several
// times over (a workgroup lives ~5 us whatever its size: more of them in flight stream faster), large
// ones for a few rows (one round of workgroups: the shorter each one's share, the sooner it ends).
template <int NT, bool VEC>
__global__ void __launch_bounds__(NT) select_filter_kernel(SelectArgs a) {
  __shared__ FilterShared sh;
  select_filter_body<NT, VEC>(sh, a, (int)blockIdx.y, (int)blockIdx.x);
}

// dynamic LDS: kFinishLdsBytes
__global__ void __launch_bounds__(kFinThreads) select_finish_kernel(SelectArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  FinishShared& sh = *reinterpret_cast<FinishShared*>(lds_dyn);
  select_finish_body(sh, reinterpret_cast<uint32_t*>(lds_dyn + sizeof(FinishShared)), a, (int)blockIdx.x);
}

SelectArgs select_args(const Workspace& ws, const float* scores, int T, int k, int W, int32_t* idx_out,
                       bool have_sample) {
  SelectArgs a = {};
  a.scores = scores;
  a.sample = have_sample ? ws.sel_sample : nullptr;
  a.T = T;
  a.n_tiles = (T + kSelTile - 1) / kSelTile;
  a.k = k;
  a.W = W;
  a.bound = ws.sel_bound;
  a.thr = ws.sel_thr;
  a.cand_key = ws.sel_cand_key;
  a.cand_idx = ws.sel_cand_idx;
  a.seg_count = ws.sel_seg_count;
  a.idx_out = idx_out;
  return a;
}

hipError_t launch_select(const Workspace& ws, const float* scores, int rows, int T, int k, int W,
                         int32_t* idx_out, hipStream_t st) {
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(select_finish_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFinishLdsBytes);
  if (attr != hipSuccess) return attr;
  // rows beyond what the candidate buffers hold at once take further rounds of the three launches
  const int rows_per_round = ws.sel_rows;
  for (int row0 = 0; row0 < rows; row0 += rows_per_round) {
    const int nr = rows - row0 < rows_per_round ? rows - row0 : rows_per_round;
    const SelectArgs a = select_args(ws, scores + (int64_t)row0 * T, T, k, W, idx_out + (int64_t)row0 * (k + W), false);
    ASL_LAUNCH(ws.prof, kKernSelHist, st, select_guess_kernel, dim3(nr), dim3(kFinThreads), 0, st, a);
    // rows that start on 16-byte boundaries are read four scores at a time
    const bool vec = (T % 4 == 0) && (reinterpret_cast<uintptr_t>(a.scores) % 16 == 0);
    const bool small = (long)a.n_tiles * nr >= kFilterSmallFrom;
    const dim3 fgrid(a.n_tiles, nr);
    if (small && vec)
      ASL_LAUNCH(ws.prof, kKernSelHist, st, (select_filter_kernel<kFilterThreads, true>), fgrid, dim3(kFilterThreads), 0, st, a);
    else if (small)
      ASL_LAUNCH(ws.prof, kKernSelHist, st, (select_filter_kernel<kFilterThreads, false>), fgrid, dim3(kFilterThreads), 0, st, a);
    else if (vec)
      ASL_LAUNCH(ws.prof, kKernSelHist, st, (select_filter_kernel<kFinThreads, true>), fgrid, dim3(kFinThreads), 0, st, a);
    else
      ASL_LAUNCH(ws.prof, kKernSelHist, st, (select_filter_kernel<kFinThreads, false>), fgrid, dim3(kFinThreads), 0, st, a);
    ASL_LAUNCH(ws.prof, kKernSelWrite, st, select_finish_kernel, dim3(nr), dim3(kFinThreads), kFinishLdsBytes, st, a);
  }
  return hipGetLastError();
}

}  // namespace asl
