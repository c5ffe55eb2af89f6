// asl_gather: KV compaction K[I], V[I] (Alg. 1 step 12 of the paper).  A bit copy: each thread
// moves 16-byte pieces of output rows, so a wavefront reads and writes whole contiguous rows
// (64 lanes x 16 B = four 256-byte rows for d = 128 bf16).  One launch covers K and V of every KV
// head and, for the many-layer call, of every layer (each layer's cache being its own allocation,
// named by a device array of pointers).
#include "gather_body.h"

namespace asl {

// grid: x = blocks of kGatherThreads * kGatherUnroll pieces of one (head, tensor, layer) slab,
//       y = KV head, z = layer * n_tensors + tensor (0 = K, 1 = V).
template <bool POW2>
__global__ void __launch_bounds__(kGatherThreads)
gather_kernel(GatherArgs a) {
  gather_body<POW2, kGatherThreads>(a, (int)blockIdx.x, (int)blockIdx.y, (int)(blockIdx.z % (unsigned)a.n_tensors),
                                    (int)(blockIdx.z / (unsigned)a.n_tensors));
}

// Sets cpr_shift; returns whether the pieces per row are a power of two.
bool gather_prepare(GatherArgs& a) {
  a.cpr_shift = 0;
  const bool pow2 = (a.cpr & (a.cpr - 1)) == 0;
  if (pow2)
    while ((1 << a.cpr_shift) < a.cpr) ++a.cpr_shift;
  return pow2;
}

hipError_t launch_gather(Prof* prof, const GatherArgs& args, int Hk, int n_layers, hipStream_t st) {
  GatherArgs a = args;
  const int64_t total = (int64_t)a.n_idx * a.cpr;
  if (total == 0 || Hk == 0 || n_layers == 0) return hipSuccess;
  if (total >= (int64_t(1) << 31) || Hk > 65535 || (int64_t)n_layers * a.n_tensors > 65535)
    return hipErrorInvalidValue;
  const int per_block = kGatherThreads * kGatherUnroll;
  const dim3 grid((unsigned)((total + per_block - 1) / per_block), (unsigned)Hk, (unsigned)(n_layers * a.n_tensors));
  const bool pow2 = gather_prepare(a);
  if (pow2)
    ASL_LAUNCH(prof, kKernGather, st, gather_kernel<true>, grid, dim3(kGatherThreads), 0, st, a);
  else
    ASL_LAUNCH(prof, kKernGather, st, gather_kernel<false>, grid, dim3(kGatherThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace asl
