// asl_gather: KV compaction K[I], V[I] (Alg. 1 step 12 of the paper).  A bit copy: each thread
// moves 16-byte pieces of output rows, so a wavefront reads and writes whole contiguous rows
// (64 lanes x 16 B = four 256-byte rows for d = 128 bf16).  One launch covers K and V of every KV
// head and, for the many-layer call, of every layer (each layer's cache being its own allocation,
// named by a device array of pointers).
#include "asl_internal.h"

namespace asl {

constexpr int kGatherThreads = 256;
constexpr int kGatherUnroll = 4;      // pieces per thread, all loads in flight before the first store

// grid: x = blocks of kGatherThreads * kGatherUnroll pieces of one (head, tensor, layer) slab,
//       y = KV head, z = layer * n_tensors + tensor (0 = K, 1 = V).
// Pieces of a slab are numbered q = row * cpr + c (row = output row, c = 16-byte piece of the row).
template <bool POW2>
__global__ void __launch_bounds__(kGatherThreads)
gather_kernel(GatherArgs a) {
  const int h = blockIdx.y;
  const int which = (int)(blockIdx.z % (unsigned)a.n_tensors);
  const int layer = (int)(blockIdx.z / (unsigned)a.n_tensors);
  const char* src_base;
  char* dst_base;
  if (a.k_ptrs != nullptr) {                        // per-layer allocations
    src_base = static_cast<const char*>(which == 0 ? a.k_ptrs[layer] : a.v_ptrs[layer]);
    dst_base = static_cast<char*>(which == 0 ? a.k_out_ptrs[layer] : a.v_out_ptrs[layer]);
  } else {
    src_base = which == 0 ? a.k : a.v;
    dst_base = which == 0 ? a.k_out : a.v_out;
  }
  const int64_t sh = which == 0 ? a.ksh : a.vsh, stt = which == 0 ? a.kst : a.vst;
  src_base += (int64_t)h * sh;
  dst_base += (int64_t)h * a.n_idx * ((int64_t)a.cpr * 16);
  const int32_t* idx = a.idx + ((int64_t)layer * a.idx_rows + (a.idx_rows == 1 ? 0 : h)) * a.n_idx;
  const uint32_t total = (uint32_t)a.n_idx * (uint32_t)a.cpr;          // < 2^31, checked by the host
  const uint32_t q0 = blockIdx.x * (kGatherThreads * kGatherUnroll) + threadIdx.x;
  uint32_t row[kGatherUnroll], c[kGatherUnroll];
  int tok[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const uint32_t q = q0 + u * kGatherThreads;
    row[u] = POW2 ? (q >> a.cpr_shift) : (q / (uint32_t)a.cpr);
    c[u] = POW2 ? (q & ((uint32_t)a.cpr - 1u)) : (q - row[u] * (uint32_t)a.cpr);
    tok[u] = (q < total) ? idx[row[u]] : 0;
  }
  uint4 val[kGatherUnroll];
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const uint32_t q = q0 + u * kGatherThreads;
    if (q < total) val[u] = *reinterpret_cast<const uint4*>(src_base + (int64_t)tok[u] * stt + c[u] * 16);
  }
#pragma unroll
  for (int u = 0; u < kGatherUnroll; ++u) {
    const uint32_t q = q0 + u * kGatherThreads;
    if (q < total) *reinterpret_cast<uint4*>(dst_base + (int64_t)q * 16) = val[u];
  }
}

hipError_t launch_gather(Prof* prof, const GatherArgs& args, int Hk, int n_layers, hipStream_t st) {
  GatherArgs a = args;
  const int64_t total = (int64_t)a.n_idx * a.cpr;
  if (total == 0 || Hk == 0 || n_layers == 0) return hipSuccess;
  if (total >= (int64_t(1) << 31) || Hk > 65535 || (int64_t)n_layers * a.n_tensors > 65535)
    return hipErrorInvalidValue;
  const int per_block = kGatherThreads * kGatherUnroll;
  const dim3 grid((unsigned)((total + per_block - 1) / per_block), (unsigned)Hk, (unsigned)(n_layers * a.n_tensors));
  a.cpr_shift = 0;
  const bool pow2 = (a.cpr & (a.cpr - 1)) == 0;
  if (pow2)
    while ((1 << a.cpr_shift) < a.cpr) ++a.cpr_shift;
  if (pow2)
    ASL_LAUNCH(prof, kKernGather, st, gather_kernel<true>, grid, dim3(kGatherThreads), 0, st, a);
  else
    ASL_LAUNCH(prof, kKernGather, st, gather_kernel<false>, grid, dim3(kGatherThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace asl
