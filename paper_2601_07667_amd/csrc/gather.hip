// asl_gather: KV compaction K[I], V[I] (Alg. 1 step 12 of the paper).  A bit copy: each thread
// moves one 16-byte piece of an output row, so a wavefront reads and writes whole contiguous
// rows (64 lanes x 16 B = four 256-byte rows for d = 128 bf16).
#include "asl_internal.h"

namespace asl {

__global__ void __launch_bounds__(256)
gather_kernel(const char* __restrict__ k, const char* __restrict__ v, const int32_t* __restrict__ idx,
              int idx_rows, int n_idx, int Hk, int cpr /* 16-byte pieces per row */,
              int64_t ksh, int64_t kst, int64_t vsh, int64_t vst, char* __restrict__ k_out,
              char* __restrict__ v_out, int n_tensors) {
  const int64_t per_tensor = (int64_t)Hk * n_idx * cpr;
  const int64_t total = per_tensor * n_tensors;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total;
       q += (int64_t)gridDim.x * blockDim.x) {
    const int which = (int)(q / per_tensor);
    const int64_t r = q - which * per_tensor;
    const int c = (int)(r % cpr);
    const int64_t orow = r / cpr;                   // h * n_idx + i
    const int i = (int)(orow % n_idx);
    const int h = (int)(orow / n_idx);
    const int tok = idx[(idx_rows == 1 ? 0 : (int64_t)h * n_idx) + i];
    const char* src = which == 0 ? k + h * ksh + (int64_t)tok * kst : v + h * vsh + (int64_t)tok * vst;
    char* dst = (which == 0 ? k_out : v_out) + orow * ((int64_t)cpr * 16);
    *reinterpret_cast<uint4*>(dst + c * 16) = *reinterpret_cast<const uint4*>(src + c * 16);
  }
}

hipError_t launch_gather(Prof* prof, const void* k, const void* v, const int32_t* idx, int idx_rows, int n_idx,
                         int Hk, int row_bytes, int64_t ksh_b, int64_t kst_b, int64_t vsh_b,
                         int64_t vst_b, void* k_out, void* v_out, hipStream_t st) {
  const int cpr = row_bytes / 16;
  const int n_tensors = (v != nullptr) ? 2 : 1;
  const int64_t total = (int64_t)Hk * n_idx * cpr * n_tensors;
  if (total == 0) return hipSuccess;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  ASL_LAUNCH(prof, kKernGather, st, gather_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const char*)k,
                     (const char*)v, idx, idx_rows, n_idx, Hk, cpr, ksh_b, kst_b, vsh_b, vst_b,
                     (char*)k_out, (char*)v_out, n_tensors);
  return hipGetLastError();
}

}  // namespace asl
