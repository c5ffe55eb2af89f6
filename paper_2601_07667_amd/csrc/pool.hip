// asl_pool: AvgPool1D(kernel S, stride 1, zero pad floor(S/2), divisor S) along the token axis
// (Alg. 1 step 7 of the paper), plus the sum of the pooled rows (Sec. 4.1 "scores" equation).
// A workgroup stages 256 outputs' worth of inputs plus the halo in LDS, row by row.
#include "asl_internal.h"

namespace asl {

constexpr int kPoolBlock = 256;
constexpr int kPoolMaxHalf = 64;   // S <= 129

__global__ void __launch_bounds__(kPoolBlock)
pool_kernel(const float* __restrict__ u, int rows, int T, int S, float* __restrict__ p_out,
            float* __restrict__ s_out) {
  __shared__ float tile[kPoolBlock + 2 * kPoolMaxHalf];
  const int h = S / 2;
  const int base = blockIdx.x * kPoolBlock;
  const int t = base + threadIdx.x;
  const float fS = (float)S;
  float total = 0.f;
  for (int row = 0; row < rows; ++row) {
    const float* ur = u + (int64_t)row * T;
    __syncthreads();                                   // previous row's reads are done
    for (int i = threadIdx.x; i < kPoolBlock + 2 * h; i += kPoolBlock) {
      int src = base - h + i;
      tile[i] = (src >= 0 && src < T) ? ur[src] : 0.f;
    }
    __syncthreads();
    if (t < T) {
      float acc = 0.f;
      for (int d = 0; d < S; ++d) acc += tile[threadIdx.x + d];   // delta = -h .. +h in order
      float p = acc / fS;
      p_out[(int64_t)row * T + t] = p;
      total += p;
    }
  }
  if (s_out != nullptr && t < T) s_out[t] = total;
}

hipError_t launch_pool(Prof* prof, const float* u, int rows, int T, int S, float* p_out, float* s_out,
                       hipStream_t st) {
  ASL_LAUNCH(prof, kKernPool, st, pool_kernel, dim3((T + kPoolBlock - 1) / kPoolBlock), dim3(kPoolBlock), 0, st, u,
                     rows, T, S, p_out, s_out);
  return hipGetLastError();
}

}  // namespace asl
