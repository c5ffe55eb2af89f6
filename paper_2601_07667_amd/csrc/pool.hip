// asl_pool: AvgPool1D(kernel S, stride 1, zero pad floor(S/2), divisor S) along the token axis
// (Alg. 1 step 7 of the paper), plus the sum of the pooled rows (Sec. 4.1 "scores" equation).
#include "asl_internal.h"

namespace asl {

constexpr int kPoolBlock = 256;
constexpr int kPoolMaxHalf = 64;   // S <= 129
constexpr int kPoolRows = 8;       // rows staged together

// A workgroup owns 256 consecutive tokens.  The inputs of up to 8 rows (tile + halo) are staged in
// LDS with coalesced loads, so every input is read from memory once and its S taps come from LDS;
// rows are summed in a fixed order.
__global__ void __launch_bounds__(kPoolBlock)
pool_kernel(const float* __restrict__ u, int rows, int T, int S, float* __restrict__ p_out,
            float* __restrict__ s_out) {
  __shared__ float tile[kPoolRows][kPoolBlock + 2 * kPoolMaxHalf];
  const int h = S / 2;
  const int base = blockIdx.x * kPoolBlock;
  const int t = base + threadIdx.x;
  const int span = kPoolBlock + 2 * h;
  const float fS = (float)S;
  float total = 0.f;
  for (int row0 = 0; row0 < rows; row0 += kPoolRows) {
    const int nr = min(kPoolRows, rows - row0);
    __syncthreads();                                   // previous group's reads are done
    for (int r = 0; r < nr; ++r) {
      const float* ur = u + (int64_t)(row0 + r) * T;
      for (int i = threadIdx.x; i < span; i += kPoolBlock) {
        const int src = base - h + i;
        tile[r][i] = (src >= 0 && src < T) ? ur[src] : 0.f;     // zero padding
      }
    }
    __syncthreads();
    if (t < T) {
      for (int r = 0; r < nr; ++r) {
        float acc = 0.f;
        for (int d = 0; d < S; ++d) acc += tile[r][threadIdx.x + d];   // delta = -h .. +h in order
        const float p = acc / fS;
        p_out[(int64_t)(row0 + r) * T + t] = p;
        total += p;
      }
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
