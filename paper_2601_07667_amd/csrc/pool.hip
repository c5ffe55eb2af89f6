// asl_pool: AvgPool1D(kernel S, stride 1, zero pad floor(S/2), divisor S) along the token axis
// (Alg. 1 step 7 of the paper), plus the sum of the pooled rows (Sec. 4.1 "scores" equation).
// On request the kernel also leaves behind, in compact form, the strided sample of every output row
// from which the top-k that follows takes its bound (so that nobody has to re-read the rows for it).
#include "asl_internal.h"

namespace asl {

constexpr int kPoolBlock = 256;
constexpr int kPoolMaxHalf = 64;   // S <= 129
constexpr int kPoolRows = 8;       // rows staged together

// A workgroup owns 256 consecutive tokens.  The inputs of up to 8 rows (tile + halo) are staged in
// LDS with coalesced loads, so every input is read from memory once and its S taps come from LDS;
// rows are summed in a fixed order.  S_CT: the window length when it is known at compile time (the
// taps of all staged rows are then read from LDS together), 0 for any other length.
template <int S_CT>
__global__ void __launch_bounds__(kPoolBlock)
pool_kernel(const float* __restrict__ u, int rows, int T, int S_any, float* __restrict__ p_out,
            float* __restrict__ s_out, uint32_t* __restrict__ sample, int n_sample, int sample_stride) {
  __shared__ float tile[kPoolRows][kPoolBlock + 2 * kPoolMaxHalf];
  const int S = S_CT > 0 ? S_CT : S_any;
  const int h = S / 2;
  const int base = blockIdx.x * kPoolBlock;
  const int t = base + threadIdx.x;
  const int span = kPoolBlock + 2 * h;
  const float fS = (float)S;
  float total = 0.f;
  // token t is the top-k's sample number t / stride of every row if it sits on the sample grid
  const bool sampled = sample != nullptr && t < T && t % sample_stride == 0 && t / sample_stride < n_sample;
  const int sample_j = sampled ? t / sample_stride : 0;
  for (int row0 = 0; row0 < rows; row0 += kPoolRows) {
    const int nr = min(kPoolRows, rows - row0);
    __syncthreads();                                   // previous group's reads are done
    // all loads of the group are issued before the first LDS store (span <= 2 * kPoolBlock)
    float v0[kPoolRows], v1[kPoolRows];
    const int src0 = base - h + threadIdx.x, src1 = src0 + kPoolBlock;
    const bool in0 = src0 >= 0 && src0 < T;
    const bool in1 = threadIdx.x + kPoolBlock < span && src1 >= 0 && src1 < T;
#pragma unroll
    for (int r = 0; r < kPoolRows; ++r) {
      const float* ur = u + (int64_t)(row0 + min(r, nr - 1)) * T;
      v0[r] = in0 ? ur[src0] : 0.f;                    // zero padding
      v1[r] = in1 ? ur[src1] : 0.f;
    }
#pragma unroll
    for (int r = 0; r < kPoolRows; ++r) {
      tile[r][threadIdx.x] = v0[r];
      if (threadIdx.x + kPoolBlock < span) tile[r][threadIdx.x + kPoolBlock] = v1[r];
    }
    __syncthreads();
    if (t < T) {
      if (S_CT > 0) {
        float p[kPoolRows];
#pragma unroll
        for (int r = 0; r < kPoolRows; ++r) {
          float acc = 0.f;
#pragma unroll
          for (int d = 0; d < S_CT; ++d) acc += tile[r][threadIdx.x + d];   // delta = -h .. +h in order
          p[r] = acc / fS;
        }
#pragma unroll
        for (int r = 0; r < kPoolRows; ++r) {
          if (r < nr) {
            p_out[(int64_t)(row0 + r) * T + t] = p[r];
            if (sampled) sample[(int64_t)(row0 + r) * kSelMaxSample + sample_j] = order_key(p[r]);
            total += p[r];
          }
        }
      } else {
        for (int r = 0; r < nr; ++r) {
          float acc = 0.f;
          for (int d = 0; d < S; ++d) acc += tile[r][threadIdx.x + d];     // delta = -h .. +h in order
          const float p = acc / fS;
          p_out[(int64_t)(row0 + r) * T + t] = p;
          if (sampled) sample[(int64_t)(row0 + r) * kSelMaxSample + sample_j] = order_key(p);
          total += p;
        }
      }
    }
  }
  if (s_out != nullptr && t < T) s_out[t] = total;
  if (sampled) sample[(int64_t)rows * kSelMaxSample + sample_j] = order_key(total);
}

hipError_t launch_pool(Prof* prof, const float* u, int rows, int T, int S, float* p_out, float* s_out,
                       uint32_t* sample, hipStream_t st) {
  const dim3 grid((T + kPoolBlock - 1) / kPoolBlock), block(kPoolBlock);
  if (S == 7)                                          // the paper's pooling window (App. C.2)
    ASL_LAUNCH(prof, kKernPool, st, pool_kernel<7>, grid, block, 0, st, u, rows, T, S, p_out, s_out, sample,
               sel_sample_size(T), sel_sample_stride(T));
  else
    ASL_LAUNCH(prof, kKernPool, st, pool_kernel<0>, grid, block, 0, st, u, rows, T, S, p_out, s_out, sample,
               sel_sample_size(T), sel_sample_stride(T));
  return hipGetLastError();
}

}  // namespace asl
