// asl_score: window-query x all-key softmax scores, column-summed over the window rows and the
// GQA group (Alg. 1 steps 5, 6, 8 of the paper; Sec. 4.1 PA equation before pooling).
//
// For one KV head the G heads x W window rows form M = G*W query rows that all read the same
// keys.  score_j = sum_r exp(l_rj - m_r) / Z_r mixes rows with different normalisers, so the
// final (m_r, Z_r) of every row must be known before rows are added: pass 1 streams K once for
// the row statistics, pass 2 streams K again for the normalised column sums.  When the caller
// hands over the rows' log-sum-exp, pass 1 is skipped.
//
// Work split: a workgroup owns one KV head and a contiguous chunk of keys; wave w owns query rows
// [32w, 32w+32) and keeps their bf16 fragments in registers for the whole kernel; K tiles of 128
// keys are staged through LDS (coalesced 16-byte global loads, padded rows) and every wave reads
// all of them as the other MFMA operand (v_mfma_f32_32x32x16_bf16).  Pass 1 puts keys on the
// accumulator's register axis (row statistics reduce in-lane), pass 2 puts query rows there
// (column sums reduce in-lane).  All reductions have a fixed order: results are deterministic.
#include "asl_internal.h"

namespace asl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KT = 128;                       // keys per LDS tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;           // finite stand-in for "no maximum yet"

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Row of the 32x32 accumulator held by register r of a lane in half `half` (lanes 32..63 = 1).
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// Global -> register staging of one K tile (KT keys x D bf16), 16 bytes per thread per step;
// rows past N are clamped to the last key (they are masked or discarded later).
#define ASL_KTILE_DECL(D, NT)                                                                  \
  constexpr int CPR = (D) / 8;                          /* 16-byte pieces per key row */       \
  constexpr int NLOAD = (KT * CPR + (NT) - 1) / (NT);   /* pieces per thread */                \
  uint4 stage[NLOAD];

#define ASL_KTILE_LOAD(key0)                                                                    \
  _Pragma("unroll") for (int i_ = 0; i_ < NLOAD; ++i_) {                                        \
    const int q_ = tid + i_ * NT;                                                               \
    const int row_ = q_ / CPR, col_ = q_ % CPR;                                                 \
    const int key_ = min((key0) + row_, N - 1);                                                 \
    uint4 v_ = make_uint4(0u, 0u, 0u, 0u);                                                      \
    if (q_ < KT * CPR) v_ = *reinterpret_cast<const uint4*>(kg + (int64_t)key_ * kst + col_ * 8); \
    stage[i_] = v_;                                                                             \
  }

#define ASL_KTILE_STORE()                                                                       \
  _Pragma("unroll") for (int i_ = 0; i_ < NLOAD; ++i_) {                                        \
    const int q_ = tid + i_ * NT;                                                               \
    const int row_ = q_ / CPR, col_ = q_ % CPR;                                                 \
    if (q_ < KT * CPR) *reinterpret_cast<uint4*>(lds_k + row_ * ROW + col_ * 8) = stage[i_];    \
  }

// Query fragments of this wave's 32-row block: lane (ln, half) holds row ln, d = 16*ks + 8*half .. +8.
#define ASL_LOAD_Q_FRAGS()                                                                      \
  bf16x8 qf[KS];                                                                                \
  {                                                                                             \
    const __bf16* qg_ = q_obs + (int64_t)g * M * D + (int64_t)min(qrow, M - 1) * D + half * 8;  \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                         \
      uint4 raw_ = *reinterpret_cast<const uint4*>(qg_ + ks * 16);                              \
      if (qrow >= M) raw_ = make_uint4(0u, 0u, 0u, 0u);     /* padded rows: zero queries */     \
      qf[ks] = __builtin_bit_cast(bf16x8, raw_);                                                \
    }                                                                                           \
  }

// max without NaN canonicalisation (inputs are never NaN here; -inf is fine)
__device__ __forceinline__ float max2(float a, float b) { return a > b ? a : b; }

// ---------------------------------------------------------------------------------------------
// Pass 1: per-row running (max, sum) over this workgroup's key chunk, in the log2 domain.
// row_part[((g*n_chunks + chunk)*M + row)*2 + {0,1}] = (m, z) with  sum_j 2^(c1*l_j) = z * 2^m.
template <int D, int NW>
__global__ void __launch_bounds__(NW * 64)
score_rowstats_kernel(const __bf16* __restrict__ q_obs, const __bf16* __restrict__ k, int64_t ksh,
                      int64_t kst, int Hk, int M, int W, int N, int tiles_per_chunk, int n_chunks,
                      float c1, float* __restrict__ row_part) {
  constexpr int NT = NW * 64;
  constexpr int ROW = D + 8;
  constexpr int KS = D / 16;
  __shared__ __attribute__((aligned(16))) __bf16 lds_k[KT * ROW];

  const int g = blockIdx.x % Hk, chunk = blockIdx.x / Hk;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, half = lane >> 5;
  const int T = N - W;
  const int qrow = wave * 32 + ln;
  const int wi = qrow % W;                      // window row of this lane's query row
  ASL_LOAD_Q_FRAGS();

  const __bf16* kg = k + (int64_t)g * ksh;
  const int n_tiles_total = (N + KT - 1) / KT;
  const int tile0 = chunk * tiles_per_chunk;
  const int tile_end = min(tile0 + tiles_per_chunk, n_tiles_total);

  float m_run = kNegBig, z_run = 0.f;
  ASL_KTILE_DECL(D, NT);
  if (tile0 < tile_end) { ASL_KTILE_LOAD(tile0 * KT); }

  for (int tile = tile0; tile < tile_end; ++tile) {
    __syncthreads();                            // every wave is done reading the previous tile
    ASL_KTILE_STORE();
    __syncthreads();
    if (tile + 1 < tile_end) { ASL_KTILE_LOAD((tile + 1) * KT); }

    const int kbase = tile * KT;
    const bool need_mask = (kbase + KT > T);    // touches the window block or the tail past N
#pragma unroll
    for (int sub = 0; sub < KT / 32; ++sub) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      const __bf16* krow = lds_k + (sub * 32 + ln) * ROW + half * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(krow + ks * 16);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc, 0, 0, 0);   // [key][query row]
      }
      float x[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) x[r] = acc[r];
      if (need_mask) {
        // visible iff key < N and (key < T or key - T <= wi)  <=>  key < min(N, T + wi + 1)
        const int lim = min(N, T + wi + 1) - (kbase + sub * 32 + 4 * half);
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = (8 * (r >> 2) + (r & 3) < lim) ? x[r] : -INFINITY;
      }
      float mx = x[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = max2(mx, x[r]);
      const float m_new = max2(m_run, mx * c1);
      float sum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(x[r], c1, -m_new));
      z_run = z_run * fast_exp2(m_run - m_new) + sum;
      m_run = m_new;
    }
  }
  // the two lane halves hold disjoint keys of the same query row
  const float m_o = __shfl_xor(m_run, 32), z_o = __shfl_xor(z_run, 32);
  const float m = max2(m_run, m_o);
  const float za = z_run * fast_exp2(m_run - m), zb = z_o * fast_exp2(m_o - m);
  const float z = (half == 0) ? (za + zb) : (zb + za);
  if (half == 0 && qrow < M) {
    float* dst = row_part + ((int64_t)(g * n_chunks + chunk) * M + qrow) * 2;
    dst[0] = m;
    dst[1] = z;
  }
}

// Fold the per-chunk partials of every row into one log2-domain offset  m + log2(Z).
// One wavefront per row: lanes stride over the chunks, then a fixed-order butterfly.
__global__ void __launch_bounds__(256)
score_combine_kernel(const float* __restrict__ row_part, int Hk, int M, int n_chunks,
                     float* __restrict__ row_const) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= Hk * M) return;
  const int g = r / M, row = r % M;
  const float2* p = reinterpret_cast<const float2*>(row_part) + (int64_t)g * n_chunks * M + row;
  float m = kNegBig, z = 0.f;
  for (int c = lane; c < n_chunks; c += 64) {
    const float2 v = p[(int64_t)c * M];
    const float mn = fmaxf(m, v.x);
    z = z * exp2f(m - mn) + v.y * exp2f(v.x - mn);
    m = mn;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float mo = __shfl_xor(m, o), zo = __shfl_xor(z, o);
    const float mn = fmaxf(m, mo);
    // add the two partial sums in lane order so both partners compute the same bits
    const float za = z * exp2f(m - mn), zb = zo * exp2f(mo - mn);
    z = (lane & o) ? (zb + za) : (za + zb);
    m = mn;
  }
  if (lane == 0) row_const[r] = m + log2f(z);
}

// ---------------------------------------------------------------------------------------------
// Pass 2: u_group[g][j] = sum over the M rows of 2^(c1*l_rj - rc_r),  j < T,
// rc_r = rc_mul * row_const[g*M + r]  (log2-domain offset that already contains log2 Z_r).
template <int D, int NW>
__global__ void __launch_bounds__(NW * 64)
score_colsum_kernel(const __bf16* __restrict__ q_obs, const __bf16* __restrict__ k, int64_t ksh,
                    int64_t kst, int Hk, int M, int N, int T, int tiles_per_chunk, float c1,
                    const float* __restrict__ row_const, float rc_mul, float* __restrict__ u_group) {
  constexpr int NT = NW * 64;
  constexpr int ROW = D + 8;
  constexpr int KS = D / 16;
  __shared__ __attribute__((aligned(16))) __bf16 lds_k[KT * ROW];
  __shared__ float red[NW][KT];

  const int g = blockIdx.x % Hk, chunk = blockIdx.x / Hk;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, half = lane >> 5;
  const int qrow = wave * 32 + ln;
  ASL_LOAD_Q_FRAGS();

  float rc[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = wave * 32 + acc_row(r, half);
    const float v = row_const[(int64_t)g * M + min(row, M - 1)] * rc_mul;
    rc[r] = (row < M) ? v : INFINITY;                    // padded rows add 2^-inf = 0
  }

  const __bf16* kg = k + (int64_t)g * ksh;
  const int n_tiles_total = (T + KT - 1) / KT;
  const int tile0 = chunk * tiles_per_chunk;
  const int tile_end = min(tile0 + tiles_per_chunk, n_tiles_total);

  ASL_KTILE_DECL(D, NT);
  if (tile0 < tile_end) { ASL_KTILE_LOAD(tile0 * KT); }

  for (int tile = tile0; tile < tile_end; ++tile) {
    __syncthreads();                            // previous tile's LDS reads (keys and red) are done
    ASL_KTILE_STORE();
    __syncthreads();
    if (tile + 1 < tile_end) { ASL_KTILE_LOAD((tile + 1) * KT); }

    const int kbase = tile * KT;
#pragma unroll
    for (int sub = 0; sub < KT / 32; ++sub) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      const __bf16* krow = lds_k + (sub * 32 + ln) * ROW + half * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(krow + ks * 16);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf, acc, 0, 0, 0);   // [query row][key]
      }
      float cs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) cs += fast_exp2(fmaf(acc[r], c1, -rc[r]));
      const float other = __shfl_xor(cs, 32);
      if (half == 0) red[wave][sub * 32 + ln] = cs + other;
    }
    __syncthreads();
    for (int j = tid; j < KT; j += NT) {
      float s = red[0][j];
#pragma unroll
      for (int w = 1; w < NW; ++w) s += red[w][j];
      if (kbase + j < T) u_group[(int64_t)g * T + kbase + j] = s;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Generic path (any d, any M, fp32 or bf16 storage, plain fp32 FMA): small shapes and the on-GPU
// cross-check of the MFMA path.
template <typename TIn> __device__ __forceinline__ float ldf(const TIn* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<__bf16>(const __bf16* p) { return (float)*p; }

// one workgroup per global query row r = h*W + wi: log2-domain offset m + log2 Z (or from lse)
template <typename TIn>
__global__ void __launch_bounds__(256)
score_rowstats_generic(const TIn* __restrict__ q_obs, const TIn* __restrict__ k, int64_t ksh, int64_t kst,
                       int G, int W, int N, int D, float c1, float* __restrict__ row_const) {
  extern __shared__ float sm[];                // D floats of q, then 2*256 for the reduction
  float* qs = sm;
  float* red_m = sm + D;
  float* red_z = red_m + 256;
  const int r = blockIdx.x, h = r / W, wi = r % W, g = h / G;
  const int T = N - W;
  for (int c = threadIdx.x; c < D; c += 256) qs[c] = ldf<TIn>(q_obs + (int64_t)r * D + c);
  __syncthreads();
  const TIn* kg = k + (int64_t)g * ksh;
  const int n_vis = T + wi + 1;                // past keys + window keys 0..wi
  float m = kNegBig, z = 0.f;
  for (int j = threadIdx.x; j < n_vis; j += 256) {
    const TIn* kr = kg + (int64_t)j * kst;
    float dot = 0.f;
    for (int c = 0; c < D; ++c) dot = fmaf(qs[c], ldf<TIn>(kr + c), dot);
    float x = dot * c1;
    float mn = fmaxf(m, x);
    z = z * exp2f(m - mn) + exp2f(x - mn);
    m = mn;
  }
  red_m[threadIdx.x] = m;
  red_z[threadIdx.x] = z;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) {
      float m1 = red_m[threadIdx.x], m2 = red_m[threadIdx.x + s];
      float mn = fmaxf(m1, m2);
      red_z[threadIdx.x] = red_z[threadIdx.x] * exp2f(m1 - mn) + red_z[threadIdx.x + s] * exp2f(m2 - mn);
      red_m[threadIdx.x] = mn;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) row_const[r] = red_m[0] + log2f(red_z[0]);
}

// one thread per (KV head g, past key j): loop over the M rows of the group
template <typename TIn>
__global__ void __launch_bounds__(256)
score_colsum_generic(const TIn* __restrict__ q_obs, const TIn* __restrict__ k, int64_t ksh, int64_t kst,
                     int M, int T, int D, float c1, const float* __restrict__ row_const, float rc_mul,
                     float* __restrict__ u_group) {
  const int g = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= T) return;
  const TIn* kr = k + (int64_t)g * ksh + (int64_t)j * kst;
  const TIn* qg = q_obs + (int64_t)g * M * D;
  float s = 0.f;
  for (int r = 0; r < M; ++r) {
    float dot = 0.f;
    for (int c = 0; c < D; ++c) dot = fmaf(ldf<TIn>(qg + (int64_t)r * D + c), ldf<TIn>(kr + c), dot);
    s += exp2f(fmaf(dot, c1, -row_const[(int64_t)g * M + r] * rc_mul));
  }
  u_group[(int64_t)g * T + j] = s;
}

// ---------------------------------------------------------------------------------------------
bool score_mfma_supported(const asl_params& p) {
  const int M = (p.n_q_heads / p.n_kv_heads) * p.window;
  return p.dtype == ASL_BF16 && (p.head_dim == 64 || p.head_dim == 128) && M <= 256;
}

// Key chunks per KV head: enough workgroups to fill 256 CUs a few times over.
int score_chunks(const asl_params& p) {
  const int n_tiles = (p.seq_len + KT - 1) / KT;
  int want = (1024 + p.n_kv_heads - 1) / p.n_kv_heads;
  if (want > kMaxChunks) want = kMaxChunks;
  if (want > n_tiles) want = n_tiles;
  if (want < 1) want = 1;
  const int tpc = (n_tiles + want - 1) / want;
  return (n_tiles + tpc - 1) / tpc;
}

template <int D, int NW>
static hipError_t launch_score_mfma(const asl_params& p, const Workspace& ws, const __bf16* q,
                                    const __bf16* k, const float* lse, float c1, hipStream_t st) {
  const int Hk = p.n_kv_heads, M = (p.n_q_heads / Hk) * p.window, N = p.seq_len, T = N - p.window;
  const int n_chunks = score_chunks(p);
  const int n_tiles1 = (N + KT - 1) / KT;
  const int tpc1 = (n_tiles1 + n_chunks - 1) / n_chunks;
  if (!lse) {
    ASL_LAUNCH(ws.prof, kKernRowstats, st, (score_rowstats_kernel<D, NW>), dim3(Hk * n_chunks), dim3(NW * 64), 0, st, q, k,
                       p.k_stride_head, p.k_stride_tok, Hk, M, p.window, N, tpc1, n_chunks, c1,
                       ws.row_part);
    const int rows = Hk * M;
    ASL_LAUNCH(ws.prof, kKernCombine, st, score_combine_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, ws.row_part,
                       Hk, M, n_chunks, ws.row_const);
  }
  const int n_tiles2 = (T + KT - 1) / KT;
  const int tpc2 = (n_tiles2 + n_chunks - 1) / n_chunks;
  const int n_chunks2 = (n_tiles2 + tpc2 - 1) / tpc2;
  ASL_LAUNCH(ws.prof, kKernColsum, st, (score_colsum_kernel<D, NW>), dim3(Hk * n_chunks2), dim3(NW * 64), 0, st, q, k,
                     p.k_stride_head, p.k_stride_tok, Hk, M, N, T, tpc2, c1,
                     lse ? lse : ws.row_const, lse ? kLog2e : 1.0f, ws.u_group);
  return hipGetLastError();
}

template <int D>
static hipError_t dispatch_nw(int nw, const asl_params& p, const Workspace& ws, const __bf16* q,
                              const __bf16* k, const float* lse, float c1, hipStream_t st) {
  switch (nw) {
    case 1: return launch_score_mfma<D, 1>(p, ws, q, k, lse, c1, st);
    case 2: return launch_score_mfma<D, 2>(p, ws, q, k, lse, c1, st);
    case 3: return launch_score_mfma<D, 3>(p, ws, q, k, lse, c1, st);
    case 4: return launch_score_mfma<D, 4>(p, ws, q, k, lse, c1, st);
    case 5: return launch_score_mfma<D, 5>(p, ws, q, k, lse, c1, st);
    case 6: return launch_score_mfma<D, 6>(p, ws, q, k, lse, c1, st);
    case 7: return launch_score_mfma<D, 7>(p, ws, q, k, lse, c1, st);
    default: return launch_score_mfma<D, 8>(p, ws, q, k, lse, c1, st);
  }
}

template <typename TIn>
static hipError_t launch_score_generic(const asl_params& p, const Workspace& ws, const TIn* q,
                                       const TIn* k, const float* lse, float c1, hipStream_t st) {
  const int Hk = p.n_kv_heads, G = p.n_q_heads / Hk, W = p.window, M = G * W, N = p.seq_len, T = N - W;
  const int D = p.head_dim;
  if (!lse) {
    size_t sm = (size_t)(D + 512) * sizeof(float);
    ASL_LAUNCH(ws.prof, kKernScoreGeneric, st, (score_rowstats_generic<TIn>), dim3(p.n_q_heads * W), dim3(256), sm, st, q, k,
                       p.k_stride_head, p.k_stride_tok, G, W, N, D, c1, ws.row_const);
  }
  ASL_LAUNCH(ws.prof, kKernScoreGeneric, st, (score_colsum_generic<TIn>), dim3((T + 255) / 256, Hk), dim3(256), 0, st, q, k,
                     p.k_stride_head, p.k_stride_tok, M, T, D, c1, lse ? lse : ws.row_const,
                     lse ? kLog2e : 1.0f, ws.u_group);
  return hipGetLastError();
}

hipError_t launch_score(const asl_params& p, const Workspace& ws, const void* q_obs, const void* k,
                        const float* lse, hipStream_t st) {
  const float scale = p.scale > 0.f ? p.scale : 1.0f / sqrtf((float)p.head_dim);
  const float c1 = scale * kLog2e;
  const int M = (p.n_q_heads / p.n_kv_heads) * p.window;
  if (score_mfma_supported(p) && !(p.flags & ASL_FLAG_GENERIC_SCORE)) {
    const int nw = (M + 31) / 32;
    const __bf16* q = static_cast<const __bf16*>(q_obs);
    const __bf16* kk = static_cast<const __bf16*>(k);
    return p.head_dim == 128 ? dispatch_nw<128>(nw, p, ws, q, kk, lse, c1, st)
                             : dispatch_nw<64>(nw, p, ws, q, kk, lse, c1, st);
  }
  if (p.dtype == ASL_BF16)
    return launch_score_generic<__bf16>(p, ws, static_cast<const __bf16*>(q_obs),
                                        static_cast<const __bf16*>(k), lse, c1, st);
  return launch_score_generic<float>(p, ws, static_cast<const float*>(q_obs),
                                     static_cast<const float*>(k), lse, c1, st);
}

}  // namespace asl
