// asl_score: window-query x all-key softmax scores, column-summed over the window rows and the
// GQA group (Alg. 1 steps 5, 6, 8 of the paper; Sec. 4.1 PA equation before pooling).
//
// For one KV head the G heads x W window rows form M = G*W query rows that all read the same
// keys.  score_j = sum_r exp(l_rj - m_r) / Z_r mixes rows with different normalisers, so the
// final (m_r, Z_r) of every row must be known before rows are added: pass 1 streams K once for
// the row statistics, pass 2 streams K again for the normalised column sums.  When the caller
// hands over the rows' log-sum-exp, pass 1 is skipped.
//
// Work split: a workgroup owns one KV head and a contiguous chunk of keys; wave w owns RB blocks of
// 32 query rows (RB = 1 up to M = 128 rows, 2 above) and keeps their bf16 fragments in registers for
// the whole kernel; K tiles of 64 keys stream global -> LDS directly (ring of 3-4 buffers,
// XOR-swizzled) and every wave reads all of them as the other MFMA operand
// (v_mfma_f32_32x32x16_bf16), each fragment once for all its row blocks.  Pass 1 puts keys on the
// accumulator's register axis (row statistics reduce in-lane), pass 2 puts query rows there
// (column sums reduce in-lane).  All reductions have a fixed order: results are deterministic.
#include "asl_internal.h"

namespace asl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#ifndef ASL_SCORE_KT
#define ASL_SCORE_KT 64
#endif
#ifndef ASL_SCORE_STAGES
#define ASL_SCORE_STAGES 3
#endif
constexpr int KT = ASL_SCORE_KT;              // keys per LDS tile (a multiple of 32)
#ifndef ASL_SCORE_STAGES_RB2
#define ASL_SCORE_STAGES_RB2 4
#endif
// LDS tile buffers of the K ring: STAGES-1 tiles in flight while one is consumed.  RB = 32-row query
// blocks per wavefront: 1 for M <= 128 query rows (three workgroups per compute unit), 2 above
// (two larger workgroups per compute unit, hence a deeper ring each).
template <int RB> constexpr int ring_stages() { return RB > 1 ? ASL_SCORE_STAGES_RB2 : ASL_SCORE_STAGES; }
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;           // finite stand-in for "no maximum yet"

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Row of the 32x32 accumulator held by register r of a lane in half `half` (lanes 32..63 = 1).
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// K tile staging: global memory -> LDS directly (global_load_lds_dwordx4: each lane names its own
// 16-byte global source, the hardware writes lane i's data to  wave base + 16*i  in LDS), a ring of
// LDS buffers, one workgroup barrier per tile.  The tile is stored unpadded; bank conflicts on the
// fragment reads are avoided by an XOR swizzle applied on the global side: LDS slot (row r,
// piece c') holds the row's 16-byte piece  c = c' ^ (r mod CPR).
// Rows past N are clamped to the last key (they are masked or discarded later).
// Per-thread constants of the tile loader: for each of its NLOAD pieces the byte offset of the
// (swizzled) source piece from the tile's first key.
// The first NT threads of the workgroup do the loading, NT = the largest power of two that is at most
// the workgroup size and the number of pieces (see loader_threads): every loading wavefront then
// issues the same number of loads per tile, which the counted waits below rely on; the other
// wavefronts issue none and are held by the workgroup barrier alone.
template <int D, int NT>
struct TilePieces {
  static constexpr int CPR = D / 8;                   // 16-byte pieces per key row
  static constexpr int SLOTS = KT * CPR;
  static_assert(SLOTS % NT == 0, "loader threads must divide the pieces of a tile");
  static constexpr int NLOAD = SLOTS / NT;
  uint32_t src_off[NLOAD];
  // tile row and first element of the (swizzled) source piece of this thread's i-th load
  static __device__ __forceinline__ int row(int i, int tid) { return (i * NT + tid) / CPR; }
  static __device__ __forceinline__ int col8(int i, int tid) {
    const int q = i * NT + tid;
    return ((q % CPR) ^ ((q / CPR) & (CPR - 1))) * 8;
  }
  __device__ __forceinline__ void init(int64_t kst, int tid) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) src_off[i] = (uint32_t)(((int64_t)row(i, tid) * kst + col8(i, tid)) * 2);
  }
};

template <int D, int NT, bool FULL>
__device__ __forceinline__ void issue_tile_loads_impl(const TilePieces<D, NT>& tp,
                                                      const __bf16* __restrict__ kg, int64_t kst, int key0,
                                                      int N, __bf16* __restrict__ lds_buf, int tid) {
  constexpr int NLOAD = TilePieces<D, NT>::NLOAD;
  const int wave_slot0 = __builtin_amdgcn_readfirstlane(tid) & ~63;
  if (wave_slot0 >= NT) return;                         // not a loading wavefront (wave-uniform)
  const char* tile_base = reinterpret_cast<const char*>(kg + (int64_t)key0 * kst);   // uniform
  if (FULL) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const char* src = tile_base + tp.src_off[i];
      __bf16* dst = lds_buf + (int64_t)(i * NT + wave_slot0) * 8;     // wave-uniform base
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
  } else {
    // last, partial tile of a head: rows past N - 1 read key N - 1 instead.  Kept as a loop (it runs
    // once per head and launch; unrolled it would hold NLOAD row addresses in registers all along)
    const int last = N - 1 - key0;                        // last valid row of the tile
#pragma unroll 1
    for (int i = 0; i < NLOAD; ++i) {
      const int r = min(TilePieces<D, NT>::row(i, tid), last);
      const char* src = tile_base + ((int64_t)r * kst + TilePieces<D, NT>::col8(i, tid)) * 2;
      __bf16* dst = lds_buf + (int64_t)(i * NT + wave_slot0) * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
  }
}

// Full tiles take the precomputed offsets; only a tile that reaches past N pays for clamping.
template <int D, int NT>
__device__ __forceinline__ void issue_tile_loads(const TilePieces<D, NT>& tp, const __bf16* __restrict__ kg,
                                                 int64_t kst, int key0, int N, __bf16* __restrict__ lds_buf,
                                                 int tid) {
  if (key0 + KT <= N)
    issue_tile_loads_impl<D, NT, true>(tp, kg, kst, key0, N, lds_buf, tid);
  else
    issue_tile_loads_impl<D, NT, false>(tp, kg, kst, key0, N, lds_buf, tid);
}

// Wait until at most CNT of this wave's vector-memory operations (incl. its LDS-direct loads) are
// still outstanding; they complete in issue order, so everything older than the last CNT is done.
// The same instruction waits for all of the wave's LDS operations (lgkmcnt 0): every use of it is
// followed by the workgroup barrier that hands this wave's LDS writes (pass 2's column partials) to
// other waves, and the wait the compiler derives from the barrier's fence was seen to disappear next
// to this hand-written one (the partials of a tile's last sub-tile were then read before they landed).
template <int CNT>
__device__ __forceinline__ void wait_vmem() {
  static_assert(CNT >= 0 && CNT < 64, "vmcnt is a 6-bit count");
  // vmcnt(CNT): low 4 bits in [3:0], high 2 bits in [15:14]; expcnt [6:4] left at "no wait"; lgkmcnt [11:8] = 0
  __builtin_amdgcn_s_waitcnt(0x0070 | (CNT & 0xF) | ((CNT >> 4) << 14));
}

// Threads of an NW-wavefront workgroup that load the K tiles.
template <int D, int NW>
constexpr int loader_threads() {
  int n = 64;
  while (n * 2 <= NW * 64 && n * 2 <= KT * (D / 8)) n *= 2;
  return n;
}

// Loads each loading wave issues per tile.
template <int D, int NT>
constexpr int tile_loads_per_wave() { return (KT * (D / 8)) / NT; }

// Top-of-iteration wait: the current tile must have landed.  `younger` = tiles issued after it that
// are still in flight (at most STAGES-2).  With a uniform per-wave load count those may stay
// outstanding; otherwise wait for everything.
template <int L, int Y>
__device__ __forceinline__ void wait_younger(int younger) {
  if constexpr (Y == 0) {
    wait_vmem<0>();
  } else {
    if (younger >= Y) wait_vmem<Y * L>();
    else wait_younger<L, Y - 1>(younger);
  }
}
template <int D, int NT, int STAGES>
__device__ __forceinline__ void wait_tile(int younger) {
  constexpr int L = tile_loads_per_wave<D, NT>();
  static_assert(STAGES >= 2, "ring depth");
  if constexpr (L > 0 && L * (STAGES - 2) < 64)
    wait_younger<L, STAGES - 2>(younger);
  else
    wait_vmem<0>();
}

// K fragment of kstep ks for the 32-key sub-tile `sub`: lane (ln, half) holds key ln,
// d = 16*ks + 8*half .. +8  (logical piece 2*ks + half, un-swizzled here).
template <int D>
__device__ __forceinline__ bf16x8 load_k_frag(const __bf16* buf, int sub, int ln, int half, int ks) {
  constexpr int CPR = D / 8;
  const int r = sub * 32 + ln;
  const int cp = (2 * ks + half) ^ (r & (CPR - 1));
  return *reinterpret_cast<const bf16x8*>(buf + (r * CPR + cp) * 8);
}

// QK^T of one 32-key sub-tile against this wave's RB blocks of 32 query rows (d/16 chained MFMAs
// per block; every K fragment is read from LDS once and used for all RB blocks).
// KEYS_ON_REGS: accumulator register axis = keys (pass 1), else = query rows (pass 2).
template <int D, bool KEYS_ON_REGS, int RB>
__device__ __forceinline__ void mma_subtile(const __bf16* __restrict__ buf, int sub, int ln, int half,
                                            const bf16x8 (&qf)[RB][D / 16], f32x16 (&acc)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    const bf16x8 kf = load_k_frag<D>(buf, sub, ln, half, ks);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      acc[rb] = KEYS_ON_REGS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][ks], acc[rb], 0, 0, 0)
                             : __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][ks], kf, acc[rb], 0, 0, 0);
  }
}

// Query fragments of this wave's RB 32-row blocks (block rb = rows row0 + 32*rb ..): lane (ln, half)
// holds row ln of each block, d = 16*ks + 8*half .. +8.
#define ASL_LOAD_Q_FRAGS()                                                                        \
  bf16x8 qf[RB][KS];                                                                              \
  _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                             \
    const int qr_ = row0 + rb * 32 + ln;                                                          \
    const __bf16* qg_ = q_obs + (int64_t)g * M * D + (int64_t)min(qr_, M - 1) * D + half * 8;     \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                           \
      uint4 raw_ = *reinterpret_cast<const uint4*>(qg_ + ks * 16);                                \
      if (qr_ >= M) raw_ = make_uint4(0u, 0u, 0u, 0u);      /* padded rows: zero queries */       \
      qf[rb][ks] = __builtin_bit_cast(bf16x8, raw_);                                              \
    }                                                                                             \
  }


// Share of the key tiles a workgroup takes.  All workgroups of a pass are resident at once (one
// round), block b being the (b / n_cu)-th workgroup placed on its compute unit; on this part the
// first-placed workgroup of a compute unit progresses fastest and the last-placed slowest
// (measured finish times 0.70 : 0.85 : 0.98 of the kernel with three per unit, 0.76 : 0.98 with two).
// With three per unit (M <= 128) the kernels are bound by the unit's share of the HBM stream and
// weighting the shares does not shorten them, so the weights are equal; with two per unit (M > 128)
// the arithmetic is not hidden any more, the second workgroup ends up alone on its unit for the last
// quarter of the kernel, and giving the first one a larger share is worth 4-5 %.  Weights in 1/1024,
// tunable at build time.
#ifndef ASL_SCORE_W3
#define ASL_SCORE_W3 1024, 1024, 1024
#endif
#ifndef ASL_SCORE_W2
#define ASL_SCORE_W2 1250, 798
#endif
struct ChunkRange {
  int tile0, tile_end;
};
__device__ __forceinline__ int pick3(int i, int a, int b, int c) { return i == 0 ? a : (i == 1 ? b : c); }
__device__ __forceinline__ int pick2(int i, int a, int b) { return i == 0 ? a : b; }
// Tiles [tile0, tile_end) of chunk `chunk` (0 .. n_chunks-1) of KV head g; the chunks of a head tile
// [0, n_tiles) exactly, in order.  (Selects instead of indexed tables: no private memory.)
__device__ __forceinline__ ChunkRange chunk_range(int chunk, int g, int Hk, int n_chunks, int n_tiles, int n_cu) {
  const int grid = n_chunks * Hk;
  const int n_slots = (grid + n_cu - 1) / n_cu;
  // cumulative weight of this head's chunks 0 .. c-1: chunk c' is block c'*Hk + g, placed as number
  // (c'*Hk + g) / n_cu on its compute unit
  auto cum = [&](int c) -> int {
    if (n_slots != 2 && n_slots != 3) return 1024 * c;
    // chunks with (c'*Hk + g) < n_cu*(s+1)  <=>  c' < ceil((n_cu*(s+1) - g) / Hk)
    const int u0 = min(max((n_cu - g + Hk - 1) / Hk, 0), c);
    const int u1 = (n_slots == 2) ? c : min(max((2 * n_cu - g + Hk - 1) / Hk, u0), c);
    const int w0 = (n_slots == 3) ? pick3(0, ASL_SCORE_W3) : pick2(0, ASL_SCORE_W2);
    const int w1 = (n_slots == 3) ? pick3(1, ASL_SCORE_W3) : pick2(1, ASL_SCORE_W2);
    const int w2 = pick3(2, ASL_SCORE_W3);
    return w0 * u0 + w1 * (u1 - u0) + w2 * (c - u1);      // < 2^21 for n_chunks <= 256
  };
  // Boundaries in fp32 (a 64-bit integer division would cost microseconds at the start of every
  // workgroup): neighbours evaluate the same expression on the same inputs, so their shared
  // boundary is the same number, and any monotone rounding gives a valid partition.
  const float per_weight = (float)n_tiles / (float)cum(n_chunks);
  ChunkRange r;
  r.tile0 = min((int)((float)cum(chunk) * per_weight), n_tiles);
  r.tile_end = (chunk + 1 == n_chunks) ? n_tiles : min((int)((float)cum(chunk + 1) * per_weight), n_tiles);
  return r;
}

// This file is compiled with NaNs assumed absent, so this is a bare v_max_f32 / v_max3_f32
// (inputs are finite or -inf here).
__device__ __forceinline__ float max2(float a, float b) { return __builtin_fmaxf(a, b); }

// Fold the logits of one 32-key sub-tile (keys on the accumulator's register axis; `key_lo` = key of
// this lane's register 0) into the running (max, sum) of the lane's query row, per row block.
template <int RB>
__device__ __forceinline__ void rowstats_fold(const f32x16 (&acc)[RB], bool need_mask, int key_lo, int N, int T,
                                              const int (&wi)[RB], float c1, float (&m_run)[RB], float (&z_run)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float x[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = acc[rb][r];
    if (need_mask) {
      // visible iff key < N and (key < T or key - T <= wi)  <=>  key < min(N, T + wi + 1)
      const int lim = min(N, T + wi[rb] + 1) - key_lo;
#pragma unroll
      for (int r = 0; r < 16; ++r) x[r] = (8 * (r >> 2) + (r & 3) < lim) ? x[r] : -INFINITY;
    }
    float mx = x[0];
#pragma unroll
    for (int r = 1; r < 16; r += 2) mx = max2(mx, max2(x[r], x[(r + 1) & 15]));
    const float m_new = max2(m_run[rb], mx * c1);
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(x[r], c1, -m_new));
    z_run[rb] = z_run[rb] * fast_exp2(m_run[rb] - m_new) + sum;
    m_run[rb] = m_new;
  }
}

// One tile of pass 1: start the next tile's LDS-direct loads into `nxt`, then fold the tile in
// `cur` into the running (max, sum).  The two LDS buffers are distinct restrict pointers so that
// the compiler knows the fragment reads of `cur` need not wait for the loads into `nxt`.
template <int D, int NT, int RB>
__device__ __forceinline__ void rowstats_tile(const __bf16* __restrict__ cur, __bf16* __restrict__ nxt,
                                              bool prefetch, const TilePieces<D, NT>& tp, const __bf16* __restrict__ kg, int64_t kst,
                                              int prefetch_key0, int tile, int N, int T, const int (&wi)[RB], int tid, int ln,
                                              int half, const bf16x8 (&qf)[RB][D / 16], float c1, float (&m_run)[RB],
                                              float (&z_run)[RB]) {
  if (prefetch) issue_tile_loads<D, NT>(tp, kg, kst, prefetch_key0, N, nxt, tid);
  const int kbase = tile * KT;
  const bool need_mask = (kbase + KT > T);      // touches the window block or the tail past N
  // Software pipeline over the 32-key sub-tiles: the MFMAs of sub-tile s+1 are issued before
  // the softmax arithmetic of sub-tile s, so the matrix pipe and the vector ALU run side by side.
  f32x16 acc[RB];
  mma_subtile<D, true, RB>(cur, 0, ln, half, qf, acc);
#pragma unroll
  for (int sub = 0; sub < KT / 32; ++sub) {
    f32x16 nxt_acc[RB];
    if (sub + 1 < KT / 32) {
      mma_subtile<D, true, RB>(cur, sub + 1, ln, half, qf, nxt_acc);
    } else {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) nxt_acc[rb] = acc[rb];
    }
    rowstats_fold<RB>(acc, need_mask, kbase + sub * 32 + 4 * half, N, T, wi, c1, m_run, z_run);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = nxt_acc[rb];
  }
}

// ---------------------------------------------------------------------------------------------
// Pass 1: per-row running (max, sum) over this workgroup's key chunk, in the log2 domain.
// row_part[((g*n_chunks + chunk)*M + row)*2 + {0,1}] = (m, z) with  sum_j 2^(c1*l_j) = z * 2^m.
template <int D, int NW, int RB>
__global__ void __launch_bounds__(NW * 64)
score_rowstats_kernel(const __bf16* __restrict__ q_obs, const __bf16* __restrict__ k, int64_t ksh,
                      int64_t kst, int Hk, int M, int W, int N, int n_cu, int n_chunks,
                      float c1, float* __restrict__ row_part) {
  constexpr int NT = loader_threads<D, NW>();      // threads that load the K tiles
  constexpr int KS = D / 16;
  constexpr int TILE_ELEMS = KT * D;
  constexpr int STAGES = ring_stages<RB>();
  __shared__ __attribute__((aligned(16))) __bf16 lds_k[STAGES * TILE_ELEMS];

  const int g = blockIdx.x % Hk, chunk = blockIdx.x / Hk;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, half = lane >> 5;
  const int T = N - W;
  const int row0 = wave * 32 * RB;              // first query row of this wave
  int wi[RB];                                   // window row of this lane's query row, per block
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) wi[rb] = (row0 + rb * 32 + ln) % W;
  const __bf16* kg = k + (int64_t)g * ksh;
  const ChunkRange cr = chunk_range(chunk, g, Hk, n_chunks, (N + KT - 1) / KT, n_cu);
  const int tile0 = cr.tile0, tile_end = cr.tile_end;

  ASL_LOAD_Q_FRAGS();
  TilePieces<D, NT> tp;
  tp.init(kst, tid);
  // prologue: STAGES-1 tiles in flight (after the Q loads, so the in-order wait counts line up)
#pragma unroll
  for (int j = 0; j < STAGES - 1; ++j)
    if (tile0 + j < tile_end) issue_tile_loads<D, NT>(tp, kg, kst, (tile0 + j) * KT, N, lds_k + j * TILE_ELEMS, tid);

  float m_run[RB], z_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = kNegBig;
    z_run[rb] = 0.f;
  }
  int stage = 0;                                  // buffer that holds tile `tile`
  for (int tile = tile0; tile < tile_end; ++tile) {
    wait_tile<D, NT, STAGES>(min(STAGES - 2, tile_end - 1 - tile));
    __syncthreads();      // tile `tile` has landed for every wave; the buffer of tile-1 is free again
    const int free_stage = (stage == 0) ? STAGES - 1 : stage - 1;
    rowstats_tile<D, NT, RB>(lds_k + stage * TILE_ELEMS, lds_k + free_stage * TILE_ELEMS,
                             tile + STAGES - 1 < tile_end, tp, kg, kst, (tile + STAGES - 1) * KT, tile, N, T, wi, tid,
                             ln, half, qf, c1, m_run, z_run);
    stage = (stage + 1 == STAGES) ? 0 : stage + 1;
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    // the two lane halves hold disjoint keys of the same query row
    const float m_o = __shfl_xor(m_run[rb], 32), z_o = __shfl_xor(z_run[rb], 32);
    const float m = max2(m_run[rb], m_o);
    const float za = z_run[rb] * fast_exp2(m_run[rb] - m), zb = z_o * fast_exp2(m_o - m);
    const float z = (half == 0) ? (za + zb) : (zb + za);
    const int qrow = row0 + rb * 32 + ln;
    if (half == 0 && qrow < M) {
      float* dst = row_part + ((int64_t)(g * n_chunks + chunk) * M + qrow) * 2;
      dst[0] = m;
      dst[1] = z;
    }
  }
}

// Fold the per-chunk partials (m_c, z_c) of one query row into the row's log2-domain softmax offset
// m + log2(Z).  Two lanes share a row (`half` = 0 or 1, partner = lane ^ 32): each takes every
// second chunk, in chunk order with a running maximum; the two halves are added in a fixed order,
// so every caller gets the same bits for the same partials.
// p points at the row's partial of chunk 0; consecutive chunks are M float2 apart.
// Batches of kB chunks per lane: all loads of a batch are issued before the first is used.
// NR rows at once (pointers p[0..NR-1]): the loads of a batch go out for all of them before the first
// is used, so NR rows cost as many memory round trips as one.
template <int NR, int kB>
__device__ __forceinline__ void combine_rows(const float2* const (&p)[NR], int M, int n_chunks, int half,
                                             float (&out)[NR]) {
  float m[NR], z[NR];
#pragma unroll
  for (int q = 0; q < NR; ++q) {
    m[q] = kNegBig;
    z[q] = 0.f;
  }
  for (int c0 = half; c0 < n_chunks; c0 += 2 * kB) {
    float2 v[NR][kB];
#pragma unroll
    for (int q = 0; q < NR; ++q)
#pragma unroll
      for (int j = 0; j < kB; ++j) {
        const int c = c0 + 2 * j;
        v[q][j] = p[q][(int64_t)min(c, n_chunks - 1) * M];
        if (c >= n_chunks) v[q][j] = make_float2(kNegBig, 0.f);
      }
#pragma unroll
    for (int q = 0; q < NR; ++q) {
      float mb = m[q];
#pragma unroll
      for (int j = 0; j < kB; ++j) mb = fmaxf(mb, v[q][j].x);
      float zb = 0.f;
#pragma unroll
      for (int j = 0; j < kB; ++j) zb += v[q][j].y * fast_exp2(v[q][j].x - mb);
      z[q] = z[q] * fast_exp2(m[q] - mb) + zb;
      m[q] = mb;
    }
  }
#pragma unroll
  for (int q = 0; q < NR; ++q) {
    const float mo = __shfl_xor(m[q], 32), zo = __shfl_xor(z[q], 32);
    const float mm = fmaxf(m[q], mo);
    const float za = z[q] * fast_exp2(m[q] - mm), zb2 = zo * fast_exp2(mo - mm);
    const float zs = (half == 0) ? (za + zb2) : (zb2 + za);
    out[q] = mm + log2f(zs);
  }
}
__device__ __forceinline__ float combine_row(const float2* __restrict__ p, int M, int n_chunks, int half) {
  const float2* const ps[1] = {p};
  float out[1];
  combine_rows<1, 48>(ps, M, n_chunks, half, out);
  return out[0];
}

// The offsets of all Hk*M rows (one wavefront per 32 rows), for callers that want the rows'
// log-sum-exp: row_const[r] = m + log2(Z) and, as a natural logarithm, lse_out[r].
__global__ void __launch_bounds__(256)
score_combine_kernel(const float* __restrict__ row_part, int Hk, int M, int n_chunks,
                     float* __restrict__ row_const, float* __restrict__ lse_out) {
  const int lane = threadIdx.x & 63, ln = lane & 31, half = lane >> 5;
  const int r = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32 + ln;
  const int rr = min(r, Hk * M - 1);
  const int g = rr / M, row = rr % M;
  const float2* p = reinterpret_cast<const float2*>(row_part) + (int64_t)g * n_chunks * M + row;
  const float c = combine_row(p, M, n_chunks, half);
  if (half == 0 && r < Hk * M) {
    row_const[r] = c;
    if (lse_out != nullptr) lse_out[r] = c * kLn2;
  }
}

// This lane's share of the column sums of one 32-key sub-tile (query rows on the accumulator's
// register axis): the normalised probabilities of its 16 rows per block, added in a fixed order.
template <int RB>
__device__ __forceinline__ float colsum_fold(const f32x16 (&acc)[RB], const float (&rc)[RB][16], float c1) {
  float cs = 0.f;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) cs += fast_exp2(fmaf(acc[rb][r], c1, -rc[rb][r]));
  return cs;
}

// One tile of pass 2: start the next tile's loads into `nxt`, then the column partial sums of
// this wave's 32*RB rows for the KT keys in `cur` (written to red_w[0..KT-1]).
template <int D, int NT, int RB>
__device__ __forceinline__ void colsum_tile(const __bf16* __restrict__ cur, __bf16* __restrict__ nxt,
                                            bool prefetch, const TilePieces<D, NT>& tp, const __bf16* __restrict__ kg, int64_t kst,
                                            int prefetch_key0, int N, int tid, int ln, int half,
                                            const bf16x8 (&qf)[RB][D / 16], const float (&rc)[RB][16], float c1,
                                            float* __restrict__ red_w) {
  if (prefetch) issue_tile_loads<D, NT>(tp, kg, kst, prefetch_key0, N, nxt, tid);
  f32x16 acc[RB];
  mma_subtile<D, false, RB>(cur, 0, ln, half, qf, acc);
#pragma unroll
  for (int sub = 0; sub < KT / 32; ++sub) {
    f32x16 nxt_acc[RB];
    if (sub + 1 < KT / 32) {
      mma_subtile<D, false, RB>(cur, sub + 1, ln, half, qf, nxt_acc);   // overlaps the exps below
    } else {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) nxt_acc[rb] = acc[rb];
    }
    const float cs = colsum_fold<RB>(acc, rc, c1);
    const float other = __shfl_xor(cs, 32);
    if (half == 0) red_w[sub * 32 + ln] = cs + other;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = nxt_acc[rb];
  }
}

// ---------------------------------------------------------------------------------------------
// Pass 2: u_group[g][j] = sum over the M rows of 2^(c1*l_rj - rc_r),  j < T,
// rc_r = rc_mul * row_const[g*M + r]  (log2-domain offset that already contains log2 Z_r).
template <int D, int NW, int RB>
__global__ void __launch_bounds__(NW * 64)
score_colsum_kernel(const __bf16* __restrict__ q_obs, const __bf16* __restrict__ k, int64_t ksh,
                    int64_t kst, int Hk, int M, int N, int T, int n_cu, float c1,
                    const float* __restrict__ row_const, float rc_mul, const float* __restrict__ row_part,
                    int n_parts, float* __restrict__ u_group) {
  constexpr int NT = loader_threads<D, NW>();      // threads that load the K tiles
  constexpr int NTHREADS = NW * 64;
  constexpr int KS = D / 16;
  constexpr int TILE_ELEMS = KT * D;
  constexpr int STAGES = ring_stages<RB>();
  __shared__ __attribute__((aligned(16))) __bf16 lds_k[STAGES * TILE_ELEMS];
  __shared__ float red[2][NW][KT];              // per-wave column partials, double-buffered

  const int g = blockIdx.x % Hk, chunk = blockIdx.x / Hk;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, ln = lane & 31, half = lane >> 5;
  const int row0 = wave * 32 * RB;              // first query row of this wave
  const __bf16* kg = k + (int64_t)g * ksh;
  const ChunkRange cr = chunk_range(chunk, g, Hk, (int)(gridDim.x / Hk), (T + KT - 1) / KT, n_cu);
  const int tile0 = cr.tile0, tile_end = cr.tile_end;

  ASL_LOAD_Q_FRAGS();
  TilePieces<D, NT> tp;
  tp.init(kst, tid);
  // The chunk is walked from its last tile to its first: pass 1 walked it first to last, so the
  // tiles read most recently (still in the last-level cache) are the ones this pass reads first.
  const int n_my = max(tile_end - tile0, 0);
  // prologue: STAGES-1 tiles in flight before the row offsets are worked out, so that their latency
  // hides behind the first tiles' (later loads complete later: the counted waits below stay valid)
#pragma unroll
  for (int j = 0; j < STAGES - 1; ++j)
    if (j < n_my) issue_tile_loads<D, NT>(tp, kg, kst, (tile_end - 1 - j) * KT, N, lds_k + j * TILE_ELEMS, tid);

  // Log2-domain softmax offsets of this lane's accumulator rows: from the caller's log-sum-exp
  // (row_const, scaled by rc_mul), or folded here from pass 1's per-chunk partials (row_part).
  float rc[RB][16];
  float mine[RB];                                       // offsets of rows  row0 + 32*rb + ln
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) mine[rb] = 0.f;
  if (row_part != nullptr) {
    const float2* ps[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      ps[rb] = reinterpret_cast<const float2*>(row_part) + (int64_t)g * n_parts * M + min(row0 + rb * 32 + ln, M - 1);
    combine_rows<RB, (RB == 1 ? 48 : 32)>(reinterpret_cast<const float2* const (&)[RB]>(ps), M, n_parts, half, mine);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = row0 + rb * 32 + acc_row(r, half);
      float v;
      if (row_part != nullptr)
        v = __shfl(mine[rb], acc_row(r, half));         // lanes 0..31 hold rows 0..31 of the block
      else
        v = row_const[(int64_t)g * M + min(row, M - 1)] * rc_mul;
      rc[rb][r] = (row < M) ? v : INFINITY;              // padded rows add 2^-inf = 0
    }
  }
  // sum the waves' partials of one finished tile in a fixed order and store the past columns
  auto reduce_store = [&](int buf_idx, int kbase) {
    for (int j = tid; j < KT; j += NTHREADS) {
      float s = red[buf_idx][0][j];
#pragma unroll
      for (int w = 1; w < NW; ++w) s += red[buf_idx][w][j];
      if (kbase + j < T) u_group[(int64_t)g * T + kbase + j] = s;
    }
  };

  int stage = 0;                                  // buffer that holds the current tile
  for (int it = 0; it < n_my; ++it) {
    const int tile = tile_end - 1 - it;
    wait_tile<D, NT, STAGES>(min(STAGES - 2, n_my - 1 - it));
    __syncthreads();      // the tile has landed; previous tile's fragment reads and partials are done
    if (it > 0) reduce_store((it - 1) & 1, (tile + 1) * KT);
    const int free_stage = (stage == 0) ? STAGES - 1 : stage - 1;
    colsum_tile<D, NT, RB>(lds_k + stage * TILE_ELEMS, lds_k + free_stage * TILE_ELEMS, it + STAGES - 1 < n_my,
                           tp, kg, kst, (tile - (STAGES - 1)) * KT, N, tid, ln, half, qf, rc, c1,
                           &red[it & 1][wave][0]);
    stage = (stage + 1 == STAGES) ? 0 : stage + 1;
  }
  if (n_my > 0) {
    __syncthreads();
    reduce_store((n_my - 1) & 1, tile0 * KT);
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
                       int G, int W, int N, int D, float c1, float* __restrict__ row_const,
                       float* __restrict__ lse_out) {
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
  if (threadIdx.x == 0) {
    const float c = red_m[0] + log2f(red_z[0]);
    row_const[r] = c;
    if (lse_out != nullptr) lse_out[r] = c * kLn2;
  }
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
// Largest number of query rows per KV head (G*W) the MFMA kernels take: eight wavefronts of two
// 32-row blocks.
constexpr int kMaxMfmaRows = 512;

bool score_mfma_supported(const asl_params& p) {
  const int M = (p.n_q_heads / p.n_kv_heads) * p.window;
  return p.dtype == ASL_BF16 && (p.head_dim == 64 || p.head_dim == 128) && M <= kMaxMfmaRows;
}

// Compute units of the current device (256 on MI355X).
static int device_cu_count() {
  static const int n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
      v = 256;
    return v;
  }();
  return n;
}

// Key chunks per KV head for a pass whose kernel fits `resident` workgroups per compute unit: one
// resident round of workgroups, so that no second, partly filled round trails behind.
static int score_chunks(const asl_params& p, int resident) {
  const int target = device_cu_count() * resident;
  const int n_tiles = (p.seq_len + KT - 1) / KT;
  int want = target / p.n_kv_heads;
  if (want > kMaxChunks) want = kMaxChunks;
  if (want > n_tiles) want = n_tiles;
  if (want < 1) want = 1;
  const int tpc = (n_tiles + want - 1) / want;
  return (n_tiles + tpc - 1) / tpc;
}

// Workgroups of `kernel` that fit on one compute unit at once (registers, LDS, wave slots).
template <typename K>
static int resident_per_cu(K kernel, int threads, size_t dynamic_lds = 0) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, dynamic_lds) != hipSuccess || n < 1) {
    (void)hipGetLastError();
    n = 1;
  }
  return n;
}

template <int D, int NW, int RB>
static hipError_t launch_score_mfma(const asl_params& p, const Workspace& ws, const __bf16* q,
                                    const __bf16* k, const float* lse, float* lse_out, float c1,
                                    hipStream_t st) {
  const int Hk = p.n_kv_heads, M = (p.n_q_heads / Hk) * p.window, N = p.seq_len, T = N - p.window;
  // both passes use the same LDS ring and nearly the same registers; take the smaller residency
  static const int resident = [] {
    const int a = resident_per_cu(score_rowstats_kernel<D, NW, RB>, NW * 64);
    const int b = resident_per_cu(score_colsum_kernel<D, NW, RB>, NW * 64);
    return a < b ? a : b;
  }();
  const int n_chunks = score_chunks(p, resident);
  const int n_cu = device_cu_count();
  if (!lse) {
    ASL_LAUNCH(ws.prof, kKernRowstats, st, (score_rowstats_kernel<D, NW, RB>), dim3(Hk * n_chunks), dim3(NW * 64), 0, st, q, k,
                       p.k_stride_head, p.k_stride_tok, Hk, M, p.window, N, n_cu, n_chunks, c1,
                       ws.row_part);
    if (lse_out) {                                 // only the row normalisers were asked for
      const int rows = Hk * M;
      ASL_LAUNCH(ws.prof, kKernCombine, st, score_combine_kernel, dim3((rows + 127) / 128), dim3(256), 0, st, ws.row_part,
                         Hk, M, n_chunks, ws.row_const, lse_out);
      return hipGetLastError();
    }
  }
  const int n_tiles2 = (T + KT - 1) / KT;
  const int n_chunks2 = n_chunks < n_tiles2 ? n_chunks : n_tiles2;
  // without the caller's log-sum-exp every pass-2 workgroup folds pass 1's partials of its own rows
  ASL_LAUNCH(ws.prof, kKernColsum, st, (score_colsum_kernel<D, NW, RB>), dim3(Hk * n_chunks2), dim3(NW * 64), 0, st, q, k,
                     p.k_stride_head, p.k_stride_tok, Hk, M, N, T, n_cu, c1,
                     lse, kLog2e, lse ? nullptr : ws.row_part, n_chunks, ws.u_group);
  return hipGetLastError();
}

// Wavefronts and 32-row blocks per wavefront for M query rows per KV head: one block per wavefront
// up to 128 rows; two above, with ceil(M / 64) wavefronts (up to eight, M <= 512).
template <int D>
static hipError_t dispatch_nw(int M, const asl_params& p, const Workspace& ws, const __bf16* q,
                              const __bf16* k, const float* lse, float* lse_out, float c1, hipStream_t st) {
  if (M <= 128) {
    switch ((M + 31) / 32) {
      case 1: return launch_score_mfma<D, 1, 1>(p, ws, q, k, lse, lse_out, c1, st);
      case 2: return launch_score_mfma<D, 2, 1>(p, ws, q, k, lse, lse_out, c1, st);
      case 3: return launch_score_mfma<D, 3, 1>(p, ws, q, k, lse, lse_out, c1, st);
      default: return launch_score_mfma<D, 4, 1>(p, ws, q, k, lse, lse_out, c1, st);
    }
  }
  switch ((M + 63) / 64) {
    case 3: return launch_score_mfma<D, 3, 2>(p, ws, q, k, lse, lse_out, c1, st);
    case 4: return launch_score_mfma<D, 4, 2>(p, ws, q, k, lse, lse_out, c1, st);
    case 5: return launch_score_mfma<D, 5, 2>(p, ws, q, k, lse, lse_out, c1, st);
    case 6: return launch_score_mfma<D, 6, 2>(p, ws, q, k, lse, lse_out, c1, st);
    case 7: return launch_score_mfma<D, 7, 2>(p, ws, q, k, lse, lse_out, c1, st);
    default: return launch_score_mfma<D, 8, 2>(p, ws, q, k, lse, lse_out, c1, st);
  }
}

template <typename TIn>
static hipError_t launch_score_generic(const asl_params& p, const Workspace& ws, const TIn* q,
                                       const TIn* k, const float* lse, float* lse_out, float c1,
                                       hipStream_t st) {
  const int Hk = p.n_kv_heads, G = p.n_q_heads / Hk, W = p.window, M = G * W, N = p.seq_len, T = N - W;
  const int D = p.head_dim;
  if (!lse) {
    size_t sm = (size_t)(D + 512) * sizeof(float);
    ASL_LAUNCH(ws.prof, kKernScoreGeneric, st, (score_rowstats_generic<TIn>), dim3(p.n_q_heads * W), dim3(256), sm, st, q, k,
                       p.k_stride_head, p.k_stride_tok, G, W, N, D, c1, ws.row_const, lse_out);
  }
  if (lse_out) return hipGetLastError();
  ASL_LAUNCH(ws.prof, kKernScoreGeneric, st, (score_colsum_generic<TIn>), dim3((T + 255) / 256, Hk), dim3(256), 0, st, q, k,
                     p.k_stride_head, p.k_stride_tok, M, T, D, c1, lse ? lse : ws.row_const,
                     lse ? kLog2e : 1.0f, ws.u_group);
  return hipGetLastError();
}

// lse != null: the rows' log-sum-exp is given, only the column-sum pass runs.  lse_out != null (and
// lse == null): only the row-statistics pass runs and the rows' log-sum-exp is written there.
hipError_t launch_score(const asl_params& p, const Workspace& ws, const void* q_obs, const void* k,
                        const float* lse, float* lse_out, hipStream_t st) {
  const float scale = p.scale > 0.f ? p.scale : 1.0f / sqrtf((float)p.head_dim);
  const float c1 = scale * kLog2e;
  const int M = (p.n_q_heads / p.n_kv_heads) * p.window;
  if (score_mfma_supported(p) && !(p.flags & ASL_FLAG_GENERIC_SCORE)) {
    const __bf16* q = static_cast<const __bf16*>(q_obs);
    const __bf16* kk = static_cast<const __bf16*>(k);
    return p.head_dim == 128 ? dispatch_nw<128>(M, p, ws, q, kk, lse, lse_out, c1, st)
                             : dispatch_nw<64>(M, p, ws, q, kk, lse, lse_out, c1, st);
  }
  if (p.dtype == ASL_BF16)
    return launch_score_generic<__bf16>(p, ws, static_cast<const __bf16*>(q_obs),
                                        static_cast<const __bf16*>(k), lse, lse_out, c1, st);
  return launch_score_generic<float>(p, ws, static_cast<const float*>(q_obs),
                                     static_cast<const float*>(k), lse, lse_out, c1, st);
}

}  // namespace asl
