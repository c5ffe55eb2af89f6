// Internal declarations shared by the libasl translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include "asl.h"

namespace asl {

// Kernel ids for the optional per-kernel event profiling (asl_profile_enable / asl_profile_collect).
enum KernelId {
  kKernRowstats = 0, kKernCombine, kKernColsum, kKernPool, kKernSortHist, kKernSortScatter,
  kKernRankvarFinal, kKernRankvar, kKernSelHist, kKernSelWrite, kKernGather,
  kKernScoreGeneric, kKernTail, kKernCount
};

// Event pairs recorded around tagged launches; owned by the ctx, created by asl_profile_enable.
struct Prof {
  uint32_t mask = 0;
  int cap = 0, n = 0;
  hipEvent_t* start = nullptr;
  hipEvent_t* stop = nullptr;
  int* id = nullptr;
};

// Record slot for one launch of kernel `kid`, or -1 when that kernel is not being timed.
inline int prof_slot(Prof* p, int kid) {
  if (p && ((p->mask >> kid) & 1u) && p->n < p->cap) {
    p->id[p->n] = kid;
    return p->n++;
  }
  return -1;
}

// Launch; a timed launch hands its event pair to the runtime, which stamps them with the kernel's own
// start and end on the device (events recorded before and after the launch would also measure the
// dispatch gap in front of the kernel, 3-5 us).
#define ASL_LAUNCH(prof, kid, st, kernel, grid, block, lds, stream, ...)                                      \
  do {                                                                                                        \
    asl::Prof* prof_ = (prof);                                                                                \
    const int slot_ = asl::prof_slot(prof_, (kid));                                                           \
    if (slot_ >= 0)                                                                                           \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, prof_->start[slot_], prof_->stop[slot_], 0,     \
                            __VA_ARGS__);                                                                     \
    else                                                                                                      \
      hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                                      \
  } while (0)

// Workspace carve-up (device memory owned by the ctx).
struct Workspace {
  // scoring
  float* row_part;      // [Hk][n_chunks][M][2]  pass-1 partial (max, sum) per row and key chunk
  float* row_const;     // [Hq*W]                log2-domain softmax offsets  m + log2(Z)
  float* u_group;       // [Hk][T]               group-summed past-only column sums (pre-pool)
  // radix sort (rank)
  uint32_t* sort_key[2];   // [T] ping-pong
  uint32_t* sort_idx[2];   // [T]
  unsigned long long* sort_table;   // [n_tiles][128] tagged per-tile digit counts of the current pass
  unsigned long long* sort_epoch;   // [1] tag of the last sort launch
  // select
  uint32_t* sel_sample;    // [sel_rows][kSelMaxSample] sampled keys of freshly pooled score rows
  uint32_t* sel_bound;     // [sel_rows] key bound guessed from the row's sample
  uint32_t* sel_thr;       // [sel_rows][2] threshold key and kept ties of each row
  uint32_t* sel_cand_key;  // [sel_rows][n_tiles][kSelSegment] keys that passed the bound, in token order
  uint32_t* sel_cand_idx;  // same shape: their token indices
  uint32_t* sel_seg_count; // [sel_rows][n_tiles] entries used in each segment
  int sel_rows;            // rows the candidate buffers hold at once
  // rank variance
  unsigned long long* var_table;    // [kVarMaxBlocks][2] tagged per-workgroup partial sums
  unsigned long long* var_epoch;    // [1]
  uint32_t* fault;         // [1] raised by a workgroup whose bounded wait for its peers ran out
  Prof* prof;              // null unless profiling is enabled
};

#ifndef ASL_SORT_TILE
#define ASL_SORT_TILE 2048
#endif
#ifndef ASL_SEL_TILE
#define ASL_SEL_TILE 4096
#endif
#ifndef ASL_SORT_THREADS
#define ASL_SORT_THREADS 1024
#endif
constexpr int kSortTile = ASL_SORT_TILE;   // elements per radix-sort workgroup tile (a multiple of 256)
constexpr int kSelTile = ASL_SEL_TILE;     // elements per select workgroup tile (a multiple of 256)
constexpr int kMaxChunks = 256;        // key chunks per KV head in scoring pass 1
constexpr int kVarMaxBlocks = 256;     // workgroups of the rank-variance kernel
constexpr int kSortMaxTiles = 512;     // workgroups of one sort launch (they wait for each other)
constexpr int kSelSegment = kSelTile / 2;   // candidate slots per select tile
constexpr int kSelCandCap = 16384;     // candidates of one row the finishing workgroup holds in LDS
constexpr int kSelMaxRowTiles = 1024;  // tiles per row the candidate path handles
constexpr int kSelMaxRowsAtOnce = 256; // rows per round of select launches (bounds the candidate buffers)

// ---- the strided sample the top-k takes its bound from -------------------------------------------
// n_s = sel_sample_size(T) keys of a row at positions j * sel_sample_stride(T), j < n_s.
constexpr int kSelMaxSample = 8192;    // sampled keys per row
__host__ __device__ inline int sel_sample_size(int T) {
  int n = T / 32;
  n = n < 1024 ? 1024 : n;
  n = n > kSelMaxSample ? kSelMaxSample : n;
  return n < T ? n : T;
}
__host__ __device__ inline int sel_sample_stride(int T) { return T / sel_sample_size(T); }   // >= 1 for T >= 1

// ---- counts handed between workgroups of one launch -------------------------------------------
// A 64-bit word = (tag << 28) | (count1 << 14) | count0, written and read whole with relaxed
// device-scope atomic accesses.  The tag names the launch, so a reader can tell a fresh word from
// whatever the table held before; nothing else has to be ordered or cleared.
constexpr int kFlagCountBits = 14;
constexpr int kFlagTagShift = 2 * kFlagCountBits;
constexpr unsigned long long kFlagTagMask = (1ull << (64 - kFlagTagShift)) - 1ull;
constexpr int kFlagBatch = 16;             // words a thread polls at once
constexpr int kFlagSpinLimit = 1 << 17;    // polls before a waiter gives up (each takes ~1 us or more)


// 256-bin digit histogram of a workgroup in LDS, kept in 8 copies (lane % 8 picks the copy, rows
// padded to 257 words so that equal digits in different copies fall into different banks): when
// most keys share a digit - the exponent byte of similar scores, or all-equal scores - a single
// copy would serialise every lane of a wavefront on one address.
constexpr int kHistCopies = 8;
constexpr int kHistStride = 257;
constexpr int kHistWords = kHistCopies * kHistStride;

#ifdef __HIPCC__
// Order-preserving 32-bit key of a score: ascending unsigned order of the keys == descending float
// order of the scores; -0 is treated as +0.
__device__ __forceinline__ uint32_t order_key(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;
}

// Inclusive prefix sum over the 64 lanes of a wavefront (all of them active), by data-parallel
// moves inside the vector ALU: within each row of 16 lanes by shifts of 1, 2, 4 and 8 lanes (a lane
// without a source adds 0), then the last lane of rows 0 and 2 to rows 1 and 3, then lane 31 to rows
// 2 and 3.  (A shuffle-based scan goes through the LDS crossbar six times, ~100 cycles each.)
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
  return x;
}

// Minimum / maximum over the 64 lanes of a wavefront (all active), the same way; every lane gets the
// result.  Lanes without a source take the operation's identity.
__device__ __forceinline__ uint32_t wave_min(uint32_t x) {
#define ASL_DPP_MIN_(ctrl, rows) x = min(x, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)x, ctrl, rows, 0xf, false))
  ASL_DPP_MIN_(0x111, 0xf);
  ASL_DPP_MIN_(0x112, 0xf);
  ASL_DPP_MIN_(0x114, 0xf);
  ASL_DPP_MIN_(0x118, 0xf);
  ASL_DPP_MIN_(0x142, 0xa);
  ASL_DPP_MIN_(0x143, 0xc);
#undef ASL_DPP_MIN_
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint32_t wave_max(uint32_t x) {
#define ASL_DPP_MAX_(ctrl, rows) x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ctrl, rows, 0xf, false))
  ASL_DPP_MAX_(0x111, 0xf);
  ASL_DPP_MAX_(0x112, 0xf);
  ASL_DPP_MAX_(0x114, 0xf);
  ASL_DPP_MAX_(0x118, 0xf);
  ASL_DPP_MAX_(0x142, 0xa);
  ASL_DPP_MAX_(0x143, 0xc);
#undef ASL_DPP_MAX_
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
// Sum of a 32-bit / a 64-bit value over the 64 lanes (all active); every lane gets the result.  The
// 64-bit sum goes through three 22-bit limbs, whose 64-lane sums fit 32 bits.
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_prefix_sum(x), 63);
}
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long x) {
  const uint32_t m22 = (1u << 22) - 1u;
  const unsigned long long l0 = wave_sum((uint32_t)x & m22), l1 = wave_sum((uint32_t)(x >> 22) & m22),
                           l2 = wave_sum((uint32_t)(x >> 44));       // x < 2^64: the top limb has 20 bits
  return l0 + (l1 << 22) + (l2 << 44);
}

__device__ __forceinline__ void hist_clear(uint32_t* h, int tid, int n_threads) {
  for (int i = tid; i < kHistWords; i += n_threads) h[i] = 0;
}
__device__ __forceinline__ void hist_add(uint32_t* h, int tid, uint32_t digit) {
  atomicAdd(&h[(tid & (kHistCopies - 1)) * kHistStride + digit], 1u);
}
__device__ __forceinline__ uint32_t hist_total(const uint32_t* h, int digit) {
  uint32_t t = 0;
#pragma unroll
  for (int c = 0; c < kHistCopies; ++c) t += h[c * kHistStride + digit];
  return t;
}

__device__ __forceinline__ void flag_publish(unsigned long long* p, unsigned long long tag, uint32_t c0,
                                             uint32_t c1) {
  const unsigned long long v = ((tag & kFlagTagMask) << kFlagTagShift) |
                               ((unsigned long long)c1 << kFlagCountBits) | (unsigned long long)c0;
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t flag_count0(unsigned long long v) {
  return (uint32_t)v & ((1u << kFlagCountBits) - 1u);
}
__device__ __forceinline__ uint32_t flag_count1(unsigned long long v) {
  return (uint32_t)(v >> kFlagCountBits) & ((1u << kFlagCountBits) - 1u);
}
// Reads the words  col[(t0 + u * STEP) * stride]  for u < kFlagBatch (those with t < n) until every
// one carries `tag`.  Returns false if that has not happened after kFlagSpinLimit polls.
template <int STEP>
__device__ __forceinline__ bool flag_poll_batch(const unsigned long long* col, int stride, int t0, int n,
                                                unsigned long long tag, unsigned long long (&v)[kFlagBatch]) {
  const unsigned long long want = tag & kFlagTagMask;
  for (int spins = 0;; ++spins) {
    bool ok = true;
#pragma unroll
    for (int u = 0; u < kFlagBatch; ++u) {
      const int t = t0 + u * STEP;
      v[u] = (t < n) ? __hip_atomic_load(col + (int64_t)t * stride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                     : (want << kFlagTagShift);
    }
#pragma unroll
    for (int u = 0; u < kFlagBatch; ++u) ok = ok && ((v[u] >> kFlagTagShift) == want);
    if (ok) return true;
    if (spins >= kFlagSpinLimit) return false;
    __builtin_amdgcn_s_sleep(1);
  }
}
#endif

// Workgroups of `kernel` that can wait for each other inside one launch: half of what the device
// holds at once (other kernels may be running beside it), never more than `cap`.
template <typename K>
static inline int coresident_limit(K kernel, int threads, int cap = 1024, size_t dynamic_lds = 0) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dynamic_lds) != hipSuccess) {
    (void)hipGetLastError();
    return 1;
  }
  const long n = (long)cus * per_cu / 2;
  return (int)(n < 1 ? 1 : (n > cap ? cap : n));
}

hipError_t launch_score(const asl_params& p, const Workspace& ws, const void* q_obs, const void* k,
                        const float* lse, float* lse_out, hipStream_t st);
// sample (optional): [rows + 1][kSelMaxSample], receives the top-k's strided sample of the pooled
// rows and, as the last row, of their sum.
hipError_t launch_pool(Prof* prof, const float* u, int rows, int T, int S, float* p_out, float* s_out,
                       uint32_t* sample, hipStream_t st);
hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st);
int rank_max_tiles();      // tiles (workgroups) one sort launch may have on this device
int64_t rank_max_tokens(); // largest T one ranking call takes on this device
// push != 0: first account for this layer's freshly written ring row in the state (a layer index
// that does not follow state->last_layer restarts the ring)
hipError_t launch_rankvar(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx,
                          int k, double tau, int push, asl_state* state, asl_stat* out, hipStream_t st);
hipError_t launch_stat_skip(Prof* prof, asl_stat* out, asl_state* state, int layer_idx, int l_obs,
                            int push, hipStream_t st);
hipError_t launch_select(const Workspace& ws, const float* scores, int rows, int T, int k, int W,
                         int32_t* idx_out, hipStream_t st);
// Arguments of the row-gather kernel.  Either k/v/k_out/v_out name one layer's tensors, or the
// *_ptrs members name device arrays with one pointer per layer (then k..v_out are unused).
struct GatherArgs {
  const char* k;
  const char* v;                 // null when n_tensors == 1
  char* k_out;
  char* v_out;
  const void* const* k_ptrs;     // device arrays [n_layers], or null
  const void* const* v_ptrs;
  void* const* k_out_ptrs;
  void* const* v_out_ptrs;
  const int32_t* idx;            // [n_layers][idx_rows][n_idx]
  int64_t ksh, kst, vsh, vst;    // head / token strides in bytes
  int idx_rows;                  // 1 (shared by the heads) or Hk
  int n_idx;
  int cpr;                       // 16-byte pieces per row
  int cpr_shift;                 // log2(cpr) when cpr is a power of two (set by launch_gather)
  int n_tensors;                 // 1 (K only) or 2 (K and V)
};
hipError_t launch_gather(Prof* prof, const GatherArgs& args, int Hk, int n_layers, hipStream_t st);
bool gather_prepare(GatherArgs& a);   // sets cpr_shift; returns whether cpr is a power of two
// Ranking sort of the last of `rows` score rows + top-k of all rows + optional statistic and KV
// compaction in five launches on one stream (tail.hip); *taken = false when the sizes do not fit and nothing was launched.
struct RankvarArgs;
hipError_t launch_tail(const Workspace& ws, const float* scores, int rows, int T, int k, int W, int32_t* rank_row,
                       int32_t* idx_out, const GatherArgs* gather, int Hk, bool have_sample, const RankvarArgs* stat,
                       hipStream_t st, bool* taken);
// Whether launch_tail would take these sizes (so that the pooling kernel can prepare the sample).
bool tail_takes(const Workspace& ws, int rows, int T);

bool score_mfma_supported(const asl_params& p);
// Looks up the device address of asl_rank_static's scratch array on `device` (which must be current).
hipError_t rank_static_prepare(int device);

}  // namespace asl
