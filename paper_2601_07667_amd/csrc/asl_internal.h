// Internal declarations shared by the libasl translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "asl.h"

namespace asl {

// Workspace carve-up (device memory owned by the ctx).
struct Workspace {
  // scoring
  float* row_part;      // [Hk][n_chunks][M][2]  pass-1 partial (max, sum) per row and key chunk
  float* row_const;     // [Hq*W]                log2-domain softmax offsets  m + log2(Z)
  float* u_group;       // [Hk][T]               group-summed past-only column sums (pre-pool)
  // radix sort (rank)
  uint32_t* sort_key[2];   // [T] ping-pong
  uint32_t* sort_idx[2];   // [T]
  uint32_t* tile_hist;     // [256][n_tiles] digit-major
  uint32_t* counters;      // small block of zero-initialised tickets / accumulators
  // select
  uint32_t* sel_hist;      // [rows][256]
  uint32_t* sel_state;     // [rows][4]  {prefix, k_remaining, unused, unused}
  uint32_t* sel_tile_cnt;  // [rows][n_tiles][2]
};

constexpr int kSortTile = 2048;        // elements per radix-sort workgroup tile
constexpr int kSelTile = 4096;         // elements per select workgroup tile
constexpr int kMaxChunks = 256;        // key chunks per KV head in scoring pass 1
constexpr int kCounterWords = 64;

// counters layout (uint32 words)
constexpr int kCntSortTicket = 0;
constexpr int kCntVarTicket = 1;
constexpr int kCntVarCount = 2;        // union size accumulator
constexpr int kCntVarNumLo = 4;        // 64-bit numerator accumulator (8-byte aligned: words 4,5)
constexpr int kCntSelTicket = 8;       // [max rows] tickets start here (up to 48 rows)

hipError_t launch_score(const asl_params& p, const Workspace& ws, const void* q_obs, const void* k,
                        const float* lse, hipStream_t st);
hipError_t launch_pool(const float* u, int rows, int T, int S, float* p_out, float* s_out,
                       hipStream_t st);
hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st);
hipError_t launch_ring_push(asl_state* state, int layer_idx, int l_obs, hipStream_t st);
hipError_t launch_rankvar(const Workspace& ws, const int32_t* ring, int l_obs, int T, int layer_idx,
                          int k, double tau, asl_state* state, asl_stat* out, hipStream_t st);
hipError_t launch_stat_skip(asl_stat* out, hipStream_t st);
hipError_t launch_select(const Workspace& ws, const float* scores, int rows, int T, int k, int W,
                         int32_t* idx_out, hipStream_t st);
hipError_t launch_gather(const void* k, const void* v, const int32_t* idx, int idx_rows, int n_idx,
                         int Hk, int row_bytes, int64_t k_stride_head_b, int64_t k_stride_tok_b,
                         int64_t v_stride_head_b, int64_t v_stride_tok_b, void* k_out, void* v_out,
                         hipStream_t st);

bool score_mfma_supported(const asl_params& p);
int score_chunks(const asl_params& p);

}  // namespace asl
