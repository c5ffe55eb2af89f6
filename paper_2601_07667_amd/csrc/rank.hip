// asl_rank: RankDesc of the all-head score vector (Alg. 1 step 11 of the paper):
// rank[t] = position of t in the order (score descending, token index ascending).
//
// A stable least-significant-digit radix sort of (key, index) pairs on an order-preserving
// 32-bit transform of the fp32 score, 8 bits per pass; the last pass scatters positions to
// rank[index] instead of writing the sorted pairs.  Per pass: a per-tile histogram kernel, then a
// scatter kernel that derives its offsets from those histograms and ranks equal digits inside a
// tile with wavefront ballots (stable by construction).
#include <cstdio>
#include <mutex>

#include "asl_internal.h"

namespace asl {

constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortRounds = kSortTile / kSortThreads;        // elements per thread
constexpr int kSortPerWave = kSortTile / kSortWaves;

// Ascending unsigned order of the result == descending float order; -0 is treated as +0.
__device__ __forceinline__ uint32_t desc_key(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;
}

// Per-tile digit histogram, written as one contiguous row tile_hist[tile][0..255].
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads)
sort_hist_kernel(const float* __restrict__ s, const uint32_t* __restrict__ keys_in, int T, int shift,
                 uint32_t* __restrict__ tile_hist) {
  __shared__ uint32_t h[kHistWords];
  const int tid = threadIdx.x;
  hist_clear(h, tid, kSortThreads);
  __syncthreads();
  const int base = blockIdx.x * kSortTile;
  uint32_t key[kSortRounds];
#pragma unroll
  for (int i = 0; i < kSortRounds; ++i) {              // all loads in flight before the first use
    const int e = base + i * kSortThreads + tid;
    key[i] = 0;
    if (e < T) key[i] = FIRST ? desc_key(s[e]) : keys_in[e];
  }
#pragma unroll
  for (int i = 0; i < kSortRounds; ++i) {
    const int e = base + i * kSortThreads + tid;
    if (e < T) hist_add(h, tid, (key[i] >> shift) & 255u);
  }
  __syncthreads();
  tile_hist[(int64_t)blockIdx.x * 256 + tid] = hist_total(h, tid);
}

// Stable scatter of one tile.  Every workgroup derives its own exclusive offsets from the
// per-tile histograms (all tiles' counts of smaller digits + earlier tiles' counts of the same
// digit): redundant across workgroups but a few tens of KB of L2 reads, with no atomics, fences
// or serial tail.
template <bool FIRST, bool LAST>
__global__ void __launch_bounds__(kSortThreads)
sort_scatter_kernel(const float* __restrict__ s, const uint32_t* __restrict__ keys_in,
                    const uint32_t* __restrict__ idx_in, int T, int shift, int n_tiles,
                    const uint32_t* __restrict__ tile_hist, uint32_t* __restrict__ keys_out,
                    uint32_t* __restrict__ idx_out, int32_t* __restrict__ rank_out) {
  __shared__ uint32_t cnt[kSortWaves][256];
  __shared__ uint32_t start[kSortWaves][256];
  __shared__ uint32_t wave_sum[kSortWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w) cnt[w][tid] = 0;

  // this wave's elements: issue every load before anything waits on one
  constexpr int R = kSortPerWave / 64;
  uint32_t key[R], idx[R], off[R];
  const int base = blockIdx.x * kSortTile + wave * kSortPerWave;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    key[r] = 0;
    idx[r] = 0;
    if (e < T) {
      key[r] = FIRST ? desc_key(s[e]) : keys_in[e];
      idx[r] = FIRST ? (uint32_t)e : idx_in[e];
    }
  }

  // digit `tid`: total over all tiles and over the tiles before this one
  uint32_t tot = 0, prev = 0;
  {
    const int me = blockIdx.x;
    int t = 0;
    for (; t + 16 <= n_tiles; t += 16) {
      uint32_t v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = tile_hist[(int64_t)(t + u) * 256 + tid];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        tot += v[u];
        prev += (t + u < me) ? v[u] : 0u;
      }
    }
    for (; t < n_tiles; ++t) {
      uint32_t v = tile_hist[(int64_t)t * 256 + tid];
      tot += v;
      prev += (t < me ? v : 0u);
    }
  }
  // exclusive scan of tot over the 256 digits (wave scan + wave totals)
  uint32_t incl = tot;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_sum[wave] = incl;
  __syncthreads();                                   // also orders the zeroing of cnt
  uint32_t digit_base = incl - tot;
  for (int w = 0; w < wave; ++w) digit_base += wave_sum[w];
  const uint32_t my_off = digit_base + prev;         // first destination of digit `tid` in this tile

  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    const bool valid = e < T;
    const uint32_t d = (key[r] >> shift) & 255u;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const uint32_t before = __popcll(peers & lt_mask);
    uint32_t old = 0;
    if (valid) old = cnt[wave][d];
    if (valid && before == 0) cnt[wave][d] = old + (uint32_t)__popcll(peers);
    off[r] = old + before;
  }
  __syncthreads();
  {
    uint32_t run = my_off;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      start[w][tid] = run;
      run += cnt[w][tid];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = base + r * 64 + lane;
    if (e < T) {
      const uint32_t d = (key[r] >> shift) & 255u;
      const uint32_t dest = start[wave][d] + off[r];
      if (LAST) {
        rank_out[idx[r]] = (int32_t)dest;
      } else {
        keys_out[dest] = key[r];
        idx_out[dest] = idx[r];
      }
    }
  }
}

hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st) {
  const int n_tiles = (T + kSortTile - 1) / kSortTile;
  const dim3 grid(n_tiles), block(kSortThreads);
  // pass 0: scores -> buffer 0
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<true>), grid, block, 0, st, s, nullptr, T, 0, ws.tile_hist);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<true, false>), grid, block, 0, st, s, nullptr, nullptr, T, 0,
                     n_tiles, ws.tile_hist, ws.sort_key[0], ws.sort_idx[0], nullptr);
  // pass 1: 0 -> 1
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[0], T, 8, ws.tile_hist);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, false>), grid, block, 0, st, nullptr, ws.sort_key[0],
                     ws.sort_idx[0], T, 8, n_tiles, ws.tile_hist, ws.sort_key[1], ws.sort_idx[1], nullptr);
  // pass 2: 1 -> 0
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[1], T, 16, ws.tile_hist);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, false>), grid, block, 0, st, nullptr, ws.sort_key[1],
                     ws.sort_idx[1], T, 16, n_tiles, ws.tile_hist, ws.sort_key[0], ws.sort_idx[0], nullptr);
  // pass 3: 0 -> rank
  ASL_LAUNCH(ws.prof, kKernSortHist, st, (sort_hist_kernel<false>), grid, block, 0, st, nullptr, ws.sort_key[0], T, 24, ws.tile_hist);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_scatter_kernel<false, true>), grid, block, 0, st, nullptr, ws.sort_key[0],
                     ws.sort_idx[0], T, 24, n_tiles, ws.tile_hist, nullptr, nullptr, rank_out);
  return hipGetLastError();
}

}  // namespace asl

// ---------------------------------------------------------------------------------------------
// asl_rank_static: asl_rank for callers that cannot allocate.  The sort's scratch (ping-pong
// key/index buffers and the per-tile histograms) lives in a file-scope device array instead of a
// context's workspace.  In host code the array's name is only a handle: its device address is
// looked up once per device and that pointer is what the kernels get.
namespace {

constexpr int kStaticMaxT = ASL_RANK_STATIC_MAX_T;
constexpr size_t kStaticTiles = (kStaticMaxT + asl::kSortTile - 1) / asl::kSortTile;
constexpr size_t kStaticWords = 4 * (size_t)kStaticMaxT + 256 * kStaticTiles;
static_assert(kStaticMaxT % 64 == 0, "keeps the four buffers 256-byte aligned");

static __device__ __align__(256) uint32_t scratch[kStaticWords];

constexpr int kMaxDevices = 64;
uint32_t* g_scratch_ptr[kMaxDevices];            // device address of `scratch` on each device
std::mutex g_scratch_mutex;
thread_local char g_static_err[192] = "";

// Device address of this device's copy of `scratch` (the current device must be `device`).
hipError_t static_scratch(int device, uint32_t** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = static_cast<uint32_t*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

asl_status static_fail(asl_status st, const char* msg, const char* detail = "") {
  snprintf(g_static_err, sizeof(g_static_err), "%s%s", msg, detail);
  return st;
}

}  // namespace

namespace asl {
hipError_t rank_static_prepare(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  uint32_t* p = nullptr;
  return static_scratch(device, &p);
}
}  // namespace asl

extern "C" {
#pragma GCC visibility push(default)

asl_status asl_rank_static(const float* s, int32_t T, int32_t* rank_out, void* stream) {
  if (!s || !rank_out) return static_fail(ASL_EINVAL, "asl_rank_static: null tensor pointer");
  if (T < 1) return static_fail(ASL_EINVAL, "asl_rank_static: need T >= 1");
  if (T > kStaticMaxT) {
    char detail[64];
    snprintf(detail, sizeof(detail), " (T=%d, limit %d)", T, kStaticMaxT);
    return static_fail(ASL_ENOMEM, "asl_rank_static: T exceeds ASL_RANK_STATIC_MAX_T", detail);
  }
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return static_fail(ASL_EHIP, "hipGetDevice: ", hipGetErrorString(e));
  if (device < 0 || device >= kMaxDevices) return static_fail(ASL_EUNSUPPORTED, "asl_rank_static: device index too large");
  uint32_t* base = nullptr;
  e = static_scratch(device, &base);
  if (e != hipSuccess) return static_fail(ASL_EHIP, "hipGetSymbolAddress(scratch): ", hipGetErrorString(e));
  asl::Workspace ws = {};
  ws.sort_key[0] = base;
  ws.sort_idx[0] = base + (size_t)kStaticMaxT;
  ws.sort_key[1] = base + 2 * (size_t)kStaticMaxT;
  ws.sort_idx[1] = base + 3 * (size_t)kStaticMaxT;
  ws.tile_hist = base + 4 * (size_t)kStaticMaxT;
  ws.prof = nullptr;
  e = asl::launch_rank(ws, s, T, rank_out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return static_fail(ASL_EHIP, "rank launch: ", hipGetErrorString(e));
  return ASL_OK;
}

const char* asl_static_last_error(void) { return g_static_err; }

#pragma GCC visibility pop
}  // extern "C"
