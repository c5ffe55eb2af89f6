// asl_rank: RankDesc of the all-head score vector (Alg. 1 step 11 of the paper):
// rank[t] = position of t in the order (score descending, token index ascending).
//
// A stable least-significant-digit radix sort of (key, index) pairs on an order-preserving
// 32-bit transform of the fp32 score, 8 bits per pass, ONE kernel per pass; the last pass scatters
// positions to rank[index] instead of writing the sorted pairs.
//
// In a pass every workgroup owns one tile of consecutive elements.  It counts its tile's digits in
// LDS, publishes the 256 counts, reads every tile's counts (total per digit and the part that
// belongs to earlier tiles), and then ranks its elements inside the tile with wavefront ballots
// (stable by construction) and scatters them.  The counts travel between workgroups of the SAME
// launch through self-validating words: each 64-bit word carries two counts and the tag of this
// launch (a counter kept in device memory, bumped once per launch by tile 0 after it has seen every
// tile's counts, i.e. after every workgroup has read the old value), written and read with relaxed
// device-scope atomic accesses.  A word is usable as soon as its tag matches, so no fences, no
// read-modify-write atomics and no zeroing are needed, and stale contents of the table are harmless.
// The workgroups of a launch wait for each other, so the launch must fit on the device at once
// (checked by the host); waits are bounded: a workgroup that gives up raises the fault word and
// skips its scatter, every wave still exits.
#include <cstdio>
#include <mutex>

#include "asl_internal.h"

namespace asl {

constexpr int kSortThreads = ASL_SORT_THREADS;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortGroups = kSortThreads / 128;              // thread groups that share the polling
// Elements per thread: kSortRounds normally (tiles of kSortTile elements); kSortRoundsBig for inputs
// whose kSortTile-element tiles would be more workgroups than one launch may have.
constexpr int kSortRounds = kSortTile / kSortThreads;
constexpr int kSortRoundsBig = 4 * kSortRounds;
static_assert(kSortTile % kSortThreads == 0 && kSortThreads % 128 == 0 && kSortThreads >= 256, "sort geometry");
static_assert(kSortThreads * kSortRoundsBig < (1 << kFlagCountBits), "a tile's digit count must fit the packed field");

// Ascending unsigned order of the result == descending float order; -0 is treated as +0.
__device__ __forceinline__ uint32_t desc_key(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;
}

template <int R, bool FIRST, bool LAST>
__global__ void __launch_bounds__(kSortThreads)
sort_pass_kernel(const float* __restrict__ s, const uint32_t* __restrict__ keys_in,
                 const uint32_t* __restrict__ idx_in, int T, int shift, int n_tiles,
                 unsigned long long* __restrict__ table, unsigned long long* __restrict__ epoch,
                 uint32_t* __restrict__ fault, uint32_t* __restrict__ keys_out,
                 uint32_t* __restrict__ idx_out, int32_t* __restrict__ rank_out) {
  __shared__ uint32_t h[kHistWords];
  __shared__ uint32_t cnt[kSortWaves][256];
  __shared__ uint32_t start[kSortWaves][256];
  __shared__ uint32_t part_tot[kSortGroups][256];
  __shared__ uint32_t part_prev[kSortGroups][256];
  __shared__ uint32_t digit_off[256];
  __shared__ uint32_t wave_sum[4];
  __shared__ int gave_up;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, me = blockIdx.x;
  const unsigned long long tag = *epoch + 1ull;

  // this wave's elements: issue every load before anything waits on one
  constexpr int kTile = kSortThreads * R, kPerWave = 64 * R;
  uint32_t key[R], idx[R], off[R];
  const int base = me * kTile + wave * kPerWave;
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
  hist_clear(h, tid, kSortThreads);
  if (tid == 0) gave_up = 0;
#pragma unroll
  for (int w = 0; w < kSortWaves; ++w)
    if (tid < 256) cnt[w][tid] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r)
    if (base + r * 64 + lane < T) hist_add(h, tid, (key[r] >> shift) & 255u);
  __syncthreads();
  // publish this tile's counts, two digits per word
  if (tid < 128)
    flag_publish(&table[(int64_t)me * 128 + tid], tag, hist_total(h, 2 * tid), hist_total(h, 2 * tid + 1));

  // every tile's counts of digits 2w, 2w+1 (w = tid % 128); the thread groups share the tiles
  {
    const int w = tid & 127, grp = tid >> 7;
    uint32_t tot0 = 0, tot1 = 0, prev0 = 0, prev1 = 0;
    bool failed = false;
    for (int t0 = grp; t0 < n_tiles; t0 += kSortGroups * kFlagBatch) {
      unsigned long long v[kFlagBatch];
      failed |= !flag_poll_batch<kSortGroups>(table + w, 128, t0, n_tiles, tag, v);
#pragma unroll
      for (int u = 0; u < kFlagBatch; ++u) {
        const int t = t0 + u * kSortGroups;
        if (t < n_tiles) {
          const uint32_t c0 = flag_count0(v[u]), c1 = flag_count1(v[u]);
          tot0 += c0;
          tot1 += c1;
          prev0 += (t < me) ? c0 : 0u;
          prev1 += (t < me) ? c1 : 0u;
        }
      }
    }
    part_tot[grp][2 * w] = tot0;
    part_tot[grp][2 * w + 1] = tot1;
    part_prev[grp][2 * w] = prev0;
    part_prev[grp][2 * w + 1] = prev1;
    if (failed) {
      gave_up = 1;
      *fault = 1u;
    }
  }
  __syncthreads();
  if (gave_up) return;                               // uniform: nothing is scattered by this workgroup
  if (me == 0 && tid == 0) *epoch = tag;             // every workgroup has read the old value by now

  // digit `tid` (first 256 threads): total over all tiles, exclusive scan over the digits
  if (tid < 256) {
    uint32_t tot = 0, prev = 0;
#pragma unroll
    for (int g = 0; g < kSortGroups; ++g) {
      tot += part_tot[g][tid];
      prev += part_prev[g][tid];
    }
    uint32_t incl = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      uint32_t up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    part_tot[0][tid] = incl - tot;                   // exclusive within the wave (own group row is consumed)
    part_prev[0][tid] = prev;
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t digit_base = part_tot[0][tid];
    for (int w = 0; w < wave; ++w) digit_base += wave_sum[w];
    digit_off[tid] = digit_base + part_prev[0][tid];   // first destination of digit `tid` in this tile
  }

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
  if (tid < 256) {
    uint32_t run = digit_off[tid];
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

int rank_max_tiles() {
  static const int n = [] {
    int m = kSortMaxTiles;
    const int c[] = {coresident_limit(sort_pass_kernel<kSortRounds, true, false>, kSortThreads),
                     coresident_limit(sort_pass_kernel<kSortRounds, false, true>, kSortThreads),
                     coresident_limit(sort_pass_kernel<kSortRoundsBig, true, false>, kSortThreads),
                     coresident_limit(sort_pass_kernel<kSortRoundsBig, false, true>, kSortThreads)};
    for (int v : c) m = v < m ? v : m;
    return m;
  }();
  return n;
}

// Largest T one ranking call takes on this device.
int64_t rank_max_tokens() { return (int64_t)rank_max_tiles() * kSortThreads * kSortRoundsBig; }

template <int R>
static hipError_t launch_rank_r(const Workspace& ws, const float* s, int T, int n_tiles, int32_t* rank_out,
                                hipStream_t st) {
  const dim3 grid(n_tiles), block(kSortThreads);
  // pass 0: scores -> buffer 0;  pass 1: 0 -> 1;  pass 2: 1 -> 0;  pass 3: 0 -> rank
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, true, false>), grid, block, 0, st, s, nullptr, nullptr, T, 0,
             n_tiles, ws.sort_table, ws.sort_epoch, ws.fault, ws.sort_key[0], ws.sort_idx[0], nullptr);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, false>), grid, block, 0, st, nullptr, ws.sort_key[0],
             ws.sort_idx[0], T, 8, n_tiles, ws.sort_table, ws.sort_epoch, ws.fault, ws.sort_key[1], ws.sort_idx[1], nullptr);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, false>), grid, block, 0, st, nullptr, ws.sort_key[1],
             ws.sort_idx[1], T, 16, n_tiles, ws.sort_table, ws.sort_epoch, ws.fault, ws.sort_key[0], ws.sort_idx[0], nullptr);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, true>), grid, block, 0, st, nullptr, ws.sort_key[0],
             ws.sort_idx[0], T, 24, n_tiles, ws.sort_table, ws.sort_epoch, ws.fault, nullptr, nullptr, rank_out);
  return hipGetLastError();
}

hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st) {
  const int limit = rank_max_tiles();
  const int n_small = (T + kSortTile - 1) / kSortTile;
  if (n_small <= limit) return launch_rank_r<kSortRounds>(ws, s, T, n_small, rank_out, st);
  const int big = kSortThreads * kSortRoundsBig;
  const int n_big = (T + big - 1) / big;
  if (n_big > limit) return hipErrorInvalidConfiguration;
  return launch_rank_r<kSortRoundsBig>(ws, s, T, n_big, rank_out, st);
}

}  // namespace asl

// ---------------------------------------------------------------------------------------------
// asl_rank_static: asl_rank for callers that cannot allocate.  The sort's scratch (ping-pong
// key/index buffers, the table of tagged per-tile digit counts, the launch counter and the fault
// word) lives in a file-scope device array instead of a context's workspace.  The array starts
// zeroed (as every device global does) and nothing in it ever needs clearing again: the launch
// counter only grows, and stale table contents carry older tags.  In host code the array's name is only a handle: its device address is
// looked up once per device and that pointer is what the kernels get.
namespace {

constexpr int kStaticMaxT = ASL_RANK_STATIC_MAX_T;
constexpr size_t kStaticTiles = (kStaticMaxT + asl::kSortTile - 1) / asl::kSortTile;
constexpr size_t kStaticTableWords = 2 * 128 * kStaticTiles;      // 64-bit entries, in 32-bit words
constexpr size_t kStaticWords = 4 * (size_t)kStaticMaxT + kStaticTableWords + 2 /* counter */ + 2 /* fault, pad */;
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
  uint32_t* tail = base + 4 * (size_t)kStaticMaxT;                 // 8-byte aligned: kStaticMaxT is even
  ws.sort_table = reinterpret_cast<unsigned long long*>(tail);
  ws.sort_epoch = reinterpret_cast<unsigned long long*>(tail + kStaticTableWords);
  ws.fault = tail + kStaticTableWords + 2;
  ws.prof = nullptr;
  if (T > asl::rank_max_tokens())
    return static_fail(ASL_EUNSUPPORTED, "asl_rank_static: T is more than one ranking launch can hold on this device");
  e = asl::launch_rank(ws, s, T, rank_out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return static_fail(ASL_EHIP, "rank launch: ", hipGetErrorString(e));
  return ASL_OK;
}

const char* asl_static_last_error(void) { return g_static_err; }

#pragma GCC visibility pop
}  // extern "C"
