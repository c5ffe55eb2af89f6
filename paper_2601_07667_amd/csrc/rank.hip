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

#include "rank_body.h"

namespace asl {

template <int R, bool FIRST, bool LAST>
__global__ void __launch_bounds__(kSortThreads) sort_pass_kernel(SortArgs a) {
  __shared__ SortShared sh;
  sort_pass_body<R, FIRST, LAST>(sh, a, (int)blockIdx.x);
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

// Arguments of pass `pass` (0..3) of a sort of T scores into rank_out.
SortArgs sort_pass_args(const Workspace& ws, const float* s, int T, int n_tiles, int32_t* rank_out, int pass) {
  // pass 0: scores -> buffer 0;  pass 1: 0 -> 1;  pass 2: 1 -> 0;  pass 3: 0 -> rank
  SortArgs a = {};
  const int in = (pass == 2) ? 1 : 0, out = (pass == 1) ? 1 : 0;
  a.s = (pass == 0) ? s : nullptr;
  a.keys_in = (pass == 0) ? nullptr : ws.sort_key[in];
  a.idx_in = (pass == 0) ? nullptr : ws.sort_idx[in];
  a.T = T;
  a.shift = 8 * pass;
  a.n_tiles = n_tiles;
  a.table = ws.sort_table;
  a.epoch = ws.sort_epoch;
  a.fault = ws.fault;
  a.keys_out = (pass == 3) ? nullptr : ws.sort_key[out];
  a.idx_out = (pass == 3) ? nullptr : ws.sort_idx[out];
  a.rank_out = (pass == 3) ? rank_out : nullptr;
  return a;
}

// Tiles of a sort of T scores and whether they are the big ones; n_tiles = 0 if T is too large.
SortPlan sort_plan(int T, int limit) {
  SortPlan p;
  p.big = false;
  p.n_tiles = (T + kSortTile - 1) / kSortTile;
  if (p.n_tiles <= limit) return p;
  const int big = kSortThreads * kSortRoundsBig;
  p.big = true;
  p.n_tiles = (T + big - 1) / big;
  if (p.n_tiles > limit) p.n_tiles = 0;
  return p;
}

template <int R>
static hipError_t launch_rank_r(const Workspace& ws, const float* s, int T, int n_tiles, int32_t* rank_out,
                                hipStream_t st) {
  const dim3 grid(n_tiles), block(kSortThreads);
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, true, false>), grid, block, 0, st,
             sort_pass_args(ws, s, T, n_tiles, rank_out, 0));
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, false>), grid, block, 0, st,
             sort_pass_args(ws, s, T, n_tiles, rank_out, 1));
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, false>), grid, block, 0, st,
             sort_pass_args(ws, s, T, n_tiles, rank_out, 2));
  ASL_LAUNCH(ws.prof, kKernSortScatter, st, (sort_pass_kernel<R, false, true>), grid, block, 0, st,
             sort_pass_args(ws, s, T, n_tiles, rank_out, 3));
  return hipGetLastError();
}

hipError_t launch_rank(const Workspace& ws, const float* s, int T, int32_t* rank_out, hipStream_t st) {
  const SortPlan plan = sort_plan(T, rank_max_tiles());
  if (plan.n_tiles == 0) return hipErrorInvalidConfiguration;
  return plan.big ? launch_rank_r<kSortRoundsBig>(ws, s, T, plan.n_tiles, rank_out, st)
                  : launch_rank_r<kSortRounds>(ws, s, T, plan.n_tiles, rank_out, st);
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
