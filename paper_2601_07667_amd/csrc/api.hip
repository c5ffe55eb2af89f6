// The C ABI of libasl: context/workspace management, host-side argument validation, and the
// launch sequences behind each entry point declared in include/asl.h.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "rankvar_body.h"

struct asl_ctx {
  int device;
  int32_t max_seq_len, max_kv_heads, max_q_rows;
  void* base;
  size_t bytes;
  asl::Workspace ws;
  asl::Prof prof;
  hipStream_t side;          // second stream of asl_layer_step's fork/join (default priority)
  hipEvent_t ev_fork, ev_join;
  bool side_pending;         // a deferred asl_layer_step left work on `side` that nobody has waited for yet
  char err[256];
};

namespace {

constexpr int kMaxSelectRows = 1024;   // rows per call (KV heads, or layers x KV heads when batched)
constexpr int kMaxPoolKernel = 129;

size_t align_up(size_t x) { return (x + 255) & ~size_t(255); }

// Lay the workspace out from `base` (may be null to only measure).  Returns total bytes.
size_t carve(char* base, int32_t max_seq_len, int32_t max_kv_heads, int32_t max_q_rows,
             asl::Workspace* ws) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> void* {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  };
  const size_t N = (size_t)max_seq_len;
  const size_t rows = (size_t)(max_kv_heads > 1 ? max_kv_heads : 1);
  const size_t sort_tiles = (N + asl::kSortTile - 1) / asl::kSortTile;
  asl::Workspace w;
  w.row_part = (float*)take((size_t)asl::kMaxChunks * max_q_rows * 2 * sizeof(float));
  w.row_const = (float*)take((size_t)max_q_rows * sizeof(float));
  w.u_group = (float*)take(rows * N * sizeof(float));
  for (int i = 0; i < 2; ++i) {
    w.sort_key[i] = (uint32_t*)take(N * sizeof(uint32_t));
    w.sort_idx[i] = (uint32_t*)take(N * sizeof(uint32_t));
  }
  w.sort_table = (unsigned long long*)take(128 * sort_tiles * sizeof(unsigned long long));
  w.sort_epoch = (unsigned long long*)take(sizeof(unsigned long long));
  const size_t sel_tiles = (N + asl::kSelTile - 1) / asl::kSelTile;
  w.sel_rows = (int)(rows < (size_t)asl::kSelMaxRowsAtOnce ? rows : (size_t)asl::kSelMaxRowsAtOnce);
  w.sel_sample = (uint32_t*)take((size_t)w.sel_rows * asl::kSelMaxSample * sizeof(uint32_t));
  w.sel_bound = (uint32_t*)take((size_t)w.sel_rows * sizeof(uint32_t));
  w.sel_thr = (uint32_t*)take((size_t)w.sel_rows * 2 * sizeof(uint32_t));
  w.sel_cand_key = (uint32_t*)take((size_t)w.sel_rows * sel_tiles * asl::kSelSegment * sizeof(uint32_t));
  w.sel_cand_idx = (uint32_t*)take((size_t)w.sel_rows * sel_tiles * asl::kSelSegment * sizeof(uint32_t));
  w.sel_seg_count = (uint32_t*)take((size_t)w.sel_rows * sel_tiles * sizeof(uint32_t));
  w.var_table = (unsigned long long*)take((size_t)asl::kVarMaxBlocks * 4 * sizeof(unsigned long long));
  w.var_epoch = (unsigned long long*)take(sizeof(unsigned long long));
  w.fault = (uint32_t*)take(sizeof(uint32_t));
  if (ws) *ws = w;
  return off;
}

asl_status fail(asl_ctx* ctx, asl_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

asl_status hip_fail(asl_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, ASL_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Makes ctx->device current for the duration of a call and restores the caller's device.
struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t err = hipSuccess;
  explicit DeviceGuard(int dev) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != dev) {
      err = hipSetDevice(dev);
      switched = (err == hipSuccess);
    }
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

int elem_bytes(int dtype) { return dtype == ASL_BF16 ? 2 : 4; }

// Shape checks shared by the entry points that take asl_params.
asl_status check_params(asl_ctx* ctx, const asl_params* p) {
  if (!ctx) return ASL_EINVAL;
  if (!p) return fail(ctx, ASL_EINVAL, "params is null");
  if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_q_heads % p->n_kv_heads != 0)
    return fail(ctx, ASL_EINVAL, "need Hq >= 1, Hk >= 1, Hq %% Hk == 0 (Hq=%d Hk=%d)", p->n_q_heads,
                p->n_kv_heads);
  if (p->head_dim < 1) return fail(ctx, ASL_EINVAL, "head_dim must be >= 1");
  if (p->window < 1 || p->seq_len <= p->window)
    return fail(ctx, ASL_EINVAL, "need 1 <= W < N (W=%d N=%d)", p->window, p->seq_len);
  if (p->pool_kernel < 1 || p->pool_kernel % 2 == 0)
    return fail(ctx, ASL_EINVAL, "pool kernel S must be odd and >= 1 (S=%d)", p->pool_kernel);
  if (p->budget <= p->window)
    return fail(ctx, ASL_EINVAL, "budget must exceed the window (budget=%d W=%d)", p->budget, p->window);
  if (p->dtype != ASL_BF16 && p->dtype != ASL_F32)
    return fail(ctx, ASL_EUNSUPPORTED, "dtype %d not supported", p->dtype);
  if (p->flags & ~(ASL_FLAG_GENERIC_SCORE | ASL_FLAG_DEFER_JOIN))
    return fail(ctx, ASL_EINVAL, "unknown bits in flags (0x%x)", (unsigned)p->flags);
  if (p->pool_kernel > kMaxPoolKernel)
    return fail(ctx, ASL_EUNSUPPORTED, "pool kernel S > %d not supported", kMaxPoolKernel);
  if (p->seq_len > ctx->max_seq_len || p->n_kv_heads > ctx->max_kv_heads ||
      (int64_t)p->n_q_heads * p->window > ctx->max_q_rows)
    return fail(ctx, ASL_ENOMEM, "problem (N=%d Hk=%d Hq*W=%lld) exceeds the context limits (%d, %d, %d)",
                p->seq_len, p->n_kv_heads, (long long)p->n_q_heads * p->window, ctx->max_seq_len,
                ctx->max_kv_heads, ctx->max_q_rows);
  return ASL_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

size_t asl_workspace_bytes(int32_t max_seq_len, int32_t max_kv_heads, int32_t max_q_rows) {
  if (max_seq_len < 2 || max_kv_heads < 1 || max_q_rows < 1) return 0;
  return carve(nullptr, max_seq_len, max_kv_heads, max_q_rows, nullptr);
}

asl_status asl_create(asl_ctx** out, int device, int32_t max_seq_len, int32_t max_kv_heads,
                      int32_t max_q_rows) {
  if (!out) return ASL_EINVAL;
  *out = nullptr;
  if (device < 0 || max_seq_len < 2 || max_kv_heads < 1 || max_q_rows < 1) return ASL_EINVAL;
  if (max_kv_heads > kMaxSelectRows) return ASL_EUNSUPPORTED;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device >= n_dev) return ASL_EHIP;
  asl_ctx* ctx = new (std::nothrow) asl_ctx();
  if (!ctx) return ASL_ENOMEM;
  ctx->device = device;
  ctx->max_seq_len = max_seq_len;
  ctx->max_kv_heads = max_kv_heads;
  ctx->max_q_rows = max_q_rows;
  ctx->err[0] = 0;
  DeviceGuard guard(device);
  if (guard.err != hipSuccess) {
    delete ctx;
    return ASL_EHIP;
  }
  ctx->bytes = carve(nullptr, max_seq_len, max_kv_heads, max_q_rows, nullptr);
  hipError_t e = hipMalloc(&ctx->base, ctx->bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return e == hipErrorOutOfMemory ? ASL_ENOMEM : ASL_EHIP;
  }
  carve(static_cast<char*>(ctx->base), max_seq_len, max_kv_heads, max_q_rows, &ctx->ws);
  ctx->ws.prof = nullptr;
  // the launch counters and the fault word start at zero; the rest needs no initial value
  e = hipMemset(ctx->base, 0, ctx->bytes);
  if (e != hipSuccess) {
    (void)hipFree(ctx->base);
    delete ctx;
    return ASL_EHIP;
  }
  (void)asl::rank_static_prepare(device);   // best effort: asl_rank_static looks it up itself otherwise
  (void)hipGetLastError();
  ctx->side = nullptr;
  ctx->side_pending = false;
  ctx->ev_fork = ctx->ev_join = nullptr;
  e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
  if (e != hipSuccess) {
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    (void)hipFree(ctx->base);
    delete ctx;
    return ASL_EHIP;
  }
  *out = ctx;
  return ASL_OK;
}

static void prof_release(asl_ctx* ctx) {
  asl::Prof& pf = ctx->prof;
  for (int i = 0; i < pf.cap; ++i) {
    (void)hipEventDestroy(pf.start[i]);
    (void)hipEventDestroy(pf.stop[i]);
  }
  delete[] pf.start;
  delete[] pf.stop;
  delete[] pf.id;
  pf = asl::Prof();
  ctx->ws.prof = nullptr;
}

asl_status asl_profile_enable(asl_ctx* ctx, uint32_t kernel_mask, int32_t max_records) {
  if (!ctx) return ASL_EINVAL;
  if (max_records < 0 || max_records > (1 << 20)) return fail(ctx, ASL_EINVAL, "max_records out of range");
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  prof_release(ctx);
  if (kernel_mask == 0 || max_records == 0) return ASL_OK;
  asl::Prof& pf = ctx->prof;
  pf.start = new (std::nothrow) hipEvent_t[max_records];
  pf.stop = new (std::nothrow) hipEvent_t[max_records];
  pf.id = new (std::nothrow) int[max_records];
  if (!pf.start || !pf.stop || !pf.id) {
    delete[] pf.start; delete[] pf.stop; delete[] pf.id;
    pf = asl::Prof();
    return fail(ctx, ASL_ENOMEM, "profile buffers");
  }
  for (int i = 0; i < max_records; ++i) {
    hipError_t e = hipEventCreate(&pf.start[i]);
    if (e == hipSuccess) e = hipEventCreate(&pf.stop[i]);
    if (e != hipSuccess) {
      pf.cap = i;
      prof_release(ctx);
      return hip_fail(ctx, e, "hipEventCreate");
    }
    pf.cap = i + 1;
  }
  pf.mask = kernel_mask;
  pf.n = 0;
  ctx->ws.prof = &ctx->prof;
  return ASL_OK;
}

asl_status asl_profile_collect(asl_ctx* ctx, int32_t kernel_id, double* total_ms, int32_t* launches) {
  if (!ctx) return ASL_EINVAL;
  if (!total_ms || !launches) return fail(ctx, ASL_EINVAL, "null output pointer");
  if (kernel_id < -1 || kernel_id >= asl::kKernCount) return fail(ctx, ASL_EINVAL, "unknown kernel id");
  *total_ms = 0.0;
  *launches = 0;
  asl::Prof& pf = ctx->prof;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  for (int i = 0; i < pf.n; ++i) {
    if (pf.id[i] != kernel_id) continue;
    hipError_t e = hipEventSynchronize(pf.stop[i]);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, pf.start[i], pf.stop[i]);
    if (e != hipSuccess) return hip_fail(ctx, e, "event read");
    *total_ms += ms;
    *launches += 1;
  }
  if (kernel_id == -1) pf.n = 0;          // -1: forget the records taken so far
  return ASL_OK;
}

asl_status asl_destroy(asl_ctx* ctx) {
  if (!ctx) return ASL_EINVAL;
  DeviceGuard guard(ctx->device);
  prof_release(ctx);
  (void)hipStreamSynchronize(ctx->side);
  (void)hipEventDestroy(ctx->ev_join);
  (void)hipEventDestroy(ctx->ev_fork);
  (void)hipStreamDestroy(ctx->side);
  hipError_t e = hipFree(ctx->base);
  delete ctx;
  return e == hipSuccess ? ASL_OK : ASL_EHIP;
}

const char* asl_last_error(const asl_ctx* ctx) { return ctx ? ctx->err : "null context"; }

// Stride and alignment rules of the scoring kernels' operands.
static asl_status check_score_operands(asl_ctx* ctx, const asl_params* p, const void* q_obs, const void* k) {
  if (p->k_stride_tok < p->head_dim || p->k_stride_head < 0)
    return fail(ctx, ASL_EINVAL, "k strides must satisfy stride_tok >= d, stride_head >= 0");
  const int eb = elem_bytes(p->dtype);
  if (asl::score_mfma_supported(*p) &&
      (!aligned16(q_obs) || !aligned16(k) || (p->k_stride_tok * eb) % 16 != 0 ||
       (p->k_stride_head * eb) % 16 != 0))
    return fail(ctx, ASL_EUNSUPPORTED, "q_obs/k must be 16-byte aligned with 16-byte-multiple strides");
  // the plain-FMA kernels walk every key with one thread per query row or per key: refuse the sizes
  // at which that would take seconds rather than hand back a call that looks hung
  if (!asl::score_mfma_supported(*p) || (p->flags & ASL_FLAG_GENERIC_SCORE)) {
    const double work = (double)p->n_q_heads * p->window * (double)p->seq_len * p->head_dim;
    if (work > 6.0e11)
      return fail(ctx, ASL_EUNSUPPORTED,
                  "this shape (dtype/head_dim/G*W) has no MFMA scoring kernel and is too large for the plain one");
  }
  return ASL_OK;
}

// Scoring + pooling.  With wait_side set, the pooling kernel (the first one that overwrites the
// score rows) is ordered behind the side-stream work a deferred asl_layer_step left behind.
static asl_status score_layer_impl(asl_ctx* ctx, const asl_params* p, const void* q_obs, const void* k,
                                   const float* lse, float* p_head, float* s_all, void* stream, bool wait_side,
                                   bool want_sample) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!q_obs || !k || !p_head || !s_all) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  st = check_score_operands(ctx, p, q_obs, k);
  if (st != ASL_OK) return st;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipStream_t hs = static_cast<hipStream_t>(stream);
  hipError_t e = asl::launch_score(*p, ctx->ws, q_obs, k, lse, nullptr, hs);
  if (e != hipSuccess) return hip_fail(ctx, e, "score launch");
  if (wait_side && ctx->side_pending) {
    e = hipStreamWaitEvent(hs, ctx->ev_join, 0);
    if (e != hipSuccess) return hip_fail(ctx, e, "join");
    ctx->side_pending = false;
  }
  const int T = p->seq_len - p->window;
  e = asl::launch_pool(ctx->ws.prof, ctx->ws.u_group, p->n_kv_heads, T, p->pool_kernel, p_head, s_all,
                       want_sample ? ctx->ws.sel_sample : nullptr, hs);
  if (e != hipSuccess) return hip_fail(ctx, e, "pool launch");
  return ASL_OK;
}

asl_status asl_score_layer(asl_ctx* ctx, const asl_params* p, const void* q_obs, const void* k,
                           const float* lse, float* p_head, float* s_all, void* stream) {
  return score_layer_impl(ctx, p, q_obs, k, lse, p_head, s_all, stream, false, false);
}

asl_status asl_window_lse(asl_ctx* ctx, const asl_params* p, const void* q_obs, const void* k,
                          float* lse_out, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!q_obs || !k || !lse_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  st = check_score_operands(ctx, p, q_obs, k);
  if (st != ASL_OK) return st;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipError_t e = asl::launch_score(*p, ctx->ws, q_obs, k, nullptr, lse_out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "score launch");
  return ASL_OK;
}

asl_status asl_pool(asl_ctx* ctx, const float* u, int32_t rows, int32_t T, int32_t S, float* p_out,
                    float* s_out, void* stream) {
  if (!ctx) return ASL_EINVAL;
  if (!u || !p_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if (rows < 1 || T < 1) return fail(ctx, ASL_EINVAL, "need rows >= 1 and T >= 1");
  if (S < 1 || S % 2 == 0) return fail(ctx, ASL_EINVAL, "pool kernel S must be odd and >= 1 (S=%d)", S);
  if (S > kMaxPoolKernel) return fail(ctx, ASL_EUNSUPPORTED, "pool kernel S > %d not supported", kMaxPoolKernel);
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipError_t e = asl::launch_pool(ctx->ws.prof, u, rows, T, S, p_out, s_out, nullptr, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "pool launch");
  return ASL_OK;
}

// The workgroups of a sort launch (one per kSortTile elements) wait for each other, so they must
// fit on the device at once.
static asl_status check_sort_size(asl_ctx* ctx, int32_t T) {
  if (T > asl::rank_max_tokens())
    return fail(ctx, ASL_EUNSUPPORTED, "T=%d is more than one ranking launch can hold on this device (%lld tokens)", T,
                (long long)asl::rank_max_tokens());
  return ASL_OK;
}

asl_status asl_rank(asl_ctx* ctx, const float* s, int32_t T, int32_t* rank_out, void* stream) {
  if (!ctx) return ASL_EINVAL;
  if (!s || !rank_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if (T < 1) return fail(ctx, ASL_EINVAL, "need T >= 1");
  if (T > ctx->max_seq_len) return fail(ctx, ASL_ENOMEM, "T=%d exceeds the context limit %d", T, ctx->max_seq_len);
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  asl_status st = check_sort_size(ctx, T);
  if (st != ASL_OK) return st;
  hipError_t e = asl::launch_rank(ctx->ws, s, T, rank_out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "rank launch");
  return ASL_OK;
}

static asl_status rankvar_checks(asl_ctx* ctx, int32_t l_obs, int32_t T, int32_t layer_idx, int32_t k) {
  if (l_obs < 2 || l_obs > 64) return fail(ctx, ASL_EINVAL, "need 2 <= L_obs <= 64 (L_obs=%d)", l_obs);
  if (T < 1 || layer_idx < 0 || k < 1) return fail(ctx, ASL_EINVAL, "need T >= 1, layer_idx >= 0, k >= 1");
  // sum over <= T tokens of n^2 * variance <= n^2 * T^2 / 4 each must fit in 64 bits
  const long double bound = (long double)l_obs * l_obs * (long double)T * T * T / 4.0L;
  if (bound >= 18446744073709551615.0L)
    return fail(ctx, ASL_EUNSUPPORTED, "L_obs^2 * T^3 / 4 does not fit in 64 bits (L_obs=%d T=%d)", l_obs, T);
  return ASL_OK;
}

asl_status asl_rankvar(asl_ctx* ctx, const int32_t* rank_ring, int32_t l_obs, int32_t T,
                       int32_t layer_idx, int32_t l_min, int32_t k, double tau, asl_state* state,
                       asl_stat* out, void* stream) {
  if (!ctx) return ASL_EINVAL;
  if (!rank_ring || !state || !out) return fail(ctx, ASL_EINVAL, "null pointer");
  asl_status st = rankvar_checks(ctx, l_obs, T, layer_idx, k);
  if (st != ASL_OK) return st;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipStream_t hs = static_cast<hipStream_t>(stream);
  hipError_t e = (layer_idx < l_min)
                     ? asl::launch_stat_skip(ctx->ws.prof, out, state, layer_idx, l_obs, 0, hs)
                     : asl::launch_rankvar(ctx->ws, rank_ring, l_obs, T, layer_idx, k, tau, 0, state, out, hs);
  if (e != hipSuccess) return hip_fail(ctx, e, "rankvar launch");
  return ASL_OK;
}

asl_status asl_rank_stat(asl_ctx* ctx, const asl_params* p, const float* s_all, int32_t layer_idx,
                         int32_t l_min, int32_t l_obs, double tau, int32_t* rank_ring,
                         asl_state* state, asl_stat* out, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!s_all || !rank_ring || !state || !out) return fail(ctx, ASL_EINVAL, "null pointer");
  const int T = p->seq_len - p->window;
  const int k = (p->budget < p->seq_len ? p->budget : p->seq_len) - p->window;
  st = rankvar_checks(ctx, l_obs, T, layer_idx, k);
  if (st != ASL_OK) return st;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipStream_t hs = static_cast<hipStream_t>(stream);
  st = check_sort_size(ctx, T);
  if (st != ASL_OK) return st;
  int32_t* row = rank_ring + (int64_t)(layer_idx % l_obs) * T;
  hipError_t e = asl::launch_rank(ctx->ws, s_all, T, row, hs);
  if (e != hipSuccess) return hip_fail(ctx, e, "rank launch");
  e = (layer_idx < l_min)
          ? asl::launch_stat_skip(ctx->ws.prof, out, state, layer_idx, l_obs, 1, hs)
          : asl::launch_rankvar(ctx->ws, rank_ring, l_obs, T, layer_idx, k, tau, 1, state, out, hs);
  if (e != hipSuccess) return hip_fail(ctx, e, "rankvar launch");
  return ASL_OK;
}

asl_status asl_select_topk(asl_ctx* ctx, const asl_params* p, const float* scores, int32_t rows,
                           int32_t* idx_out, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!scores || !idx_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if (rows < 1) return fail(ctx, ASL_EINVAL, "need rows >= 1");
  if (rows > ctx->max_kv_heads && rows > 1)
    return fail(ctx, ASL_ENOMEM, "rows=%d exceeds the context limit %d", rows, ctx->max_kv_heads);
  const int T = p->seq_len - p->window;
  const int k = (p->budget < p->seq_len ? p->budget : p->seq_len) - p->window;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipError_t e = asl::launch_select(ctx->ws, scores, rows, T, k, p->window, idx_out,
                                    static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "select launch");
  return ASL_OK;
}

// Validates the operands of a one-layer KV compaction and fills the kernel's argument block.
static asl_status make_gather_args(asl_ctx* ctx, const asl_params* p, const void* k, const void* v,
                                   const int32_t* idx, int32_t idx_rows, int32_t n_idx, void* k_out, void* v_out,
                                   asl::GatherArgs* out) {
  if (!k || !idx || !k_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if ((v == nullptr) != (v_out == nullptr)) return fail(ctx, ASL_EINVAL, "v and v_out must both be given or both be null");
  if (idx_rows != 1 && idx_rows != p->n_kv_heads)
    return fail(ctx, ASL_EINVAL, "idx_rows must be 1 or Hk (got %d)", idx_rows);
  if (n_idx < 0) return fail(ctx, ASL_EINVAL, "n_idx must be >= 0");
  const int eb = elem_bytes(p->dtype);
  const int64_t row_bytes = (int64_t)p->head_dim * eb;
  if (row_bytes % 16 != 0 || !aligned16(k) || !aligned16(k_out) || (p->k_stride_tok * eb) % 16 != 0 ||
      (p->k_stride_head * eb) % 16 != 0 ||
      (v && (!aligned16(v) || !aligned16(v_out) || (p->v_stride_tok * eb) % 16 != 0 ||
             (p->v_stride_head * eb) % 16 != 0)))
    return fail(ctx, ASL_EUNSUPPORTED, "gather needs 16-byte aligned rows, pointers and strides");
  if (p->k_stride_tok < p->head_dim || (v && p->v_stride_tok < p->head_dim))
    return fail(ctx, ASL_EINVAL, "token stride smaller than head_dim");
  asl::GatherArgs ga = {};
  ga.k = static_cast<const char*>(k);
  ga.v = static_cast<const char*>(v);
  ga.k_out = static_cast<char*>(k_out);
  ga.v_out = static_cast<char*>(v_out);
  ga.idx = idx;
  ga.ksh = p->k_stride_head * eb;
  ga.kst = p->k_stride_tok * eb;
  ga.vsh = p->v_stride_head * eb;
  ga.vst = p->v_stride_tok * eb;
  ga.idx_rows = idx_rows;
  ga.n_idx = n_idx;
  ga.cpr = (int)(row_bytes / 16);
  ga.n_tensors = v ? 2 : 1;
  *out = ga;
  return ASL_OK;
}

asl_status asl_gather_kv(asl_ctx* ctx, const asl_params* p, const void* k, const void* v,
                         const int32_t* idx, int32_t idx_rows, int32_t n_idx, void* k_out,
                         void* v_out, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  asl::GatherArgs ga;
  st = make_gather_args(ctx, p, k, v, idx, idx_rows, n_idx, k_out, v_out, &ga);
  if (st != ASL_OK) return st;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipError_t e = asl::launch_gather(ctx->ws.prof, ga, p->n_kv_heads, 1, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "gather launch");
  return ASL_OK;
}

asl_status asl_gather_kv_layers(asl_ctx* ctx, const asl_params* p, const void* const* k_ptrs,
                                const void* const* v_ptrs, const int32_t* idx, int32_t idx_rows,
                                int32_t n_idx, int32_t n_layers, void* const* k_out_ptrs,
                                void* const* v_out_ptrs, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!k_ptrs || !idx || !k_out_ptrs) return fail(ctx, ASL_EINVAL, "null pointer");
  if ((v_ptrs == nullptr) != (v_out_ptrs == nullptr))
    return fail(ctx, ASL_EINVAL, "v_ptrs and v_out_ptrs must both be given or both be null");
  if (idx_rows != 1 && idx_rows != p->n_kv_heads)
    return fail(ctx, ASL_EINVAL, "idx_rows must be 1 or Hk (got %d)", idx_rows);
  if (n_idx < 0 || n_layers < 0) return fail(ctx, ASL_EINVAL, "n_idx and n_layers must be >= 0");
  if (n_layers > 16384) return fail(ctx, ASL_EUNSUPPORTED, "more than 16384 layers per call");
  const int eb = elem_bytes(p->dtype);
  const int64_t row_bytes = (int64_t)p->head_dim * eb;
  // the per-layer pointers live in device memory and are not inspected here: their 16-byte
  // alignment is the caller's contract
  if (row_bytes % 16 != 0 || (p->k_stride_tok * eb) % 16 != 0 || (p->k_stride_head * eb) % 16 != 0 ||
      (v_ptrs && ((p->v_stride_tok * eb) % 16 != 0 || (p->v_stride_head * eb) % 16 != 0)))
    return fail(ctx, ASL_EUNSUPPORTED, "gather needs 16-byte aligned rows and strides");
  if (p->k_stride_tok < p->head_dim || (v_ptrs && p->v_stride_tok < p->head_dim))
    return fail(ctx, ASL_EINVAL, "token stride smaller than head_dim");
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  asl::GatherArgs ga = {};
  ga.k_ptrs = k_ptrs;
  ga.v_ptrs = v_ptrs;
  ga.k_out_ptrs = k_out_ptrs;
  ga.v_out_ptrs = v_out_ptrs;
  ga.idx = idx;
  ga.ksh = p->k_stride_head * eb;
  ga.kst = p->k_stride_tok * eb;
  ga.vsh = p->v_stride_head * eb;
  ga.vst = p->v_stride_tok * eb;
  ga.idx_rows = idx_rows;
  ga.n_idx = n_idx;
  ga.cpr = (int)(row_bytes / 16);
  ga.n_tensors = v_ptrs ? 2 : 1;
  hipError_t e = asl::launch_gather(ctx->ws.prof, ga, p->n_kv_heads, n_layers, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "gather launch");
  return ASL_OK;
}

asl_status asl_gather_rows(asl_ctx* ctx, const void* src, int64_t src_row_stride_bytes, int32_t row_bytes,
                           const int32_t* idx, int32_t n_idx, void* dst, void* stream) {
  if (!ctx) return ASL_EINVAL;
  if (!src || !idx || !dst) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if (row_bytes < 1 || n_idx < 0 || src_row_stride_bytes < row_bytes)
    return fail(ctx, ASL_EINVAL, "need row_bytes >= 1, n_idx >= 0, stride >= row_bytes");
  if (row_bytes % 16 != 0 || src_row_stride_bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
    return fail(ctx, ASL_EUNSUPPORTED, "gather needs 16-byte aligned rows, pointers and strides");
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  asl::GatherArgs ga = {};
  ga.k = static_cast<const char*>(src);
  ga.k_out = static_cast<char*>(dst);
  ga.idx = idx;
  ga.kst = src_row_stride_bytes;
  ga.idx_rows = 1;
  ga.n_idx = n_idx;
  ga.cpr = row_bytes / 16;
  ga.n_tensors = 1;
  hipError_t e = asl::launch_gather(ctx->ws.prof, ga, 1, 1, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "gather launch");
  return ASL_OK;
}

asl_status asl_layer_step(asl_ctx* ctx, const asl_params* p, const void* q_obs, const void* k, const void* v,
                          const float* lse, int32_t layer_idx, int32_t l_min, int32_t l_obs, double tau,
                          float* scores, int32_t* rank_ring, asl_state* state, asl_stat* out,
                          int32_t* idx_out, void* k_out, void* v_out, void* stream) {
  asl_status st = check_params(ctx, p);
  if (st != ASL_OK) return st;
  if (!scores || !idx_out) return fail(ctx, ASL_EINVAL, "null tensor pointer");
  if (p->n_kv_heads + 1 > ctx->max_kv_heads)
    return fail(ctx, ASL_ENOMEM, "asl_layer_step selects Hk+1 rows: create the context with max_kv_heads >= %d",
                p->n_kv_heads + 1);
  const int Hk = p->n_kv_heads, T = p->seq_len - p->window;
  const int k_sel = (p->budget < p->seq_len ? p->budget : p->seq_len) - p->window;
  float* p_head = scores;
  float* s_all = scores + (int64_t)Hk * T;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  // when the four-launch tail will follow, the pooling kernel leaves the top-k's sample behind
  const bool fused = !(p->flags & ASL_FLAG_DEFER_JOIN) && asl::tail_takes(ctx->ws, Hk + 1, T);
  st = score_layer_impl(ctx, p, q_obs, k, lse, p_head, s_all, stream, true, fused);
  if (st != ASL_OK) return st;
  if (fused) {
    // one stream: launch i carries pass i of the ranking sort and stage i of top-k + compaction
    if (!rank_ring || !state || !out) return fail(ctx, ASL_EINVAL, "null pointer");
    st = rankvar_checks(ctx, l_obs, T, layer_idx, k_sel);
    if (st != ASL_OK) return st;
    asl::GatherArgs ga;
    if (k_out != nullptr) {
      st = make_gather_args(ctx, p, k, v, idx_out, Hk, k_sel + p->window, k_out, v_out, &ga);
      if (st != ASL_OK) return st;
    }
    bool taken = false;
    int32_t* row = rank_ring + (int64_t)(layer_idx % l_obs) * T;
    // below L_min nothing is evaluated: the statistic's place in the last launch stays empty and the
    // state is advanced by the one-thread kernel instead
    const asl::RankvarArgs ra = asl::rankvar_args(ctx->ws, rank_ring, l_obs, T, layer_idx, k_sel, tau, 1, state, out);
    hipError_t et = asl::launch_tail(ctx->ws, scores, Hk + 1, T, k_sel, p->window, row, idx_out,
                                     k_out != nullptr ? &ga : nullptr, Hk, true, layer_idx < l_min ? nullptr : &ra, hs,
                                     &taken);
    if (et != hipSuccess) return hip_fail(ctx, et, "tail launch");
    if (taken) {
      if (layer_idx < l_min) {
        et = asl::launch_stat_skip(ctx->ws.prof, out, state, layer_idx, l_obs, 1, hs);
        if (et != hipSuccess) return hip_fail(ctx, et, "rankvar launch");
      }
      return ASL_OK;
    }
    // sizes these launches do not take: the two-stream sequence of single calls below
  }
  // fork: top-k + KV compaction on the side stream, ranking + statistic on the caller's stream
  hipError_t e = hipEventRecord(ctx->ev_fork, hs);
  if (e == hipSuccess) e = hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0);
  if (e != hipSuccess) return hip_fail(ctx, e, "fork");
  // the longer chain (ranking + statistic) is queued first and stays on the caller's stream
  asl_status st_main = asl_rank_stat(ctx, p, s_all, layer_idx, l_min, l_obs, tau, rank_ring, state, out, stream);
  asl_status st_side = asl_select_topk(ctx, p, scores, Hk + 1, idx_out, ctx->side);
  if (st_side == ASL_OK && k_out != nullptr)
    st_side = asl_gather_kv(ctx, p, k, v, idx_out, Hk, k_sel + p->window, k_out, v_out, ctx->side);
  e = hipEventRecord(ctx->ev_join, ctx->side);
  // join now, or leave it to the next asl_layer_step / asl_join; a failed launch always joins, so
  // that the side stream never stays forked (e.g. under capture)
  const bool defer = (p->flags & ASL_FLAG_DEFER_JOIN) && st_side == ASL_OK && st_main == ASL_OK && e == hipSuccess;
  if (defer) {
    ctx->side_pending = true;
  } else if (e == hipSuccess) {
    e = hipStreamWaitEvent(hs, ctx->ev_join, 0);
  }
  if (st_side != ASL_OK) return st_side;
  if (st_main != ASL_OK) return st_main;
  if (e != hipSuccess) return hip_fail(ctx, e, "join");
  return ASL_OK;
}

asl_status asl_device_fault(asl_ctx* ctx, int32_t* fault_out) {
  if (!ctx) return ASL_EINVAL;
  if (!fault_out) return fail(ctx, ASL_EINVAL, "null output pointer");
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  uint32_t v = 0;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(&v, ctx->ws.fault, sizeof(v), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(ctx, e, "fault word read");
  *fault_out = (int32_t)v;
  if (v != 0) {
    const uint32_t zero = 0;
    e = hipMemcpy(ctx->ws.fault, &zero, sizeof(zero), hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(ctx, e, "fault word reset");
  }
  return ASL_OK;
}

asl_status asl_join(asl_ctx* ctx, void* stream) {
  if (!ctx) return ASL_EINVAL;
  if (!ctx->side_pending) return ASL_OK;
  DeviceGuard guard(ctx->device);
  if (guard.err != hipSuccess) return hip_fail(ctx, guard.err, "set device");
  hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), ctx->ev_join, 0);
  if (e != hipSuccess) return hip_fail(ctx, e, "join");
  ctx->side_pending = false;
  return ASL_OK;
}

#pragma GCC visibility pop
}  // extern "C"
