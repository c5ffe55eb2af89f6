// Device code of asl_select's three kernels (see select.hip for the method), written as functions
// over explicit shared-state structs so that another kernel can host them beside a second body.
#pragma once
#include "asl_internal.h"

namespace asl {

constexpr int kFinThreads = 1024;                      // workgroup of all three kernels
constexpr int kFinWaves = kFinThreads / 64;
constexpr int kFinPerThread = 8;                       // consecutive elements per thread in the ordered write
constexpr int kFilterThreads = 256;                    // filter workgroup of its own launch over many tiles ...
constexpr int kFilterSmallFrom = 2048;                 // ... (rows x tiles per row) from this many on; kFinThreads below
constexpr uint32_t kSegOverflow = 0xffffffffu;         // a tile's count when its segment was too small
static_assert(kSelTile % kFinThreads == 0 && kSelTile % kFilterThreads == 0, "filter tile geometry");

// Rank m of the sample key taken as the bound: f = n_s / T of the row is sampled, the top-k members
// among the sample are ~Binomial(n_s, k / T) with mean k f; m = k f + 5 sqrt(c k f) + 4 leaves the
// bound too low with probability < 1e-6.  c = 1 for single sampled keys; c = `run` when the sample
// consists of runs of `run` neighbouring keys, which may be as correlated as identical (pooled
// scores are): the count's variance is then at most `run` times the binomial one.
__host__ __device__ inline int sel_sample_rank(int T, int k, int n_s, int run) {
  const float kf = (float)k * (float)n_s / (float)T;
  const int m = (int)(kf + 5.0f * sqrtf((float)run * kf) + 4.0f);
  return m;                                            // >= n_s means: no usable bound, admit everything
}
// Without a prepared sample the bound kernel reads runs of kSelSampleRun neighbouring keys, one run
// per kSelSampleRun sample strides: the same number of keys from a quarter of the cache lines.
constexpr int kSelSampleRun = 4;
static_assert(kSelMaxSample % kFinThreads == 0, "the bound kernel's threads share the sample evenly");

// Exclusive prefix over the workgroup's threads of two counters (kFinThreads threads), plus totals.
__device__ __forceinline__ void block_scan2(uint32_t a, uint32_t b, uint32_t* sm /* 2*kFinWaves+2 */,
                                            uint32_t& a_excl, uint32_t& b_excl, uint32_t& a_tot, uint32_t& b_tot) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const uint32_t ai = wave_prefix_sum(a), bi = wave_prefix_sum(b);
  __syncthreads();                                     // sm may still be in use
  if (lane == 63) {
    sm[wave] = ai;
    sm[kFinWaves + wave] = bi;
  }
  __syncthreads();
  uint32_t ab = 0, bb = 0, at = 0, bt = 0;
  for (int w = 0; w < kFinWaves; ++w) {
    const uint32_t x = sm[w], y = sm[kFinWaves + w];
    ab += (w < wave) ? x : 0u;
    bb += (w < wave) ? y : 0u;
    at += x;
    bt += y;
  }
  a_excl = ab + ai - a;
  b_excl = bb + bi - b;
  a_tot = at;
  b_tot = bt;
}

// Radix select over n keys read through `key_at(i)`: returns the k-th smallest key (1 <= k <= n)
// and how many of the keys equal to it belong to the k smallest (k_rem >= 1).  All kFinThreads
// threads take part.  The keys' common leading bits are skipped: digits are taken from
// key - min over the bits in which min and max differ, so the first digit already spreads the keys
// over the bins (scores of one row share their sign and most of their exponent).
// h: kHistWords-word LDS histogram (bank-staggered copies), sm: >= 2 * kFinWaves + 2 words.
constexpr int kSelBatch = 4;                           // keys a thread reads together in the selection loops
template <typename KeyAt>
__device__ __forceinline__ void radix_select_block(int n, uint32_t k, KeyAt key_at, uint32_t* h, uint32_t* sm,
                                                   uint32_t& thr_out, uint32_t& k_rem_out) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // The loops over the keys take kSelBatch of a thread's keys at a time (positions past the end
  // re-read the thread's first key of the batch), so that their reads are in flight together.
  uint32_t lo = 0xffffffffu, hi = 0u;
  for (int i0 = tid; i0 < n; i0 += kSelBatch * kFinThreads) {
    uint32_t key[kSelBatch];
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) key[u] = key_at(i0 + u * kFinThreads < n ? i0 + u * kFinThreads : i0);
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      lo = key[u] < lo ? key[u] : lo;
      hi = key[u] > hi ? key[u] : hi;
    }
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __syncthreads();                                     // sm may still be in use
  if (lane == 0) {
    sm[wave] = lo;
    sm[kFinWaves + wave] = hi;
  }
  __syncthreads();
  for (int w = 0; w < kFinWaves; ++w) {
    const uint32_t l2 = sm[w], h2 = sm[kFinWaves + w];
    lo = l2 < lo ? l2 : lo;
    hi = h2 > hi ? h2 : hi;
  }
  const uint32_t span = hi - lo;
  const int bits = span == 0 ? 0 : 32 - __clz((int)span);
  const int n_pass = (bits + 7) / 8;                   // uniform; 0 when all keys are equal
  uint32_t prefix = 0, k_rem = k;
  for (int pass = 0; pass < n_pass; ++pass) {
    const int shift = 8 * (n_pass - 1 - pass);
    __syncthreads();                                   // h and sm of the previous pass are consumed
    hist_clear(h, tid, kFinThreads);
    __syncthreads();
    for (int i0 = tid; i0 < n; i0 += kSelBatch * kFinThreads) {
      uint32_t v[kSelBatch];
#pragma unroll
      for (int u = 0; u < kSelBatch; ++u) v[u] = key_at(i0 + u * kFinThreads < n ? i0 + u * kFinThreads : i0) - lo;
#pragma unroll
      for (int u = 0; u < kSelBatch; ++u)
        if (i0 + u * kFinThreads < n && (pass == 0 || (v[u] >> (shift + 8)) == prefix)) hist_add(h, tid, (v[u] >> shift) & 255u);
    }
    __syncthreads();
    // exclusive scan of the 256 counts by the first four wavefronts; the digit d with
    // excl < k_rem <= excl + count holds the k-th key
    uint32_t cnt = 0, incl = 0;
    if (tid < 256) {
      cnt = hist_total(h, tid);
      incl = wave_prefix_sum(cnt);
      if (lane == 63) sm[wave] = incl;
    }
    if (tid == 0) {
      sm[4] = 0;                                       // defined even if no digit qualifies
      sm[5] = 1;                                       // (cannot happen while 1 <= k <= n)
    }
    __syncthreads();
    if (tid < 256) {
      uint32_t excl = incl - cnt;
      for (int w = 0; w < wave; ++w) excl += sm[w];
      if (excl < k_rem && excl + cnt >= k_rem) {       // exactly one digit satisfies this
        sm[4] = (uint32_t)tid;
        sm[5] = k_rem - excl;
      }
    }
    __syncthreads();
    prefix = (prefix << 8) | sm[4];
    k_rem = sm[5];
  }
  thr_out = lo + prefix;
  k_rem_out = k_rem;
}

struct SelectArgs {
  const float* scores;           // [rows][T]
  const uint32_t* sample;        // [rows][kSelMaxSample] keys at the sample positions, or null
  int T, n_tiles, k, W;
  uint32_t* bound;               // [rows]
  uint32_t* thr;                 // [rows][2] (threshold key, kept ties) when step 3 spans two launches
  uint32_t* cand_key;            // [rows][n_tiles][kSelSegment]
  uint32_t* cand_idx;
  uint32_t* seg_count;           // [rows][n_tiles]
  int32_t* idx_out;              // [rows][k + W]
};

struct GuessShared {
  uint32_t samp[kSelMaxSample];
  uint32_t h[kHistWords];
  uint32_t sm[2 * kFinWaves + 2];
};

// Step 1: bound[row] = the m-th smallest key of the row's strided sample (0xffffffff: admit all).
__device__ __forceinline__ void select_guess_body(GuessShared& sh, const SelectArgs& a, int row) {
  const int tid = threadIdx.x, T = a.T;
  const int stride = sel_sample_stride(T);
  const bool runs = a.sample == nullptr && stride >= 2;           // stride 1: the sample is the row itself
  const int n_s = runs ? (sel_sample_size(T) / kSelSampleRun) * kSelSampleRun : sel_sample_size(T);
  const int m = sel_sample_rank(T, a.k, n_s, runs ? kSelSampleRun : 1);
  if (m >= n_s) {                                      // uniform
    if (tid == 0) a.bound[row] = 0xffffffffu;
    return;
  }
  // Every thread's keys are loaded before the first is stored (positions past the sample re-read its
  // last key): one memory round trip for the whole sample.
  constexpr int kSampPer = kSelMaxSample / kFinThreads;
  uint32_t v[kSampPer];
  if (a.sample != nullptr) {                           // the producer of the scores left the sample behind
    const uint32_t* sp = a.sample + (int64_t)row * kSelMaxSample;
#pragma unroll
    for (int u = 0; u < kSampPer; ++u) v[u] = sp[min(tid + u * kFinThreads, n_s - 1)];
  } else {
    const float* sr = a.scores + (int64_t)row * T;
    if (runs) {                                        // key j = member j % run of run j / run
#pragma unroll
      for (int u = 0; u < kSampPer; ++u) {
        const int j = min(tid + u * kFinThreads, n_s - 1);
        v[u] = order_key(sr[(j / kSelSampleRun) * (kSelSampleRun * stride) + (j % kSelSampleRun)]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kSampPer; ++u) v[u] = order_key(sr[min(tid + u * kFinThreads, n_s - 1) * stride]);
    }
  }
#pragma unroll
  for (int u = 0; u < kSampPer; ++u)
    if (tid + u * kFinThreads < n_s) sh.samp[tid + u * kFinThreads] = v[u];
  uint32_t thr, k_rem;
  radix_select_block(n_s, (uint32_t)m, [&](int i) { return sh.samp[i]; }, sh.h, sh.sm, thr, k_rem);
  if (tid == 0) a.bound[row] = thr;
}

// key(score) <= bound, decided on the score's bits without forming the key: non-negative scores
// (bits u < 2^31) have key 2^31 - 1 - u, negative ones key u, and -0 counts as +0.  So for a bound
// below 2^31 - 1 exactly the bits in [2^31 - 1 - bound, 2^31 - 1] pass, and for any other bound the
// bits in [0, max(bound, 2^31)] (every non-negative score, -0, and the negative ones up to the
// bound): one subtraction and one unsigned comparison per score.
struct KeepTest {
  uint32_t lo, span;
};
__device__ __forceinline__ KeepTest keep_test(uint32_t bound) {
  KeepTest t;
  if (bound >= 0x7fffffffu) {
    t.lo = 0u;
    t.span = bound > 0x80000000u ? bound : 0x80000000u;
  } else {
    t.lo = 0x7fffffffu - bound;
    t.span = bound;
  }
  return t;
}
__device__ __forceinline__ bool keeps(const KeepTest& t, float score) { return (__float_as_uint(score) - t.lo) <= t.span; }
// Set bits of a wavefront ballot that belong to lanes below the calling one.
__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

struct FilterShared {
  uint32_t wave_tot[kFinWaves];
};

// Step 2: the tile's keys <= bound, in token order, to the tile's segment of the candidate buffer.
// NT threads per workgroup: each wavefront takes kSelTile / (NT / 64) consecutive tokens.
// VEC: a lane reads four neighbouring scores with one 16-byte load (the row must start on a 16-byte
// boundary: T % 4 == 0 and an aligned base); otherwise one score per load.
template <int NT, bool VEC>
__device__ __forceinline__ void select_filter_body(FilterShared& sh, const SelectArgs& a, int row, int tile) {
  constexpr int kWaves = NT / 64, kSelPerWave = kSelTile / kWaves;
  constexpr int kPer = VEC ? 4 : 1;                     // neighbouring tokens per lane and round
  constexpr int kSelRounds = kSelPerWave / (64 * kPer);
  static_assert(kSelRounds >= 1, "filter tile geometry");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, T = a.T;
  const float* sr = a.scores + (int64_t)row * T;
  const int base = tile * kSelTile + wave * kSelPerWave;
  float sc[kSelRounds][kPer];
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {               // all loads in flight before the first use
    const int e = base + (r * 64 + lane) * kPer;
    if (VEC) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e + 3 < T) {
        v = *reinterpret_cast<const float4*>(sr + e);
      } else {                                          // the row's last, partial piece
        if (e < T) v.x = sr[e];
        if (e + 1 < T) v.y = sr[e + 1];
        if (e + 2 < T) v.z = sr[e + 2];
      }
      sc[r][0] = v.x;
      sc[r][1 % kPer] = v.y;
      sc[r][2 % kPer] = v.z;
      sc[r][3 % kPer] = v.w;
    } else {
      sc[r][0] = (e < T) ? sr[e] : 0.f;
    }
  }
  const KeepTest kt = keep_test(a.bound[row]);
  // per round: which of the lane's tokens are kept (bit j), how many lower lanes keep, the round's total
  uint32_t kept[kSelRounds], before[kSelRounds], round_tot[kSelRounds];
  uint32_t w_cnt = 0;
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    const int e0 = base + (r * 64 + lane) * kPer;
    kept[r] = 0;
    before[r] = 0;
    round_tot[r] = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const bool keep = (e0 + j < T) && keeps(kt, sc[r][j]);
      const uint64_t bal = __ballot(keep);
      kept[r] |= keep ? (1u << j) : 0u;
      before[r] += lanes_below(bal);
      round_tot[r] += (uint32_t)__popcll(bal);
    }
    w_cnt += round_tot[r];
  }
  if (lane == 0) sh.wave_tot[wave] = w_cnt;
  __syncthreads();
  uint32_t run = 0, total = 0;
  for (int w = 0; w < kWaves; ++w) {
    run += (w < wave) ? sh.wave_tot[w] : 0u;
    total += sh.wave_tot[w];
  }
  const int64_t seg = ((int64_t)row * a.n_tiles + tile);
  if (tid == 0) a.seg_count[seg] = (total > (uint32_t)kSelSegment) ? kSegOverflow : total;
  if (total > (uint32_t)kSelSegment) return;           // uniform: the finish step takes the whole row instead
  uint32_t* ck = a.cand_key + seg * kSelSegment;
  uint32_t* ci = a.cand_idx + seg * kSelSegment;
#pragma unroll
  for (int r = 0; r < kSelRounds; ++r) {
    // token order inside a round: lane by lane, a lane's kPer tokens in a row.  Few tokens are kept:
    // the loop runs as often as the busiest lane has kept tokens.
    const int e0 = base + (r * 64 + lane) * kPer;
    uint32_t pos = run + before[r], m = kept[r];
    while (m != 0u) {
      const int j = __ffs((int)m) - 1;
      const float f = (j == 0) ? sc[r][0] : (j == 1) ? sc[r][1 % kPer] : (j == 2) ? sc[r][2 % kPer] : sc[r][3 % kPer];
      ck[pos] = order_key(f);
      ci[pos] = (uint32_t)(e0 + j);
      ++pos;
      m &= m - 1u;
    }
    run += round_tot[r];
  }
}

// Ordered write of the kept elements of a sequence of n (key, token) pairs given in token order:
// kept = key < thr, or key == thr and fewer than k_rem equal keys precede it.
template <typename KeyAt, typename TokAt>
__device__ __forceinline__ void ordered_write(int n, uint32_t thr, uint32_t k_rem, int k, KeyAt key_at, TokAt tok_at,
                                              uint32_t* sm, int32_t* __restrict__ out) {
  const int tid = threadIdx.x;
  uint32_t lt_base = 0, eq_base = 0;
  for (int c0 = 0; c0 < n; c0 += kFinThreads * kFinPerThread) {
    const int i0 = c0 + tid * kFinPerThread;
    uint32_t key[kFinPerThread];
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kFinPerThread; ++j) {
      key[j] = (i0 + j < n) ? key_at(i0 + j) : 0xffffffffu;
      lt += (i0 + j < n && key[j] < thr) ? 1u : 0u;
      eq += (i0 + j < n && key[j] == thr) ? 1u : 0u;
    }
    uint32_t lt_excl, eq_excl, lt_tot, eq_tot;
    block_scan2(lt, eq, sm, lt_excl, eq_excl, lt_tot, eq_tot);
    uint32_t lt_run = lt_base + lt_excl, eq_run = eq_base + eq_excl;
#pragma unroll
    for (int j = 0; j < kFinPerThread; ++j) {
      if (i0 + j < n) {
        const bool is_lt = key[j] < thr, is_eq = key[j] == thr;
        if (is_lt || (is_eq && eq_run < k_rem)) {
          const uint32_t pos = lt_run + (eq_run < k_rem ? eq_run : k_rem);
          if (pos < (uint32_t)k) out[pos] = (int32_t)tok_at(i0 + j);      // always true for consistent counts
        }
        lt_run += is_lt ? 1u : 0u;
        eq_run += is_eq ? 1u : 0u;
      }
    }
    lt_base += lt_tot;
    eq_base += eq_tot;
  }
}

// Shared state of step 3; kSelCandCap candidate keys, then kSelCandCap candidate tokens, follow it in
// the workgroup's dynamic LDS.
struct FinishShared {
  uint32_t h[kHistWords];
  uint32_t sm[2 * kFinWaves + 2];
  uint32_t seg_off[kSelMaxRowTiles + 1];
  int whole_row;
  uint32_t pad[2];
};
constexpr size_t kFinishLdsBytes = sizeof(FinishShared) + 2 * (size_t)kSelCandCap * sizeof(uint32_t);

// Step 3 has two halves, usable from one kernel or from two consecutive launches.
// Common start: offsets of the tiles' candidates in the row's candidate sequence and, unless the
// whole row has to be taken instead (sh.whole_row), the candidates copied into LDS.  Returns the
// number of candidates.
__device__ __forceinline__ int finish_load(FinishShared& sh, uint32_t* lds_cand, const SelectArgs& a, int row) {
  const int tid = threadIdx.x, n_tiles = a.n_tiles, k = a.k;
  {
    uint32_t c = 0, over = 0;                          // thread t takes tile t
    if (tid < n_tiles && n_tiles <= kSelMaxRowTiles) {
      c = a.seg_count[(int64_t)row * n_tiles + tid];
      over = (c == kSegOverflow) ? 1u : 0u;
      c = over ? 0u : c;
    }
    uint32_t c_excl, o_excl, c_tot, o_tot;
    block_scan2(c, over, sh.sm, c_excl, o_excl, c_tot, o_tot);
    if (tid < n_tiles && n_tiles <= kSelMaxRowTiles) sh.seg_off[tid] = c_excl;
    if (tid == 0) {
      if (n_tiles <= kSelMaxRowTiles) sh.seg_off[n_tiles] = c_tot;
      sh.whole_row = (n_tiles > kSelMaxRowTiles || o_tot != 0 || c_tot < (uint32_t)k || c_tot > (uint32_t)kSelCandCap) ? 1 : 0;
    }
  }
  __syncthreads();
  if (sh.whole_row) return 0;                          // uniform
  uint32_t* lk = lds_cand;
  uint32_t* li = lds_cand + kSelCandCap;
  // Wavefront w copies tiles w, w + kFinWaves, ..., two tiles and 128 candidates of each at a time:
  // the eight loads of such a step are in flight together (a tile holds ~100 candidates at the
  // usual budgets, so a row takes one memory round trip instead of one per tile and 64 candidates).
  const int lane = tid & 63;
  for (int t0 = tid >> 6; t0 < n_tiles; t0 += 2 * kFinWaves) {
    uint32_t o[2], c[2];
    int64_t seg[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int t = t0 + q * kFinWaves;
      const bool in = t < n_tiles;
      o[q] = in ? sh.seg_off[t] : 0u;
      c[q] = in ? sh.seg_off[t + 1] - o[q] : 0u;
      seg[q] = ((int64_t)row * n_tiles + (in ? t : 0)) * kSelSegment;
    }
    const uint32_t c_max = c[0] > c[1] ? c[0] : c[1];
    for (uint32_t j0 = 0; j0 < c_max; j0 += 128) {
      uint32_t kk[2][2], ii[2][2];
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const uint32_t j = j0 + u * 64 + lane;
          kk[q][u] = 0;
          ii[q][u] = 0;
          if (j < c[q]) {
            kk[q][u] = a.cand_key[seg[q] + j];
            ii[q][u] = a.cand_idx[seg[q] + j];
          }
        }
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const uint32_t j = j0 + u * 64 + lane;
          if (j < c[q]) {
            lk[o[q] + j] = kk[q][u];
            li[o[q] + j] = ii[q][u];
          }
        }
    }
  }
  __syncthreads();
  return (int)sh.seg_off[n_tiles];
}

// First half: the k-th smallest key of the row and how many keys equal to it are kept.
// n: finish_load's result.  With `publish` the pair is also stored for a later launch.
__device__ __forceinline__ void finish_threshold(FinishShared& sh, const uint32_t* lds_cand, const SelectArgs& a, int row,
                                                 int n, bool publish, uint32_t& thr, uint32_t& k_rem) {
  if (!sh.whole_row) {                                 // uniform
    radix_select_block(n, (uint32_t)a.k, [&](int i) { return lds_cand[i]; }, sh.h, sh.sm, thr, k_rem);
  } else {
    const float* sr = a.scores + (int64_t)row * a.T;
    radix_select_block(a.T, (uint32_t)a.k, [&](int i) { return order_key(sr[i]); }, sh.h, sh.sm, thr, k_rem);
  }
  if (publish && threadIdx.x == 0) {
    a.thr[2 * row] = thr;
    a.thr[2 * row + 1] = k_rem;
  }
}

// Second half: the kept tokens in ascending order, then the window tokens.
__device__ __forceinline__ void finish_write(FinishShared& sh, const uint32_t* lds_cand, const SelectArgs& a, int row,
                                             int n, uint32_t thr, uint32_t k_rem) {
  const int tid = threadIdx.x, T = a.T, k = a.k, W = a.W;
  int32_t* out = a.idx_out + (int64_t)row * (k + W);
  if (!sh.whole_row) {                                 // uniform
    const uint32_t* lk = lds_cand;
    const uint32_t* li = lds_cand + kSelCandCap;
    ordered_write(n, thr, k_rem, k, [&](int i) { return lk[i]; }, [&](int i) { return li[i]; }, sh.sm, out);
  } else {
    const float* sr = a.scores + (int64_t)row * T;
    ordered_write(T, thr, k_rem, k, [&](int i) { return order_key(sr[i]); }, [&](int i) { return (uint32_t)i; }, sh.sm, out);
  }
  // window tokens T .. T+W-1 (Alg. 1 step 10: Concat with I_w)
  for (int i = tid; i < W; i += kFinThreads) out[k + i] = T + i;
}

// Step 3 in one kernel: one workgroup per row.
__device__ __forceinline__ void select_finish_body(FinishShared& sh, uint32_t* lds_cand, const SelectArgs& a, int row) {
  const int n = finish_load(sh, lds_cand, a, row);
  uint32_t thr, k_rem;
  finish_threshold(sh, lds_cand, a, row, n, false, thr, k_rem);
  finish_write(sh, lds_cand, a, row, n, thr, k_rem);
}

// Step 3 over two launches: the first stores (threshold key, kept ties) of every row in a.thr ...
__device__ __forceinline__ void select_threshold_body(FinishShared& sh, uint32_t* lds_cand, const SelectArgs& a, int row) {
  const int n = finish_load(sh, lds_cand, a, row);
  uint32_t thr, k_rem;
  finish_threshold(sh, lds_cand, a, row, n, true, thr, k_rem);
}
// ... the second loads the candidates again and writes the indices.
__device__ __forceinline__ void select_write_body(FinishShared& sh, uint32_t* lds_cand, const SelectArgs& a, int row) {
  const int n = finish_load(sh, lds_cand, a, row);
  finish_write(sh, lds_cand, a, row, n, a.thr[2 * row], a.thr[2 * row + 1]);
}

// Arguments of a select over `rows` rows of scores (buffers from the workspace; rows <= ws.sel_rows).
SelectArgs select_args(const Workspace& ws, const float* scores, int T, int k, int W, int32_t* idx_out,
                       bool have_sample);

}  // namespace asl
