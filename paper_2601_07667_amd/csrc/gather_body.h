// Device code of the row-gather kernel (see gather.hip), written as a function so that another
// kernel can host it beside a second body.
#pragma once
#include "asl_internal.h"

namespace asl {

constexpr int kGatherThreads = 256;
constexpr int kGatherUnroll = 4;      // pieces per thread (the body is written out for four)

// Workgroup (bx, h, which, layer) of NT threads: bx = block of NT * kGatherUnroll pieces of the slab
// of KV head h, tensor `which` (0 = K, 1 = V), layer `layer`.  Pieces of a slab are numbered
// q = row * cpr + c (row = output row, c = 16-byte piece of the row).
template <bool POW2, int NT>
__device__ __forceinline__ void gather_body(const GatherArgs& a, int bx, int h, int which, int layer) {
  const char* src_base;
  char* dst_base;
  if (a.k_ptrs != nullptr) {                        // per-layer allocations
    src_base = static_cast<const char*>(which == 0 ? a.k_ptrs[layer] : a.v_ptrs[layer]);
    dst_base = static_cast<char*>(which == 0 ? a.k_out_ptrs[layer] : a.v_out_ptrs[layer]);
  } else {
    src_base = which == 0 ? a.k : a.v;
    dst_base = which == 0 ? a.k_out : a.v_out;
  }
  const int64_t sh = which == 0 ? a.ksh : a.vsh, stt = which == 0 ? a.kst : a.vst;
  src_base += (int64_t)h * sh;
  dst_base += (int64_t)h * a.n_idx * ((int64_t)a.cpr * 16);
  const int32_t* idx = a.idx + ((int64_t)layer * a.idx_rows + (a.idx_rows == 1 ? 0 : h)) * a.n_idx;
  const uint32_t total = (uint32_t)a.n_idx * (uint32_t)a.cpr;          // < 2^31, checked by the host
  const uint32_t q0 = (uint32_t)bx * (NT * kGatherUnroll) + threadIdx.x;
  // The tensors are device (global) memory: say so, so that plain global loads and stores are used.
  typedef const char __attribute__((address_space(1))) * GSrc;
  typedef char __attribute__((address_space(1))) * GDst;
  typedef uint32_t Piece __attribute__((ext_vector_type(4)));          // 16 bytes
  typedef const Piece __attribute__((address_space(1))) * GSrc16;
  typedef Piece __attribute__((address_space(1))) * GDst16;
  typedef const int32_t __attribute__((address_space(1))) * GIdx;
  const GSrc src = (GSrc)src_base;
  const GDst dst = (GDst)dst_base;
  const GIdx gi = (GIdx)idx;
  // Loads are unconditional (piece numbers past the end are clamped to the last piece) so that all
  // four index loads, then all four row loads, are in flight together; only the stores are
  // predicated.  Written out rather than looped: the values must stay in registers.
  const uint32_t last = total - 1u;
  const uint32_t qa = q0, qb = q0 + NT, qc = q0 + 2 * NT, qd = q0 + 3 * NT;
  const uint32_t ca = min(qa, last), cb = min(qb, last), cc = min(qc, last), cd = min(qd, last);
  const uint32_t cpr = (uint32_t)a.cpr;
  const uint32_t ra = POW2 ? (ca >> a.cpr_shift) : (ca / cpr), rb = POW2 ? (cb >> a.cpr_shift) : (cb / cpr);
  const uint32_t rc = POW2 ? (cc >> a.cpr_shift) : (cc / cpr), rd = POW2 ? (cd >> a.cpr_shift) : (cd / cpr);
  const int ta = gi[ra], tb = gi[rb], tc = gi[rc], td = gi[rd];
  const Piece va = *(GSrc16)(src + (int64_t)ta * stt + (int64_t)(ca - ra * cpr) * 16);
  const Piece vb = *(GSrc16)(src + (int64_t)tb * stt + (int64_t)(cb - rb * cpr) * 16);
  const Piece vc = *(GSrc16)(src + (int64_t)tc * stt + (int64_t)(cc - rc * cpr) * 16);
  const Piece vd = *(GSrc16)(src + (int64_t)td * stt + (int64_t)(cd - rd * cpr) * 16);
  if (qa < total) *(GDst16)(dst + (int64_t)qa * 16) = va;
  if (qb < total) *(GDst16)(dst + (int64_t)qb * 16) = vb;
  if (qc < total) *(GDst16)(dst + (int64_t)qc * 16) = vc;
  if (qd < total) *(GDst16)(dst + (int64_t)qd * 16) = vd;
}

}  // namespace asl
