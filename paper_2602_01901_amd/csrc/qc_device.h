// Device-side helpers shared by the kernels: element types, 16-byte vector access,
// wave64 / sub-wave reductions on DPP, per-sequence metadata access.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qc_internal.h"

namespace qc {

constexpr float kLog2e = 1.4426950408889634f;

typedef __bf16 bf16_t;

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
  static constexpr int kPer16 = 4;
};
template <> struct ElemTraits<bf16_t> {
  static constexpr int kPer16 = 8;
};

// 16 bytes of T -> floats.
__device__ __forceinline__ void unpack16(const uint4& raw, float (&f)[4], float*) {
  f[0] = __uint_as_float(raw.x);
  f[1] = __uint_as_float(raw.y);
  f[2] = __uint_as_float(raw.z);
  f[3] = __uint_as_float(raw.w);
}
__device__ __forceinline__ void unpack16(const uint4& raw, float (&f)[8], bf16_t*) {
  f[0] = __uint_as_float(raw.x << 16);
  f[1] = __uint_as_float(raw.x & 0xffff0000u);
  f[2] = __uint_as_float(raw.y << 16);
  f[3] = __uint_as_float(raw.y & 0xffff0000u);
  f[4] = __uint_as_float(raw.z << 16);
  f[5] = __uint_as_float(raw.z & 0xffff0000u);
  f[6] = __uint_as_float(raw.w << 16);
  f[7] = __uint_as_float(raw.w & 0xffff0000u);
}

// 16 bytes of a cache row that is read once per launch: loaded with the non-temporal hint (measurably
// faster HBM streaming than ordinary loads on this part).
__device__ __forceinline__ uint4 stream_load16(const char* p) {
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return (float)x; }
// Round-to-nearest-even conversions to the storage type.
__device__ __forceinline__ void store_elem(float* p, float x) { *p = x; }
__device__ __forceinline__ void store_elem(bf16_t* p, float x) { *p = (bf16_t)x; }

// ---- DPP lane exchange (row = 16 lanes) -----------------------------------
template <int kCtrl> __device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, false));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within each 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within each 16

__device__ __forceinline__ float swap32(float x) {  // value held by lane ^ 32
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return __int_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// Sum over aligned groups of kLanes consecutive lanes; every lane receives the total.
template <int kLanes> __device__ __forceinline__ float group_sum(float x) {
  static_assert(kLanes == 8 || kLanes == 16 || kLanes == 32 || kLanes == 64, "group size");
  x += dpp_move<kDppXor1>(x);
  x += dpp_move<kDppXor2>(x);
  x += dpp_move<kDppHalfMirror>(x);
  if (kLanes >= 16) x += dpp_move<kDppMirror>(x);
  if (kLanes >= 32) x += __shfl_xor(x, 16);
  if (kLanes >= 64) x += __shfl_xor(x, 32);
  return x;
}
// Value held by lane `src` (0 .. kLanes-1) of the caller's aligned group of kLanes lanes.
template <int kLanes> __device__ __forceinline__ float group_broadcast(float x, int src) {
  return __shfl(x, src, kLanes);
}
template <int kLanes> __device__ __forceinline__ float group_max(float x) {
  static_assert(kLanes == 8 || kLanes == 16 || kLanes == 32 || kLanes == 64, "group size");
  x = fmaxf(x, dpp_move<kDppXor1>(x));
  x = fmaxf(x, dpp_move<kDppXor2>(x));
  x = fmaxf(x, dpp_move<kDppHalfMirror>(x));
  if (kLanes >= 16) x = fmaxf(x, dpp_move<kDppMirror>(x));
  if (kLanes >= 32) x = fmaxf(x, __shfl_xor(x, 16));
  if (kLanes >= 64) x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}

// Wave-uniform integer that an earlier launch wrote and no lane of this launch writes: fetched through
// the constant address space, so that it arrives by a scalar load instead of a per-lane one.
__device__ __forceinline__ int32_t uniform_load(const int32_t* p) {
  return *(const __attribute__((address_space(4))) int32_t*)(uintptr_t)p;
}

struct SeqMeta {
  int32_t tok0, len0, vis_start, vis_len;
};
// With inherit_all (Global Lazy Attention) the span a lazy layer inherits is the whole prompt.
__device__ __forceinline__ SeqMeta load_meta(const LayerView& lv, int b, int inherit_all = 0) {
  SeqMeta m;
  m.tok0 = uniform_load(lv.meta + META_TOK0 * lv.max_batch + b);
  m.len0 = uniform_load(lv.meta + META_LEN0 * lv.max_batch + b);
  m.vis_start = inherit_all ? 0 : uniform_load(lv.meta + META_VIS_START * lv.max_batch + b);
  m.vis_len = inherit_all ? m.len0 : uniform_load(lv.meta + META_VIS_LEN * lv.max_batch + b);
  return m;
}

// Paged regions: index of row r of head h, given the sequence's page list of the pool (in global memory or
// staged in LDS).
template <typename PageList>
__device__ __forceinline__ int64_t paged_row(PageList pages, int r, int h, int n_heads) {
  return ((int64_t)pages[r >> 6] * n_heads + h) * kPageRows + (r & (kPageRows - 1));
}

// Index of row 0 of (sequence b, head h) in each cache region a layer call touches, in rows.
struct RowBase {
  int64_t k, v, anchor, q;   // k_own, v_own, k_anchor, q_cache
};
__device__ __forceinline__ RowBase row_bases(const LayerView& lv, int b, int h, int n_heads) {
  RowBase r;
  if (!(lv.flags & LV_RAGGED)) {
    const int64_t bh = (int64_t)b * n_heads + h;
    r.k = bh * lv.cap_k;
    r.v = bh * lv.cap_v;
    r.anchor = bh * lv.cap_k_anchor;
    r.q = bh * lv.cap_q;
    return r;
  }
  // per-sequence capacities: sequence b's rows start where those of the sequences before it end
  const int32_t* caps = lv.meta + (META_BLOCKS - ((lv.flags & LV_LATE) ? 1 : 0)) * META_ROWS * lv.max_batch + META_COUNTER_WORDS;
  const int64_t seq = (int64_t)uniform_load(caps + BASE_SEQ * lv.max_batch + b) * n_heads +
                      (int64_t)h * uniform_load(caps + CAP_SEQ * lv.max_batch + b);
  r.v = seq;
  r.anchor = seq;
  r.k = (lv.flags & LV_K_TEXT) ? (int64_t)uniform_load(caps + BASE_TEXT * lv.max_batch + b) * n_heads +
                                     (int64_t)h * uniform_load(caps + CAP_TEXT * lv.max_batch + b)
                               : seq;
  r.q = (lv.flags & LV_Q_VIS) ? (int64_t)uniform_load(caps + BASE_VIS * lv.max_batch + b) * n_heads +
                                    (int64_t)h * uniform_load(caps + CAP_VIS * lv.max_batch + b)
                              : seq;
  return r;
}

// Row indices of one (sequence, head) in either layout, chosen at run time (for the paths that are
// not tuned; the tuned kernels take the layout as a template parameter).
struct RowIndex {
  RowBase rb;
  const int32_t *pk, *pv, *pq;   // page lists of this sequence: k_own's pool, positions, q_cache's pool
  int32_t h, n_heads;
  bool paged;
  __device__ __forceinline__ int64_t k(int r) const { return paged ? paged_row(pk, r, h, n_heads) : rb.k + r; }
  __device__ __forceinline__ int64_t v(int r) const { return paged ? paged_row(pv, r, h, n_heads) : rb.v + r; }
  __device__ __forceinline__ int64_t anchor(int r) const { return paged ? paged_row(pv, r, h, n_heads) : rb.anchor + r; }
  __device__ __forceinline__ int64_t q(int r) const { return paged ? paged_row(pq, r, h, n_heads) : rb.q + r; }
};
__device__ __forceinline__ RowIndex row_index(const LayerView& lv, int b, int h, int n_heads) {
  RowIndex x;
  x.paged = (lv.flags & LV_PAGED) != 0;
  x.h = h;
  x.n_heads = n_heads;
  x.pk = x.pv = x.pq = nullptr;
  x.rb = RowBase{0, 0, 0, 0};
  if (x.paged) {
    x.pk = lv.pt_k + (int64_t)b * lv.pt_k_stride;
    x.pv = lv.pt_seq + (int64_t)b * lv.pt_seq_stride;
    x.pq = lv.pt_q + (int64_t)b * lv.pt_q_stride;
  } else {
    x.rb = row_bases(lv, b, h, n_heads);
  }
  return x;
}

}  // namespace qc
