// Prefill attention, plain-ALU version (paper Eq. 1; Eq. 7 in a lazy layer), used for fp32 and
// for shapes the matrix-core kernel does not cover.  Also holds the cache writer that both
// prefill paths share.
//
// One workgroup takes 16 consecutive query rows of one (sequence, head): four rows per wave.
// Keys are visited in tiles staged in LDS as fp32.  In the score phase a lane is a key; in the
// value phase a lane is a slice of head_dim.  Softmax is the usual running (max, sum) form in
// fp32 with base-2 exponentials.
#include "qc_device.h"

namespace qc {

// Row address of query/key `pos` of sequence `sm`, head h, honouring the lazy substitution:
// inside the visual span a lazy layer reads the Q Cache / the anchor layer's K rows.
template <typename T, int D>
__device__ __forceinline__ const T* q_row_ptr(const PrefillArgs& a, const SeqMeta& sm, const RowIndex& rb, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len)
    return (const T*)a.lv.q_cache + rb.q(pos - sm.vis_start) * D;
  return (const T*)a.q + (int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride;
}
template <typename T, int D>
__device__ __forceinline__ const T* k_row_ptr(const PrefillArgs& a, const SeqMeta& sm, const RowIndex& rb, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len)
    return (const T*)a.lv.k_anchor + rb.anchor(pos) * D;
  return (const T*)a.k + (int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_simple_kernel(PrefillArgs a) {
  constexpr int BQ = 16, RPW = 4;            // query rows per workgroup / per wave
  constexpr int BK = D == 64 ? 64 : 32;      // keys per tile
  constexpr int EPL = ElemTraits<T>::kPer16;
  constexpr int CPR = D / EPL;               // 16-byte chunks per row
  constexpr int DPL = D / 64;                // output columns per lane
  __shared__ float Ks[BK][D + 1];
  __shared__ float Vs[BK][D];
  __shared__ float Qs[BQ][D];
  __shared__ float Ps[4][RPW][BK];

  const int h = blockIdx.y, b = blockIdx.z;
  const SeqMeta sm = load_meta(a.lv, b, a.inherit_all);
  const int len = sm.len0;
  const int q0 = blockIdx.x * BQ;
  if (q0 >= len) return;
  const RowIndex rb = row_index(a.lv, b, h, a.n_heads);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float c = a.scale * kLog2e;

  for (int i = tid; i < BQ * CPR; i += 256) {
    const int r = i / CPR, ch = i % CPR;
    float f[EPL];
    if (q0 + r < len) {
      const uint4 raw = *(const uint4*)(q_row_ptr<T, D>(a, sm, rb, h, q0 + r) + ch * EPL);
      unpack16(raw, f, (T*)nullptr);
    } else {
      for (int j = 0; j < EPL; ++j) f[j] = 0.f;
    }
    for (int j = 0; j < EPL; ++j) Qs[r][ch * EPL + j] = f[j] * c;
  }

  float m[RPW], l[RPW], acc[RPW][DPL];
  for (int r = 0; r < RPW; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
    for (int j = 0; j < DPL; ++j) acc[r][j] = 0.f;
  }
  const int last_q = min(q0 + BQ, len) - 1;
  for (int k0 = 0; k0 <= last_q; k0 += BK) {
    __syncthreads();
    for (int i = tid; i < BK * CPR; i += 256) {
      const int r = i / CPR, ch = i % CPR;
      float kf[EPL], vf[EPL];
      if (k0 + r < len) {
        const uint4 kraw = *(const uint4*)(k_row_ptr<T, D>(a, sm, rb, h, k0 + r) + ch * EPL);
        const uint4 vraw = *(const uint4*)((const T*)a.v + (int64_t)(sm.tok0 + k0 + r) * a.token_stride +
                                          (int64_t)h * a.head_stride + ch * EPL);
        unpack16(kraw, kf, (T*)nullptr);
        unpack16(vraw, vf, (T*)nullptr);
      } else {
        for (int j = 0; j < EPL; ++j) kf[j] = vf[j] = 0.f;
      }
      for (int j = 0; j < EPL; ++j) {
        Ks[r][ch * EPL + j] = kf[j];
        Vs[r][ch * EPL + j] = vf[j];
      }
    }
    __syncthreads();
    for (int r = 0; r < RPW; ++r) {
      const int qi = q0 + wave * RPW + r;
      float sc = -INFINITY;
      if (lane < BK) {
        const int kj = k0 + lane;
        if (kj <= qi && qi < len) {
          float d = 0.f;
          const float* qs = Qs[wave * RPW + r];
#pragma unroll 8
          for (int x = 0; x < D; ++x) d = fmaf(qs[x], Ks[lane][x], d);
          sc = d;
        }
      }
      const float mt = group_max<64>(sc);
      float p = 0.f;
      if (mt > -INFINITY) {  // at least one key of this tile is visible to the row
        const float mn = fmaxf(m[r], mt);
        const float alpha = __builtin_amdgcn_exp2f(m[r] - mn);
        p = __builtin_amdgcn_exp2f(sc - mn);
        l[r] = l[r] * alpha + group_sum<64>(p);
        for (int j = 0; j < DPL; ++j) acc[r][j] *= alpha;
        m[r] = mn;
      }
      if (lane < BK) Ps[wave][r][lane] = p;
    }
    __syncthreads();
    for (int j = 0; j < BK; ++j) {
      float v[DPL];
      for (int x = 0; x < DPL; ++x) v[x] = Vs[j][lane + 64 * x];
      for (int r = 0; r < RPW; ++r) {
        const float p = Ps[wave][r][j];
        for (int x = 0; x < DPL; ++x) acc[r][x] = fmaf(p, v[x], acc[r][x]);
      }
    }
  }
  for (int r = 0; r < RPW; ++r) {
    const int qi = q0 + wave * RPW + r;
    if (qi < len) {
      T* o = (T*)a.out + (int64_t)(sm.tok0 + qi) * a.token_stride + (int64_t)h * a.head_stride;
      const float inv = 1.f / l[r];
      for (int x = 0; x < DPL; ++x) store_elem(o + lane + 64 * x, acc[r][x] * inv);
    }
  }
}

// Store this layer's rows into the caches: every V row; every K row, or in a lazy layer only
// the text rows, compacted; and the span rows of Q into the Q Cache when the next layer is lazy.
// Pure 16-byte copies.  grid = (row tiles, H, B).
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_cache_write_kernel(PrefillArgs a) {
  constexpr int EPL = ElemTraits<T>::kPer16;
  constexpr int CPR = D / EPL;
  constexpr int ROWS = 256 / CPR * 4;
  const int h = blockIdx.y, b = blockIdx.z;
  const SeqMeta sm = load_meta(a.lv, b, a.inherit_all);
  const int r0 = blockIdx.x * ROWS;
  if (r0 >= sm.len0) return;
  const RowIndex rb = row_index(a.lv, b, h, a.n_heads);
  const int ch = threadIdx.x % CPR;
  const int s = sm.vis_start, e = s + sm.vis_len;
  for (int pos = r0 + threadIdx.x / CPR; pos < min(r0 + ROWS, sm.len0); pos += 256 / CPR) {
    const int64_t in = (int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride + ch * EPL;
    const bool in_span = pos >= s && pos < e;
    *(uint4*)((T*)a.lv.v_own + rb.v(pos) * D + ch * EPL) = *(const uint4*)((const T*)a.v + in);
    if (!a.is_lazy) {
      *(uint4*)((T*)a.lv.k_own + rb.k(pos) * D + ch * EPL) = *(const uint4*)((const T*)a.k + in);
      if (a.write_q && in_span)
        *(uint4*)((T*)a.lv.q_cache + rb.q(pos - s) * D + ch * EPL) = *(const uint4*)((const T*)a.q + in);
    } else if (!in_span) {
      const int row = pos < s ? pos : pos - sm.vis_len;
      *(uint4*)((T*)a.lv.k_own + rb.k(row) * D + ch * EPL) = *(const uint4*)((const T*)a.k + in);
    }
  }
}

template <typename T, int D> hipError_t launch_cache_write_t(const PrefillArgs& a, hipStream_t stream) {
  constexpr int ROWS = 256 / (D / ElemTraits<T>::kPer16) * 4;
  dim3 grid((a.max_len + ROWS - 1) / ROWS, a.n_heads, a.batch);
  hipLaunchKernelGGL((prefill_cache_write_kernel<T, D>), grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

template <typename T, int D> hipError_t launch_prefill_simple_t(const PrefillArgs& a, hipStream_t stream, KernelTimer* timer) {
  hipError_t e = launch_cache_write_t<T, D>(a, stream);
  if (e != hipSuccess) return e;
  dim3 grid((a.max_len + 15) / 16, a.n_heads, a.batch);
  if (timer) timer->begin(stream);
  hipLaunchKernelGGL((prefill_simple_kernel<T, D>), grid, dim3(256), 0, stream, a);
  if (timer) timer->end(stream);
  return hipGetLastError();
}

hipError_t launch_prefill_mfma_bf16_d128(const PrefillArgs& a, hipStream_t stream, KernelTimer* timer);

hipError_t launch_prefill(const PrefillArgs& a, int dtype, hipStream_t stream, KernelTimer* timer) {
  if (dtype == 0) {
    if (a.head_dim == 64) return launch_prefill_simple_t<float, 64>(a, stream, timer);
    if (a.head_dim == 128) return launch_prefill_simple_t<float, 128>(a, stream, timer);
  } else {
    if (a.head_dim == 64) return launch_prefill_simple_t<bf16_t, 64>(a, stream, timer);
    if (a.head_dim == 128) return launch_prefill_mfma_bf16_d128(a, stream, timer);
  }
  return hipErrorInvalidValue;
}

}  // namespace qc
