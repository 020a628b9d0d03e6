// Lazy-block selection statistics (paper Eq. 3): the head-averaged last row of a layer's attention
// matrix, and the Jensen-Shannon similarity of two layers' rows averaged over samples.
//
// All three passes are bound by HBM reads of a few megabytes and run once per model, offline.
//   last_row_scores_kernel : one workgroup per (sequence, head): scaled scores q.k of the last
//                            prompt token against every cached key, plus the row's (max, sum).
//   last_row_probs_kernel  : one thread per position: mean over heads of exp2(s - max) / sum.
//   js_kernel / mean_kernel: one workgroup per sample, fixed-order tree reductions (bitwise
//                            reproducible), natural logarithms (JS <= ln 2), 0 log 0 = 0.
#include "qc_device.h"

namespace qc {

template <typename T, int D>
__global__ __launch_bounds__(256) void last_row_scores_kernel(SelectArgs a) {
  constexpr int EPL = ElemTraits<T>::kPer16;
  constexpr int LPR = D / EPL;
  constexpr int GPW = 64 / LPR;
  constexpr int GROUPS = 4 * GPW;
  constexpr int ROWB = D * (int)sizeof(T);
  const int h = blockIdx.x, b = blockIdx.y;
  const int len = a.lv.meta[META_LEN0 * a.lv.max_batch + b] + a.generated;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane % LPR, gid = wave * GPW + lane / LPR;
  const int64_t bh = (int64_t)b * a.n_heads + h;
  const RowIndex ri = row_index(a.lv, b, h, a.n_heads);
  const char* krows = a.lv.k_own + li * 16;
  // score rows: score_stride floats each, or (per-sequence capacities, pages) laid out like the layer's rows
  const bool like_rows = (a.lv.flags & (LV_RAGGED | LV_PAGED)) != 0;
  float* srow = a.scores + (like_rows ? 0 : bh * a.score_stride);

  float qf[EPL];
  {
    const uint4 raw = *(const uint4*)((const char*)a.q_last + bh * ROWB + li * 16);
    unpack16(raw, qf, (T*)nullptr);
    const float c = a.scale * kLog2e;
#pragma unroll
    for (int i = 0; i < EPL; ++i) qf[i] *= c;
  }
  float m = -INFINITY, l = 0.f;
  constexpr int U = 8;   // rows in flight per group: the kernel streams every K row of the layer once
  // The scores are not stored from inside the row loop (loads and stores share one counter: a store in
  // flight would hold up the wait for the next rows); kStage of them are collected in LDS and written out
  // together.
  constexpr int kStage = 2048;
  static_assert(kStage % (GROUPS * U) == 0, "a block is a whole number of iterations");
  __shared__ float s_stage[kStage];
  for (int block0 = 0; block0 < len; block0 += kStage) {
  const int block_end = min(block0 + kStage, len);
  for (int p0 = block0 + gid; p0 < block_end; p0 += GROUPS * U) {
    uint4 raw[U];
    int64_t row[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pos = min(p0 + u * GROUPS, len - 1);   // rows past the end repeat the last one and are dropped below
      row[u] = ri.k(pos);
      raw[u] = stream_load16(krows + row[u] * ROWB);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pos = p0 + u * GROUPS;
      float kf[EPL];
      unpack16(raw[u], kf, (T*)nullptr);
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) d = fmaf(qf[i], kf[i], d);
      d = group_sum<LPR>(d);
      if (pos < len) {
        if (li == 0) s_stage[pos - block0] = d;
        const float mn = fmaxf(m, d);
        l = l * __builtin_amdgcn_exp2f(m - mn) + __builtin_amdgcn_exp2f(d - mn);
        m = mn;
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < block_end - block0; i += 256) srow[like_rows ? ri.k(block0 + i) : (int64_t)(block0 + i)] = s_stage[i];
  if (block_end < len) __syncthreads();   // the next block writes the stage again
  }
  __shared__ float s_m[GROUPS], s_l[GROUPS];
  if (li == 0) {
    s_m[gid] = m;
    s_l[gid] = l;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = -INFINITY;
    for (int g = 0; g < GROUPS; ++g) M = fmaxf(M, s_m[g]);
    float L = 0.f;
    for (int g = 0; g < GROUPS; ++g) L = fmaf(__builtin_amdgcn_exp2f(s_m[g] - M), s_l[g], L);  // exp2(-inf) = 0 for idle groups
    a.row_stats[bh * 2] = M;
    a.row_stats[bh * 2 + 1] = L;
  }
}

__global__ __launch_bounds__(256) void last_row_probs_kernel(SelectArgs a) {
  const int b = blockIdx.y;
  const int pos = blockIdx.x * 256 + threadIdx.x;
  const int len = a.lv.meta[META_LEN0 * a.lv.max_batch + b] + a.generated;
  if (pos >= len) return;
  float acc = 0.f;
  for (int h = 0; h < a.n_heads; ++h) {
    const int64_t bh = (int64_t)b * a.n_heads + h;
    const bool like_rows = (a.lv.flags & (LV_RAGGED | LV_PAGED)) != 0;
    const float s = a.scores[like_rows ? row_index(a.lv, b, h, a.n_heads).k(pos) : bh * a.score_stride + pos];
    acc += __builtin_amdgcn_exp2f(s - a.row_stats[bh * 2]) / a.row_stats[bh * 2 + 1];
  }
  a.probs[(int64_t)b * a.probs_stride + pos] = acc / (float)a.n_heads;
}

// Sum over the 256 threads of a workgroup in a fixed order; every thread gets the total.
__device__ __forceinline__ float block_sum_256(float x, float* lds) {
  lds[threadIdx.x] = x;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) lds[threadIdx.x] += lds[threadIdx.x + s];
    __syncthreads();
  }
  const float r = lds[0];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void js_kernel(const float* pm, const float* pn, int64_t stride, int first, JsChunk c, float* js_out) {
  __shared__ float lds[256];
  const int i = blockIdx.x;
  const int len = c.len[i];
  const float* p = pm + (int64_t)(first + i) * stride;
  const float* q = pn + (int64_t)(first + i) * stride;
  float acc = 0.f;
  for (int pos = threadIdx.x; pos < len; pos += 256) {
    const float x = p[pos], y = q[pos];
    const float lm = __log2f(0.5f * (x + y));
    if (x > 0.f) acc += x * (__log2f(x) - lm);
    if (y > 0.f) acc += y * (__log2f(y) - lm);
  }
  const float tot = block_sum_256(acc, lds);
  if (threadIdx.x == 0) js_out[first + i] = 0.5f * 0.6931471805599453f * tot;   // base-2 logarithms above: to nats
}

__global__ __launch_bounds__(256) void mean_kernel(const float* x, int n, float* out) {
  __shared__ float lds[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) acc += x[i];
  const float tot = block_sum_256(acc, lds);
  if (threadIdx.x == 0) *out = tot / (float)n;
}

hipError_t launch_last_row_attention(const SelectArgs& a, int dtype, int max_len, hipStream_t stream) {
  dim3 g1(a.n_heads, a.batch);
  if (dtype == 0) {
    if (a.head_dim == 64) hipLaunchKernelGGL((last_row_scores_kernel<float, 64>), g1, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((last_row_scores_kernel<float, 128>), g1, dim3(256), 0, stream, a);
  } else {
    if (a.head_dim == 64) hipLaunchKernelGGL((last_row_scores_kernel<bf16_t, 64>), g1, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((last_row_scores_kernel<bf16_t, 128>), g1, dim3(256), 0, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(last_row_probs_kernel, dim3((max_len + 255) / 256, a.batch), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_js(const float* pm, const float* pn, int64_t stride, int first, int count, const JsChunk& c,
                     float* js_out, hipStream_t stream) {
  hipLaunchKernelGGL(js_kernel, dim3(count), dim3(256), 0, stream, pm, pn, stride, first, c, js_out);
  return hipGetLastError();
}

hipError_t launch_mean(const float* x, int n, float* out, hipStream_t stream) {
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, stream, x, n, out);
  return hipGetLastError();
}

}  // namespace qc
