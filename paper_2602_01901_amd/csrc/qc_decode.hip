// Decode attention for one generated token per sequence (paper Eq. 2; Eq. 8 in a lazy layer).
//
// The kernel is bound by HBM bandwidth: every cached K and V row of a (sequence, head) pair is
// streamed exactly once.  The key axis is cut into chunks; one workgroup takes one chunk of one
// (sequence, head).  A row (head_dim elements) is covered by a group of 16-byte lanes, so a wave
// reads whole consecutive rows with one load instruction per lane.  Each group keeps its own
// running softmax (max, sum, weighted V) in fp32; groups are merged through LDS at the end of the
// chunk and chunks are merged by a second, tiny kernel in fixed order (bitwise reproducible).
//
// Lazy layers differ only in where a key row comes from: positions before the visual span and
// after it are the layer's own (compacted) rows, positions inside it are rows of the block's
// first layer.  The new token's k/v are taken from the call's inputs, appended to the caches by
// the one group that owns that position.
//
// Global Lazy Attention (Eq. 6): a lazy layer attends with the query and the keys of its block's
// first layer, so its scores q.k are the ones that layer computed earlier in the same step.  The
// first layer of a block therefore stores its scaled scores (one float per position) next to the
// split partials and its query at row `len` of the Q Cache; a lazy layer (SHARED instantiation)
// reads those scores instead of any key row: it streams V only, half the bytes, and gets
// bit-identical scores.  It appends its v row only.
#include <atomic>

#include "qc_device.h"

#ifndef QC_U_SHARED
#define QC_U_SHARED 8
#endif
#ifndef QC_U_PLAIN
#define QC_U_PLAIN 4
#endif

namespace qc {

// ---- scratch memory for callers that cannot allocate ----------------------------------------------
// The split partials (and, under Global Lazy Attention, the score rows) of a decode call normally
// live in a workspace the caller allocates.  For callers that cannot allocate, the same kernels are
// handed this array instead.  Every GPU the library runs on holds its own copy at its own address:
// in host code the array's name is only a stand-in, so the device address is looked up once per
// device and that pointer is what reaches the kernels.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t decode_static_scratch(void** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> per_device[kMaxDevices];
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = per_device[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // address of the current device's copy
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

// Per-sequence integers: from the kernel arguments for small batches (INLINE), else from the arena's
// meta region.  Two instantiations rather than a run-time choice: with a choice the compiler selects
// between the two addresses and issues one per-lane load, a full memory round trip ahead of
// everything else; kept apart, both become scalar loads.
template <bool INLINE> __device__ __forceinline__ SeqMeta decode_meta(const DecodeArgs& a, int b) {
  if constexpr (INLINE) {
    SeqMeta m;
    m.tok0 = 0;
    m.len0 = a.len0_inline[b];
    m.vis_start = a.vis_start_inline[b];
    m.vis_len = a.vis_len_inline[b];
    return m;
  } else {
    return load_meta(a.lv, b);
  }
}
// Decode steps completed before this one: by value, or (launches recorded in a graph that is replayed
// step after step) from the counter in device memory that the replayed graph itself advances.
__device__ __forceinline__ int decode_generated(const DecodeArgs& a) {
  if (a.generated_dev) return uniform_load(a.generated_dev);
  return a.generated;
}

// MODE 0: ordinary and Visual Lazy Attention layers.  MODE 1: first layer of a Global Lazy Attention
// block (also stores its scores and its query).  MODE 2: lazy layer under Global Lazy Attention
// (reuses the stored scores, streams V only).
// PAGED: rows live on pages; the workgroup stages the sequence's two page lists (positions, and the
// pool its own K rows live in) in LDS before it streams.
template <typename T, int D, int MODE, bool INLINE, bool PAGED>
__device__ __forceinline__ void decode_split_body(const DecodeArgs& a, const DecodeGlaArgs& g) {
  constexpr bool SHARED = MODE == 2, STORE = MODE == 1;
  constexpr int EPL = ElemTraits<T>::kPer16;  // elements per lane (16 bytes)
  constexpr int LPR = D / EPL;                // lanes per row
  constexpr int GPW = 64 / LPR;               // row groups per wave
  constexpr int GROUPS = 4 * GPW;             // row groups per workgroup
  constexpr int U = SHARED ? QC_U_SHARED : QC_U_PLAIN;   // rows in flight per group
  constexpr int ROWB = D * (int)sizeof(T);

  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const SeqMeta sm = decode_meta<INLINE>(a, b);
  const int len = sm.len0 + decode_generated(a);  // position of the new token
  const int kbeg = chunk * a.chunk_keys;
  if (kbeg > len) return;
  const int kend = min(kbeg + a.chunk_keys, len + 1);
  const int s = sm.vis_start, e = sm.vis_start + sm.vis_len;
  const bool lazy = a.is_lazy != 0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane % LPR, gid = wave * GPW + lane / LPR;
  const int64_t bh = (int64_t)b * a.n_heads + h;

  __shared__ int32_t s_pg_seq[PAGED ? kMaxPagesPerSeq : 1], s_pg_k[PAGED ? kMaxPagesPerSeq : 1];
  RowBase rb = {0, 0, 0, 0};
  if constexpr (PAGED) {
    const int n_seq = (len >> 6) + 1;                                   // pages holding positions 0 .. len
    const int n_k = (((lazy && !SHARED) ? len - sm.vis_len : len) >> 6) + 1;   // pages holding its own K rows
    for (int i = threadIdx.x; i < n_seq; i += 256) s_pg_seq[i] = a.lv.pt_seq[(int64_t)b * a.lv.pt_seq_stride + i];
    if (!SHARED)
      for (int i = threadIdx.x; i < n_k; i += 256) s_pg_k[i] = a.lv.pt_k[(int64_t)b * a.lv.pt_k_stride + i];
    __syncthreads();
  } else {
    rb = row_bases(a.lv, b, h, a.n_heads);
  }
  // addresses of this lane's 16 bytes of a row: own K row r, the first layer's K row of a position, own V row
  char* kown = a.lv.k_own + rb.k * ROWB + li * 16;
  const char* kanc = lazy ? a.lv.k_anchor + rb.anchor * ROWB + li * 16 : nullptr;
  char* vown = a.lv.v_own + rb.v * ROWB + li * 16;
  auto k_own_at = [&](int r) -> char* {
    if constexpr (PAGED) return kown + paged_row(s_pg_k, r, h, a.n_heads) * ROWB;
    else return kown + (int64_t)r * ROWB;
  };
  auto k_anchor_at = [&](int pos) -> const char* {
    if constexpr (PAGED) return kanc + paged_row(s_pg_seq, pos, h, a.n_heads) * ROWB;
    else return kanc + (int64_t)pos * ROWB;
  };
  auto v_own_at = [&](int pos) -> char* {
    if constexpr (PAGED) return vown + paged_row(s_pg_seq, pos, h, a.n_heads) * ROWB;
    else return vown + (int64_t)pos * ROWB;
  };
  const char* knew = (const char*)a.k + bh * ROWB + li * 16;
  const char* vnew = (const char*)a.v + bh * ROWB + li * 16;

  // one score per position: rows of score_stride floats, or (per-sequence capacities) laid out like the V rows
  float* score_row = (SHARED || STORE) ? g.scores + ((a.lv.flags & LV_RAGGED) ? rb.v : bh * g.score_stride) : nullptr;
  // where the score of a position is kept: paged batches lay the scores out like the V rows
  auto score_at = [&](int pos) -> float* {
    if constexpr (PAGED) return g.scores + paged_row(s_pg_seq, pos, h, a.n_heads);
    else return score_row + pos;
  };

  float qf[EPL];
  uint4 qraw = make_uint4(0, 0, 0, 0);
  if (!SHARED) {
    qraw = *(const uint4*)((const char*)a.q + bh * ROWB + li * 16);
    unpack16(qraw, qf, (T*)nullptr);
    const float c = a.scale * kLog2e;
#pragma unroll
    for (int i = 0; i < EPL; ++i) qf[i] *= c;
  }

  float m = -INFINITY, l = 0.f;
  float acc[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

  // A first layer of a Global Lazy Attention block keeps its scores.  They are not stored from inside the
  // row loop: loads and stores share one counter, so a store in flight would hold up the wait for the
  // next iteration's rows (measured: 80.6 instead of 76.2 us per launch).  The scores of kStage positions
  // are collected in LDS and written out together.
  constexpr int kStage = 2048;
  __shared__ float s_stage[STORE ? kStage : 1];
  const int block_step = STORE ? kStage : kend - kbeg;   // other modes: one block
  for (int block0 = kbeg; block0 < kend; block0 += block_step) {
  const int block_end = min(block0 + block_step, kend);
  for (int r0 = block0 + gid; r0 < block_end; r0 += GROUPS * U) {
    uint4 kr[U], vr[U];
    float sc[U];
    float mine = -INFINITY;
    if (SHARED) {  // lane li < U of a group fetches the score of the group's row u = li; broadcast below
      const int pos = r0 + li * GROUPS;
      if (li < U && pos < kend) mine = *score_at(pos);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pos = r0 + u * GROUPS;
      kr[u] = make_uint4(0, 0, 0, 0);
      vr[u] = make_uint4(0, 0, 0, 0);
      sc[u] = -INFINITY;
      if (pos < kend) {
        if (pos == len) {  // the token being decoded: read the inputs, append to the caches
          vr[u] = *(const uint4*)vnew;
          *(uint4*)v_own_at(len) = vr[u];
          if (!SHARED) {
            kr[u] = *(const uint4*)knew;
            const int krow = lazy ? len - sm.vis_len : len;
            *(uint4*)k_own_at(krow) = kr[u];
            if (STORE) {   // Global Lazy Attention: the Q Cache row of a position lives like its V row
              if constexpr (PAGED) *(uint4*)(a.lv.q_cache + paged_row(s_pg_seq, len, h, a.n_heads) * ROWB + li * 16) = qraw;
              else *(uint4*)(a.lv.q_cache + (rb.q + len) * ROWB + li * 16) = qraw;
            }
          }
        } else {
          if (!SHARED) {
            const char* kp;
            if (lazy && pos >= s) kp = pos < e ? k_anchor_at(pos) : k_own_at(pos - sm.vis_len);
            else kp = k_own_at(pos);
            kr[u] = stream_load16(kp);
          }
          vr[u] = stream_load16(v_own_at(pos));
        }
      }
    }
    float mt = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (SHARED) {
        sc[u] = group_broadcast<LPR>(mine, u);
      } else {
        float kf[EPL];
        unpack16(kr[u], kf, (T*)nullptr);
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) d = fmaf(qf[i], kf[i], d);
        d = group_sum<LPR>(d);
        const int pos = r0 + u * GROUPS;
        if (pos < kend) {
          sc[u] = d;
          if (STORE && li == 0) s_stage[pos - block0] = d;
        }
      }
      mt = fmaxf(mt, sc[u]);
    }
    const float mn = fmaxf(m, mt);  // finite: the first row of every iteration is valid
    const float alpha = __builtin_amdgcn_exp2f(m - mn);
    l *= alpha;
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = __builtin_amdgcn_exp2f(sc[u] - mn);
      l += p;
      float vf[EPL];
      unpack16(vr[u], vf, (T*)nullptr);
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc[i] = fmaf(p, vf[i], acc[i]);
    }
    m = mn;
  }
  if (STORE) {
    __syncthreads();
    for (int i = threadIdx.x; i < block_end - block0; i += 256) *score_at(block0 + i) = s_stage[i];
    if (block_end < kend) __syncthreads();   // the next block writes the stage again
  }
  }

  __shared__ float s_acc[GROUPS][D];
  __shared__ float s_m[GROUPS], s_l[GROUPS];
#pragma unroll
  for (int i = 0; i < EPL; ++i) s_acc[gid][li * EPL + i] = acc[i];
  if (li == 0) {
    s_m[gid] = m;
    s_l[gid] = l;
  }
  __syncthreads();
  const int d = threadIdx.x;
  if (d < D) {
    float M = -INFINITY;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) M = fmaxf(M, s_m[g]);
    float o = 0.f, lsum = 0.f;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
      const float w = __builtin_amdgcn_exp2f(s_m[g] - M);  // 0 for groups that saw no row
      o = fmaf(w, s_acc[g][d], o);
      lsum = fmaf(w, s_l[g], lsum);
    }
    if (a.max_chunks == 1) {
      store_elem((T*)a.out + bh * D + d, o / lsum);
    } else {
      float* w = a.workspace + (bh * a.max_chunks + chunk) * (D + 2);
      w[d] = o;
      if (d == 0) {
        w[D] = M;
        w[D + 1] = lsum;
      }
    }
  }
}

template <typename T, int D, bool INLINE, bool PAGED>
__global__ __launch_bounds__(256) void decode_split_kernel(DecodeArgs a) {
  decode_split_body<T, D, 0, INLINE, PAGED>(a, DecodeGlaArgs{nullptr, 0, 0});
}
template <typename T, int D, int MODE, bool INLINE, bool PAGED>
__global__ __launch_bounds__(256) void decode_split_gla_kernel(DecodeArgs a, DecodeGlaArgs g) {
  decode_split_body<T, D, MODE, INLINE, PAGED>(a, g);
}

// Merge the chunk partials of one (sequence, head) in chunk order.  Partials are loaded in batches
// of 16 chunks (all loads of a batch are independent, so their latencies overlap); within a batch
// the usual running (max, sum) update is applied chunk by chunk in a fixed order, so results are
// bitwise reproducible.
template <typename T, int D, bool INLINE>
__global__ __launch_bounds__(D) void decode_merge_kernel(DecodeArgs a) {
  const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int len = decode_meta<INLINE>(a, b).len0 + decode_generated(a);
  if (len < 0) return;   // a free slot of the batch: nothing was computed, nothing is written
  const int n = (len + a.chunk_keys) / a.chunk_keys;  // ceil((len + 1) / chunk_keys)
  const int64_t bh = (int64_t)b * a.n_heads + h;
  const float* w = a.workspace + bh * a.max_chunks * (D + 2);
  constexpr int G = 16;
  float M = -INFINITY, o = 0.f, l = 0.f;
  for (int c0 = 0; c0 < n; c0 += G) {
    float mv[G], lv[G], ov[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const bool ok = c0 + g < n;
      const float* p = w + (ok ? c0 + g : 0) * (D + 2);
      mv[g] = ok ? p[D] : -INFINITY;
      lv[g] = p[D + 1];
      ov[g] = p[d];
    }
    float Mb = M;
#pragma unroll
    for (int g = 0; g < G; ++g) Mb = fmaxf(Mb, mv[g]);
    const float keep = __builtin_amdgcn_exp2f(M - Mb);  // 0 on the first batch (M = -inf)
    o *= keep;
    l *= keep;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float f = __builtin_amdgcn_exp2f(mv[g] - Mb);  // 0 for slots past the last chunk
      o = fmaf(f, ov[g], o);
      l = fmaf(f, lv[g], l);
    }
    M = Mb;
  }
  store_elem((T*)a.out + bh * D + d, o / l);
}

template <typename T, int D, bool INLINE, bool PAGED>
static void launch_split(const DecodeArgs& a, const DecodeGlaArgs& g, hipStream_t stream) {
  dim3 grid(a.max_chunks, a.n_heads, a.batch);
  if (g.mode == 2) hipLaunchKernelGGL((decode_split_gla_kernel<T, D, 2, INLINE, PAGED>), grid, dim3(256), 0, stream, a, g);
  else if (g.mode == 1) hipLaunchKernelGGL((decode_split_gla_kernel<T, D, 1, INLINE, PAGED>), grid, dim3(256), 0, stream, a, g);
  else hipLaunchKernelGGL((decode_split_kernel<T, D, INLINE, PAGED>), grid, dim3(256), 0, stream, a);
}

template <typename T, int D, bool INLINE>
static hipError_t launch_decode_t(const DecodeArgs& a, const DecodeGlaArgs& g, hipStream_t stream, KernelTimer* timer) {
  const bool paged = (a.lv.flags & LV_PAGED) != 0;
  if (paged && INLINE) return hipErrorInvalidValue;   // paged batches read their per-sequence integers from memory
  if (timer) timer->begin(stream);
  if constexpr (!INLINE) {
    if (paged) launch_split<T, D, false, true>(a, g, stream);
    else launch_split<T, D, false, false>(a, g, stream);
  } else {
    launch_split<T, D, true, false>(a, g, stream);
  }
  if (timer) timer->end(stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.max_chunks == 1) return e;
  hipLaunchKernelGGL((decode_merge_kernel<T, D, INLINE>), dim3(a.n_heads, a.batch), dim3(D), 0, stream, a);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_decode_m(const DecodeArgs& a, const DecodeGlaArgs& g, hipStream_t stream, KernelTimer* timer) {
  return a.inline_meta ? launch_decode_t<T, D, true>(a, g, stream, timer) : launch_decode_t<T, D, false>(a, g, stream, timer);
}

hipError_t launch_decode(const DecodeArgs& a, const DecodeGlaArgs& g, int dtype, hipStream_t stream, KernelTimer* timer) {
  if (dtype == 0) {
    if (a.head_dim == 64) return launch_decode_m<float, 64>(a, g, stream, timer);
    if (a.head_dim == 128) return launch_decode_m<float, 128>(a, g, stream, timer);
  } else {
    if (a.head_dim == 64) return launch_decode_m<bf16_t, 64>(a, g, stream, timer);
    if (a.head_dim == 128) return launch_decode_m<bf16_t, 128>(a, g, stream, timer);
  }
  return hipErrorInvalidValue;
}

}  // namespace qc
