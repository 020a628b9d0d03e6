// Token-wise pruning on top of Lazy Attention ("Compatibility" paragraph of the paper): choosing the
// visual tokens that survive, and dropping the other rows of a packed per-token tensor.
#include "qc_device.h"

namespace qc {

// One workgroup per sequence.  A visual token survives when fewer than `keep` tokens of its span rank
// ahead of it, where token j ranks ahead of token i if its score is higher, or equal with j < i.
// Scores are compared through an integer key that orders floats as their values do (-0 and +0 made
// equal first) and also gives NaNs a fixed place, so the ranks are a permutation of 0..V-1 whatever
// the input holds and exactly `keep` survivors are written.
//
// The key of rank keep-1 is found by a radix select over the key's four bytes, most significant
// first: a 256-bin histogram of the keys that match the bytes decided so far, then the bin in which
// the wanted rank falls.  Each wave counts into a histogram of its own (rows padded to 257 words so
// that equal bins of different waves sit in different LDS banks); the span's scores are re-read from
// memory in every pass (at most 128 KB: they stay in cache).  Work per sequence is O(V), whatever
// the scores hold.  What is left after the last byte is the threshold key T and the number of
// tokens with exactly that key that still fit; those are taken in position order (the tie rule).
// Survivors are written in position order: 1024 candidates per round, a ballot prefix within the
// round, running counts across rounds.
constexpr int kPruneThreads = 1024;
constexpr int kPruneWaves = kPruneThreads / 64;
constexpr int kHistStride = 257;

__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

__global__ __launch_bounds__(kPruneThreads) void prune_select_kernel(const float* __restrict__ scores, int64_t stride,
                                                                    int first, PruneChunk c,
                                                                    int32_t* __restrict__ row_map) {
  const int i = blockIdx.x, t = threadIdx.x;
  const int tok0 = c.tok0[i], len = c.len[i], s = c.vis_start[i], V = c.vis_len[i], keep = c.keep[i];
  const float* sc = scores + (int64_t)(first + i) * stride + s;
  int32_t* out = row_map + c.out0[i];

  for (int p = t; p < s; p += kPruneThreads) out[p] = tok0 + p;
  for (int p = s + V + t; p < len; p += kPruneThreads) out[p - V + keep] = tok0 + p;
  if (keep == 0) return;   // uniform over the workgroup

  __shared__ uint32_t hist[kPruneWaves * kHistStride];
  __shared__ uint32_t total[4];      // keys per group of 64 bins
  __shared__ uint32_t chosen[2];     // selected bin, survivors still to be found inside it
  __shared__ int wave_count[2][kPruneWaves];
  const int lane = t & 63, wave = t >> 6;

  uint32_t prefix = 0, prefix_mask = 0;   // bytes decided so far (the same in every thread)
  uint32_t remaining = (uint32_t)keep;    // survivors still to be found among the keys matching them
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int j = t; j < kPruneWaves * kHistStride; j += kPruneThreads) hist[j] = 0;
    __syncthreads();
    for (int j = t; j < V; j += kPruneThreads) {
      const uint32_t k = order_key(sc[j]);
      if ((k & prefix_mask) == prefix) atomicAdd(&hist[wave * kHistStride + ((k >> shift) & 255u)], 1u);
    }
    __syncthreads();
    // bins 0..255 sit in threads 0..255 (waves 0..3): suffix sums inside each wave by shuffles, then
    // across the four waves through LDS
    uint32_t n = 0, from_here = 0;   // keys in this bin; keys in this bin and the higher bins of the same wave
    if (t < 256) {
#pragma unroll
      for (int w = 0; w < kPruneWaves; ++w) n += hist[w * kHistStride + t];
      from_here = n;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_down(from_here, d);
        if (lane + d < 64) from_here += up;
      }
      if (lane == 0) total[wave] = from_here;
    }
    __syncthreads();
    if (t < 256) {
      uint32_t above = from_here - n;   // matching keys in higher bins
      for (int w = wave + 1; w < 4; ++w) above += total[w];
      if (above < remaining && remaining <= above + n) {   // true for exactly one bin
        chosen[0] = (uint32_t)t;
        chosen[1] = remaining - above;
      }
    }
    __syncthreads();
    prefix |= chosen[0] << shift;
    prefix_mask |= 255u << shift;
    remaining = chosen[1];
    __syncthreads();   // chosen is rewritten in the next pass
  }
  const uint32_t T = prefix;              // key of rank keep-1
  const int need_eq = (int)remaining;     // tokens with key T that survive: the first need_eq in position order

  int base_kept = 0, base_eq = 0;         // survivors / keys equal to T in earlier rounds (the same in every thread)
  for (int c0 = 0; c0 < V; c0 += kPruneThreads) {
    const int cand = c0 + t;
    const bool live = cand < V;
    const uint32_t my = live ? order_key(sc[cand]) : 0u;
    const bool eq = live && my == T;
    const unsigned long long eq_ballot = __ballot(eq);
    if (lane == 0) wave_count[0][wave] = __popcll(eq_ballot);
    __syncthreads();
    int eq_before = 0, eq_total = 0;
    for (int w = 0; w < kPruneWaves; ++w) {
      const int n = wave_count[0][w];
      eq_before += w < wave ? n : 0;
      eq_total += n;
    }
    const int eq_rank = base_eq + eq_before + __popcll(eq_ballot & ((1ull << lane) - 1ull));
    const bool kept = live && (my > T || (eq && eq_rank < need_eq));
    const unsigned long long ballot = __ballot(kept);
    if (lane == 0) wave_count[1][wave] = __popcll(ballot);
    __syncthreads();
    int wave_base = 0, kept_total = 0;
    for (int w = 0; w < kPruneWaves; ++w) {
      const int n = wave_count[1][w];
      wave_base += w < wave ? n : 0;
      kept_total += n;
    }
    const int slot = base_kept + wave_base + __popcll(ballot & ((1ull << lane) - 1ull));
    if (kept && slot < keep) out[s + slot] = tok0 + s + cand;
    base_kept += kept_total;
    base_eq += eq_total;
    __syncthreads();   // wave_count is rewritten in the next round
  }
}

hipError_t launch_prune_select(const float* scores, int64_t stride, int first, int count, const PruneChunk& c,
                               int32_t* row_map, hipStream_t stream) {
  hipLaunchKernelGGL(prune_select_kernel, dim3(count), dim3(kPruneThreads), 0, stream, scores, stride, first, c,
                     row_map);
  return hipGetLastError();
}

// dst row r = src row row_map[r], 16 bytes per lane, consecutive lanes on consecutive pieces of a row.
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ src, int64_t src_stride,
                                                          const int32_t* __restrict__ row_map, int64_t n_rows,
                                                          int32_t pieces, char* __restrict__ dst, int64_t dst_stride) {
  const int64_t total = n_rows * pieces;
  const int64_t step = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += step) {
    const int64_t r = i / pieces;
    const int64_t p = i - r * pieces;
    const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)row_map[r] * src_stride + p * 16);
    *reinterpret_cast<uint4*>(dst + r * dst_stride + p * 16) = v;
  }
}

hipError_t launch_gather_rows(const void* src, int64_t src_stride, const int32_t* row_map, int64_t n_rows,
                              int64_t row_bytes, void* dst, int64_t dst_stride, hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  const int64_t total = n_rows * (row_bytes / 16);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const char*)src, src_stride,
                     row_map, n_rows, (int32_t)(row_bytes / 16), (char*)dst, dst_stride);
  return hipGetLastError();
}

}  // namespace qc
