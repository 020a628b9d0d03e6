// Token-wise pruning on top of Lazy Attention ("Compatibility" paragraph of the paper): choosing the
// visual tokens that survive, and dropping the other rows of a packed per-token tensor.
#include "qc_device.h"

namespace qc {

// One workgroup per sequence.  A visual token survives when fewer than `keep` tokens of its span rank
// ahead of it, where token j ranks ahead of token i if its score is higher, or equal with j < i: every
// token's rank is a plain count, so the result does not depend on any ordering of the work.
// Scores are compared through an integer key that orders floats as their values do (-0 and +0 made
// equal first) and also gives NaNs a fixed place: the ranks are then a permutation of 0..V-1 whatever
// the input holds, so exactly `keep` survivors are written.
// Candidates are taken 1024 at a time; the span's scores pass through LDS in tiles that every lane
// reads at the same address (broadcast).  Survivors are written in position order: within a round by
// a ballot prefix, across rounds by a running count.
constexpr int kPruneThreads = 1024;
constexpr int kPruneTile = 4096;

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

  __shared__ uint4 tile[kPruneTile / 4];
  __shared__ int wave_count[kPruneThreads / 64];
  uint32_t* tile_u = reinterpret_cast<uint32_t*>(tile);
  const int lane = t & 63, wave = t >> 6;
  int base = 0;   // survivors of earlier rounds (the same in every lane)
  for (int c0 = 0; c0 < V; c0 += kPruneThreads) {
    const int cand = c0 + t;
    const bool live = cand < V;
    const uint32_t my = live ? order_key(sc[cand]) : 0u;
    int rank = 0;
    for (int j0 = 0; j0 < V; j0 += kPruneTile) {
      const int n = V - j0 < kPruneTile ? V - j0 : kPruneTile;
      const int n4 = (n + 3) & ~3;
      __syncthreads();
      // entries past the span's end get the lowest key; their index is beyond every candidate's
      for (int j = t; j < n4; j += kPruneThreads) tile_u[j] = j < n ? order_key(sc[j0 + j]) : 0u;
      __syncthreads();
      for (int j = 0; j < n4; j += 4) {
        const uint4 x = tile[j >> 2];
        const int jj = j0 + j;
        rank += (x.x > my) || (x.x == my && jj < cand);
        rank += (x.y > my) || (x.y == my && jj + 1 < cand);
        rank += (x.z > my) || (x.z == my && jj + 2 < cand);
        rank += (x.w > my) || (x.w == my && jj + 3 < cand);
      }
    }
    const bool kept = live && rank < keep;
    const unsigned long long ballot = __ballot(kept);
    if (lane == 0) wave_count[wave] = __popcll(ballot);
    __syncthreads();
    int wave_base = 0, total = 0;
    for (int w = 0; w < kPruneThreads / 64; ++w) {
      const int n = wave_count[w];
      wave_base += w < wave ? n : 0;
      total += n;
    }
    const int slot = base + wave_base + __popcll(ballot & ((1ull << lane) - 1ull));
    if (kept && slot < keep) out[s + slot] = tok0 + s + cand;
    base += total;
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
