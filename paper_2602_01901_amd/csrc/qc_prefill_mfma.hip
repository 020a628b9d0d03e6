// Prefill attention on the matrix cores: bf16 inputs, head_dim 128 (paper Eq. 1; Eq. 7 in a lazy
// layer).  Flash-style: the score matrix is never materialised; softmax runs online in fp32.
//
// Work split.  One workgroup (4 waves) takes BM = 128 consecutive query rows of one (sequence,
// head); each wave owns 32 of them for the whole kernel.  Keys/values are visited in tiles of
// BN = 64 rows, staged in LDS (double buffered: the global loads of tile t+1 are in flight while
// tile t is multiplied).
//
// Operand layout.  Scores are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the A operand is a K fragment read from LDS with one 16-byte read per lane, the B operand is a
// Q fragment that stays in registers.  In the accumulator a lane then holds, for ONE query
// (column = lane % 32), runs of 4 consecutive keys - which is, after conversion to bf16, already
// the B operand layout of the second product O^T = V^T P^T once the 16 contraction slots of a
// k-step are assigned to keys as {4 keys, 4 keys} per lane half.  The matching V^T fragment
// (A operand: 4 consecutive keys for one output column) is fetched from the row-major V tile in
// LDS with the transposing read ds_read_b64_tr_b16.  Nothing is shuffled between the products.
//
// Softmax.  All 64 scores a query has in a tile live in two lanes (l and l ^ 32): the row maximum
// costs one cross-half exchange per tile; row sums stay per lane until the end.  The running
// maximum is only moved when it grows by more than 2^8 (the result is independent of the
// reference point; this keeps the accumulator rescale off the common path).
//
// Lazy layers.  Query rows inside the visual span are read from the Q Cache and key rows inside
// it from the anchor layer's K cache; row addresses are selected per row while loading, the rest
// of the kernel is unchanged.  Cache writes are done by the shared cache-writer kernel.
#include "qc_device.h"

namespace qc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

namespace pf {
constexpr int BM = 128, BN = 64, D = 128;
constexpr int KSTRIDE = 272;  // bytes per K row in LDS: 256 + 16, 16-byte reads of 16 rows hit 64 distinct banks
constexpr int VSTRIDE = 320;  // bytes per V row in LDS: 256 + 64, the 4-row transposing reads hit distinct banks
constexpr int KTILE = BN * KSTRIDE;
constexpr int VTILE = BN * VSTRIDE;
constexpr int LDS_BYTES = 2 * (KTILE + VTILE);
constexpr float kRescaleThreshold = 8.0f;  // log2 units
}  // namespace pf

hipError_t launch_cache_write_bf16_d128(const PrefillArgs& a, hipStream_t stream);

__device__ __forceinline__ const char* pf_q_row(const PrefillArgs& a, const SeqMeta& sm, int64_t bh, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len)
    return a.lv.q_cache + (bh * a.lv.cap_q + (pos - sm.vis_start)) * (pf::D * 2);
  return (const char*)a.q + ((int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride) * 2;
}
__device__ __forceinline__ const char* pf_k_row(const PrefillArgs& a, const SeqMeta& sm, int64_t bh, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len)
    return a.lv.k_anchor + (bh * a.lv.cap_k_anchor + pos) * (pf::D * 2);
  return (const char*)a.k + ((int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride) * 2;
}

__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(PrefillArgs a, int n_qt, int xcd_map) {
  using namespace pf;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // ---- which tile: heavy (late) query tiles first; heads grouped per XCD so K/V stay in its L2
  int qt, bhi;
  {
    const int id = blockIdx.x;
    if (xcd_map) {
      const int xcd = id & 7, slot = id >> 3;
      bhi = (slot / n_qt) * 8 + xcd;
      qt = n_qt - 1 - slot % n_qt;
    } else {
      const int nbh = a.batch * a.n_heads;
      bhi = id % nbh;
      qt = n_qt - 1 - id / nbh;
    }
  }
  const int b = bhi / a.n_heads, h = bhi % a.n_heads;
  const SeqMeta sm = load_meta(a.lv, b);
  const int len = sm.len0;
  const int q0 = qt * BM;
  if (q0 >= len) return;
  const int64_t bh = bhi;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int wrow0 = q0 + wave * 32;        // first query row of this wave
  const int qi = wrow0 + l32;              // this lane's query row
  const float c = a.scale * kLog2e;

  // ---- Q fragments (B operand of S^T = K Q^T): query qi, dims ks*16 + hf*8 .. +8
  bf16x8 qf[8];
  {
    const bool ok = qi < len;
    const char* qp = ok ? pf_q_row(a, sm, bh, h, qi) : nullptr;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (ok) raw = *(const uint4*)(qp + (ks * 16 + hf * 8) * 2);
      qf[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  // ---- tile loader: thread -> (row = tid/16 + 16p, 16-byte chunk = tid%16)
  const int lrow = tid >> 4, lchunk = tid & 15;
  const int n_tiles = min((len + BN - 1) / BN, (q0 + BM + BN - 1) / BN);
  const int64_t v_head_off = (int64_t)h * a.head_stride * 2 + lchunk * 16;
  uint4 kreg[4], vreg[4];
  auto load_tile = [&](int t) {
    const int k0 = t * BN;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int pos = k0 + lrow + 16 * p;
      kreg[p] = make_uint4(0, 0, 0, 0);
      vreg[p] = make_uint4(0, 0, 0, 0);
      if (pos < len) {
        kreg[p] = *(const uint4*)(pf_k_row(a, sm, bh, h, pos) + lchunk * 16);
        vreg[p] = *(const uint4*)((const char*)a.v + (int64_t)(sm.tok0 + pos) * a.token_stride * 2 + v_head_off);
      }
    }
  };
  auto store_tile = [&](int buf) {
    char* kb = lds + buf * KTILE;
    char* vb = lds + 2 * KTILE + buf * VTILE;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int r = lrow + 16 * p;
      *(uint4*)(kb + r * KSTRIDE + lchunk * 16) = kreg[p];
      *(uint4*)(vb + r * VSTRIDE + lchunk * 16) = vreg[p];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  // per-lane LDS offsets that do not depend on the tile
  const int k_rd = l32 * KSTRIDE + hf * 16;                                    // + jb*32*KSTRIDE + ks*32
  const int v_rd = (hf * 4 + ((lane & 15) >> 2)) * VSTRIDE + (((l32 >> 4) * 16) + 4 * (lane & 3)) * 2;

  for (int t = 0; t < n_tiles; ++t) {
    const bool more = t + 1 < n_tiles;
    if (more) load_tile(t + 1);
    const int k0 = t * BN;
    if (k0 <= wrow0 + 31) {  // wave-uniform: otherwise every key of the tile is above the diagonal
      const char* kb = lds + (t & 1) * KTILE;
      const char* vb = lds + 2 * KTILE + (t & 1) * VTILE;
      f32x16 s[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[jb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
          const bf16x8 kf = *(const bf16x8*)(kb + k_rd + jb * 32 * KSTRIDE + ks * 32);
          s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[jb], 0, 0, 0);
        }
      }
      // accumulator register r of block jb holds key k0 + jb*32 + (r/4)*8 + hf*4 + r%4 for query qi
      if (k0 + BN - 1 > wrow0 || k0 + BN > len) {
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kj = k0 + jb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
            if (kj > qi || kj >= len) s[jb][r] = -INFINITY;
          }
      }
      float mloc = s[0][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mloc = fmaxf(mloc, s[0][r]);
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[1][r]);
      mloc = fmaxf(mloc, swap32(mloc));
      const float mnew = fmaxf(m, mloc);
      const bool upd = (mnew - m) * c > kRescaleThreshold;  // also true while m is -inf
      if (__builtin_amdgcn_ballot_w64(upd) != 0) {
        const float mu = upd ? mnew : m;
        const float alpha = __builtin_amdgcn_exp2f((m - mu) * c);
        m = mu;
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
      }
      const float mc = m * c;
      bf16x8 pb[4];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[jb][r], c, -mc));
          lsum += p;
          pb[jb * 2 + (r >> 3)][r & 7] = (__bf16)p;
        }
      // O^T += V^T P^T: k-step kk covers keys k0 + kk*16 .. +15; lane half hf supplies keys
      // {hf*4 .. +3} and {8 + hf*4 .. +3} of that run, exactly the keys its P registers hold.
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const char* vp = vb + v_rd + kk * 16 * VSTRIDE + db * 64;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp + 8 * VSTRIDE));
          const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v8), pb[kk], o[db], 0, 0, 0);
        }
      }
    }
    if (more) store_tile((t + 1) & 1);
    __syncthreads();
  }

  // ---- normalise and store: register r of block db is column db*32 + (r/4)*8 + hf*4 + r%4
  const float ltot = lsum + swap32(lsum);
  if (qi < len) {
    const float inv = 1.f / ltot;
    char* op = (char*)a.out + ((int64_t)(sm.tok0 + qi) * a.token_stride + (int64_t)h * a.head_stride) * 2;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        bf16x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = (__bf16)(o[db][g * 4 + x] * inv);
        *(bf16x4*)(op + (db * 32 + g * 8 + hf * 4) * 2) = w;
      }
  }
}

hipError_t launch_prefill_mfma_bf16_d128(const PrefillArgs& a, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)prefill_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, pf::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipError_t e = launch_cache_write_bf16_d128(a, stream);
  if (e != hipSuccess) return e;
  const int n_qt = (a.max_len + pf::BM - 1) / pf::BM;
  const int nbh = a.batch * a.n_heads;
  hipLaunchKernelGGL(prefill_mfma_kernel, dim3(n_qt * nbh), dim3(256), pf::LDS_BYTES, stream, a, n_qt, (nbh % 8 == 0) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace qc
