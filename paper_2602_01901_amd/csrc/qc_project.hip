// Query/key projection with rotary embedding, text rows only in a lazy layer (paper Eq. 7, first
// terms of Q and K; "Efficiency Analysis", FLOPs paragraph: this is where the omitted work lives).
//
//   Y[m][n] = sum_k X[row(m)][k] * W[n][k]        X: [tokens][d_model], W: [H*D][d_model], bf16
//
// over the compacted list of rows to project (up to two contiguous token ranges per sequence: the
// text before and behind the visual span; everything for an ordinary layer), followed by the
// rotate-half rotary embedding at each row's true position and a bf16 store into the [token][H][D]
// tensors the attention entry points take.  Rows inside the span are neither computed nor written.
//
// One workgroup = 8 waves = a 256 x 256 output tile of one matrix (W_Q or W_K); K is walked in
// steps of 64 through a double-buffered LDS ring filled by global_load_lds_dwordx4.  Wave (wm, wn)
// owns 128 rows x 2 column blocks of 32 that form a rotary pair (d, d + D/2) of one head, so the
// rotation needs no data exchange: both halves of a pair sit in the same lane and register index.
// Per k-step of 16 a wave reads 4 row fragments and 2 column fragments for 8 MFMAs (0.75 KB of LDS
// per v_mfma_f32_32x32x16_bf16).  LDS rows are 128 bytes; 16-byte chunk c of row r is stored at
// chunk c ^ ((r >> 1) & 7), which makes both the DMA writes and the fragment reads conflict-free.
#include "qc_device.h"

namespace qc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace pj {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROWB = BK * 2;            // bytes per tile row
constexpr int TILE_A = BM * ROWB;       // 32 KB
constexpr int TILE_B = BN * ROWB;       // 32 KB
constexpr int STAGE = TILE_A + TILE_B;  // 64 KB
constexpr int STAGES = 2;
constexpr int TABLE = BM * 8;           // row table: (token, position) per tile row
constexpr int LDS_BYTES = STAGES * STAGE + TABLE;
}  // namespace pj

__device__ __forceinline__ void pj_async_copy16(const char* sbase, uint32_t voff, uint32_t lds_off) {
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(voff), "s"(sbase), "s"(lds_off)
               : "memory");
}
__device__ __forceinline__ const char* pj_uniform_ptr(const char* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}
template <int N> __device__ __forceinline__ void pj_wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <int D>
__global__ __launch_bounds__(512, 1) void project_qk_kernel(ProjectArgs a) {
  using namespace pj;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  int2* table = (int2*)(lds + STAGES * STAGE);

  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM, which = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- row table: compact row m0 + r -> (token index, position), token = -1 past the end
  if (tid < BM) {
    const int m = m0 + tid;
    int tok = -1, pos = 0, base = 0;
    for (int s = 0; s < a.segs.n; ++s) {
      const int c = a.segs.count[s];
      if (m >= base && m < base + c) {
        tok = a.segs.tok_start[s] + (m - base);
        pos = a.segs.pos_start[s] + (m - base);
      }
      base += c;
    }
    table[tid] = make_int2(tok, pos);
  }
  __syncthreads();

  // ---- tile loader: wave w fills rows w*32 + p*8 + lane/8 (p = 0..3) of the A and of the B tile
  const int lrow = wave * 32 + (lane >> 3), lchunk = lane & 7;
  uint32_t off_a[4], off_b[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int r = lrow + p * 8;
    const int tok = max(table[r].x, 0);  // rows past the end repeat token 0; their results are not stored
    const int sw = (lchunk ^ ((r >> 1) & 7)) * 16;
    off_a[p] = (uint32_t)tok * (uint32_t)(a.x_stride * 2) + sw;
    off_b[p] = (uint32_t)(n0 + r) * (uint32_t)(a.d_model * 2) + sw;
  }
  const char* xbase = pj_uniform_ptr((const char*)a.x);
  const char* wbase = pj_uniform_ptr((const char*)a.w[which]);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)lds;
  auto load_tile = [&](int t) {
    const uint32_t ab = __builtin_amdgcn_readfirstlane(lds_base + (t % STAGES) * STAGE + wave * 32 * ROWB);
    const uint32_t bb = ab + TILE_A;
    const char* xs = xbase + (uint64_t)t * (BK * 2);
    const char* ws = wbase + (uint64_t)t * (BK * 2);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      pj_async_copy16(xs, off_a[p], ab + p * 8 * ROWB);
      pj_async_copy16(ws, off_b[p], bb + p * 8 * ROWB);
    }
  };

  // ---- fragment read offsets (tile-independent): k-substep ks uses logical chunk ks*2 + hf
  int a_off[4][4], b_off[2][4];  // [block][ks]
  constexpr int PAIR = D / 2;    // distance of a rotary pair inside a head
  // column blocks of this wave inside the 256-column tile: a head's block j and j + PAIR/32
  const int col0 = (D == 128) ? (wn >> 1) * 128 + (wn & 1) * 32 : wn * 64;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const int r = wm * 128 + mb * 32 + l32;
      a_off[mb][ks] = r * ROWB + (((ks * 2 + hf) ^ ((r >> 1) & 7)) * 16);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int r = col0 + nb * PAIR + l32;
      b_off[nb][ks] = TILE_A + r * ROWB + (((ks * 2 + hf) ^ ((r >> 1) & 7)) * 16);
    }
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

  const int n_steps = a.d_model / BK;
  load_tile(0);
  for (int t = 0; t < n_steps; ++t) {
    pj_wait_vmcnt<0>();
    __syncthreads();  // tile t visible to every wave; every wave is done with tile t-1
    if (t + 1 < n_steps) load_tile(t + 1);
    const char* sb = lds + (t % STAGES) * STAGE;
    bf16x8 af[2][4], bf[2][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) af[0][mb] = *(const bf16x8*)(sb + a_off[mb][0]);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) bf[0][nb] = *(const bf16x8*)(sb + b_off[nb][0]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      if (ks + 1 < 4) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) af[nxt][mb] = *(const bf16x8*)(sb + a_off[mb][ks + 1]);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) bf[nxt][nb] = *(const bf16x8*)(sb + b_off[nb][ks + 1]);
      }
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][mb], bf[cur][nb], acc[mb][nb], 0, 0, 0);
    }
  }

  // ---- rotary embedding and store.  Accumulator register r of block (mb, nb) holds row
  // wm*128 + mb*32 + (r/4)*8 + hf*4 + r%4 and column col0 + nb*PAIR + l32 of the tile.
  const int col = n0 + col0 + l32;      // output feature of the lower half of the pair
  const int head = col / D, d = col % D;  // d < PAIR
  double inv_freq = 0.0;
  if (a.rope_theta > 0.f) inv_freq = exp2(-2.0 * (double)d / (double)D * a.log2_theta);
  char* obase = (char*)a.out[which] + ((int64_t)head * a.head_stride + d) * 2;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = wm * 128 + mb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
      const int2 tp = table[row];
      if (tp.x < 0) continue;
      float lo = acc[mb][0][r], hi = acc[mb][1][r];
      if (a.rope_theta > 0.f) {
        // angle reduced to [-pi, pi] in double, sine and cosine in single precision
        const double ang = (double)tp.y * inv_freq;
        const double turns = ang * 0.15915494309189535;  // 1 / (2 pi)
        const float red = (float)((turns - rint(turns)) * 6.283185307179586);
        float sn, cs;
        __sincosf(red, &sn, &cs);
        const float nlo = lo * cs - hi * sn, nhi = hi * cs + lo * sn;
        lo = nlo;
        hi = nhi;
      }
      bf16_t* o = (bf16_t*)(obase + (int64_t)tp.x * a.token_stride * 2);
      o[0] = (bf16_t)lo;
      o[PAIR] = (bf16_t)hi;
    }
}

hipError_t launch_project_qk(const ProjectArgs& a, int m_tiles, hipStream_t stream) {
  static bool attr_set[2] = {false, false};
  const int which = a.head_dim == 128 ? 1 : 0;
  const void* fn = which ? (const void*)project_qk_kernel<128> : (const void*)project_qk_kernel<64>;
  if (!attr_set[which]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, pj::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set[which] = true;
  }
  dim3 grid(a.n_heads * a.head_dim / pj::BN, m_tiles, 2);
  if (which) hipLaunchKernelGGL(project_qk_kernel<128>, grid, dim3(512), pj::LDS_BYTES, stream, a);
  else hipLaunchKernelGGL(project_qk_kernel<64>, grid, dim3(512), pj::LDS_BYTES, stream, a);
  return hipGetLastError();
}

}  // namespace qc
