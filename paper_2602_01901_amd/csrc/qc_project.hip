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
// steps of 64 through a double-buffered LDS ring filled by global_load_lds_dwordx4 (steps of 32
// with a four-stage ring, three tiles ahead, measured 8 % slower: twice as many half-line requests).  Wave (wm, wn)
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
constexpr int BN = 256, BK = 64;      // BM = 64 * MB rows: MB row blocks of 32 per wave, two wave rows
constexpr int ROWB = BK * 2;            // bytes per tile row
constexpr int CH = ROWB / 16;           // 16-byte chunks per row
constexpr int RPI = 64 / CH;            // tile rows one wave-wide load instruction fills
constexpr int LPT = 32 / RPI;           // load instructions per wave for the 256-row B tile (a wave fills 32 rows)
constexpr int KSUB = BK / 16;           // MFMA k-steps per tile
constexpr int TILE_B = BN * ROWB;
constexpr int AHEAD = 1;                // tiles in flight ahead of the one being multiplied
constexpr int STAGES = AHEAD + 1;
// chunk c of row r is stored at chunk c ^ swz(r): 16 consecutive rows then cover all 64 banks
__device__ __forceinline__ int swz(int r) { return BK == 32 ? (r >> 2) & 3 : (r >> 1) & 7; }
constexpr int OUT_ROWB = BN * 2 + 16;   // output staging tile (bf16): padded rows, see the epilogue
template <int MB> struct Shape {
  static constexpr int BM = 64 * MB;
  static constexpr int TILE_A = BM * ROWB;
  static constexpr int STAGE = TILE_A + TILE_B;
  static constexpr int LPT_A = (BM / 8) / RPI;   // A-tile load instructions per wave (a wave fills BM/8 rows)
  static constexpr int TABLE = BM * 8;           // row table: (token, position) per tile row
  static constexpr int LDS_BYTES = TABLE + (STAGES * STAGE > BM * OUT_ROWB ? STAGES * STAGE : BM * OUT_ROWB);
};
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

template <int D, int MB>
__global__ __launch_bounds__(512, 1) void project_qk_kernel(ProjectArgs a, int m_tiles) {
  using namespace pj;
  using S = Shape<MB>;
  constexpr int BM = S::BM, TILE_A = S::TILE_A, STAGE = S::STAGE, LPT_A = S::LPT_A, TABLE = S::TABLE;
  static_assert(LPT_A >= 1, "a wave must fill at least one load instruction's worth of A rows");
  extern __shared__ __attribute__((aligned(16))) char lds_all[];
  int2* table = (int2*)lds_all;
  char* lds = lds_all + TABLE;  // the tile ring; reused as the output staging tile at the end

  // ---- which tile: column tiles (both matrices) fastest, so that the workgroups running together
  // share a few row tiles of x.  (Dealing blocks of 4 x 8 tiles to each XCD was measured: +2 %, and
  // it unbalances the XCDs when there are few row tiles.)
  const int nt2 = 2 * (a.n_heads * a.head_dim / BN);
  const int n_tile2 = blockIdx.x % nt2, m_tile = blockIdx.x / nt2;
  if (m_tile >= m_tiles) return;
  const int which = n_tile2 >= nt2 / 2;
  const int n0 = (n_tile2 - which * (nt2 / 2)) * BN, m0 = m_tile * BM;
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

  // ---- tile loader: wave w fills rows w*(BM/8) + p*RPI + lane/CH (p < LPT_A) of the A tile and
  // rows w*32 + p*RPI + lane/CH (p < LPT) of the B tile
  const int lchunk = lane % CH;
  uint32_t off_a[LPT_A], off_b[LPT];
#pragma unroll
  for (int p = 0; p < LPT_A; ++p) {
    const int r = wave * (BM / 8) + lane / CH + p * RPI;
    const int tok = max(table[r].x, 0);  // rows past the end repeat token 0; their results are not stored
    off_a[p] = (uint32_t)tok * (uint32_t)(a.x_stride * 2) + (lchunk ^ swz(r)) * 16;
  }
#pragma unroll
  for (int p = 0; p < LPT; ++p) {
    const int r = wave * 32 + lane / CH + p * RPI;
    off_b[p] = (uint32_t)(n0 + r) * (uint32_t)(a.w_stride * 2) + (lchunk ^ swz(r)) * 16;
  }
  const char* xbase = pj_uniform_ptr((const char*)a.x);
  const char* wbase = pj_uniform_ptr((const char*)a.w[which]);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)lds;
  auto load_tile = [&](int t) {
    const uint32_t st = lds_base + (t % STAGES) * STAGE;
    const uint32_t ab = __builtin_amdgcn_readfirstlane(st + wave * (BM / 8) * ROWB);
    const uint32_t bb = __builtin_amdgcn_readfirstlane(st + TILE_A + wave * 32 * ROWB);
    const char* xs = xbase + (uint64_t)t * (BK * 2);
    const char* ws = wbase + (uint64_t)t * (BK * 2);
#pragma unroll
    for (int p = 0; p < LPT_A; ++p) pj_async_copy16(xs, off_a[p], ab + p * RPI * ROWB);
#pragma unroll
    for (int p = 0; p < LPT; ++p) pj_async_copy16(ws, off_b[p], bb + p * RPI * ROWB);
  };
  constexpr int LOADS = LPT_A + LPT;  // load instructions per wave and tile

  // ---- fragment read offsets (tile-independent): k-substep ks uses logical chunk ks*2 + hf
  int a_off[MB][KSUB], b_off[2][KSUB];  // [block][ks]
  constexpr int PAIR = D / 2;    // distance of a rotary pair inside a head
  // column blocks of this wave inside the 256-column tile: a head's block j and j + PAIR/32
  const int col0 = (D == 128) ? (wn >> 1) * 128 + (wn & 1) * 32 : wn * 64;
#pragma unroll
  for (int ks = 0; ks < KSUB; ++ks) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int r = wm * (32 * MB) + mb * 32 + l32;
      a_off[mb][ks] = r * ROWB + (((ks * 2 + hf) ^ swz(r)) * 16);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int r = col0 + nb * PAIR + l32;
      b_off[nb][ks] = TILE_A + r * ROWB + (((ks * 2 + hf) ^ swz(r)) * 16);
    }
  }

  f32x16 acc[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

  const int n_steps = a.d_model / BK;
#pragma unroll
  for (int t = 0; t < AHEAD; ++t)
    if (t < n_steps) load_tile(t);

  for (int t = 0; t < n_steps; ++t) {
    // Tile t has landed when at most the loads of the tiles behind it are outstanding (loads complete
    // in order); near the end fewer tiles are in flight, so wait for everything.
    if (t + AHEAD <= n_steps) pj_wait_vmcnt<(AHEAD - 1) * LOADS>();
    else pj_wait_vmcnt<0>();
    __syncthreads();  // tile t visible to every wave; every wave is done with tile t-1, whose stage is refilled next
    if (t + AHEAD < n_steps) load_tile(t + AHEAD);
    const char* sb = lds + (t % STAGES) * STAGE;
    // Fragment reads and MFMAs of the four k-steps are left to the compiler's scheduler (hand-placed
    // double buffering across the barrier with scheduling fences measured 30 % slower).
#pragma unroll
    for (int ks = 0; ks < KSUB; ++ks) {
      bf16x8 af[MB], bf[2];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) af[mb] = *(const bf16x8*)(sb + a_off[mb][ks]);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) bf[nb] = *(const bf16x8*)(sb + b_off[nb][ks]);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mb], bf[nb], acc[mb][nb], 0, 0, 0);
    }
  }

  // ---- rotary embedding, then the tile goes through LDS so that it leaves in 16-byte pieces
  // (two whole 512-byte output rows per wave instruction).  Accumulator register r of block
  // (mb, nb) holds row wm*32*MB + mb*32 + (r/4)*8 + hf*4 + r%4 and column col0 + nb*PAIR + l32.
  const int tcol = col0 + l32;            // tile column of the lower half of the pair
  const int d = (n0 + tcol) % D;          // rotary index, < PAIR
  // The hardware sine and cosine take their argument in revolutions: the angle pos * theta^(-2d/D)
  // is formed and reduced to [-1/2, 1/2] revolutions in double precision, then evaluated in single.
  double rev_per_pos = 0.0;
  if (a.rope_theta > 0.f) rev_per_pos = exp2(-2.0 * (double)d / (double)D * a.log2_theta) * 0.15915494309189535;
  __syncthreads();  // every wave is done with the ring
  // Staging rows are 16 bytes longer than the tile row: the two lane halves of a wave write rows
  // four apart, which then fall into different banks.
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = wm * (32 * MB) + mb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
      float lo = acc[mb][0][r], hi = acc[mb][1][r];
      if (a.rope_theta > 0.f) {
        const double rev = (double)table[row].y * rev_per_pos;
        const float frac = (float)(rev - rint(rev));
        const float sn = __builtin_amdgcn_sinf(frac), cs = __builtin_amdgcn_cosf(frac);
        const float nlo = lo * cs - hi * sn, nhi = hi * cs + lo * sn;
        lo = nlo;
        hi = nhi;
      }
      bf16_t* o = (bf16_t*)(lds + row * OUT_ROWB) + tcol;
      o[0] = (bf16_t)lo;
      o[PAIR] = (bf16_t)hi;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < BM * (BN / 8) / 512; ++it) {
    const int piece = it * 512 + tid;
    const int row = piece / (BN / 8), ch = piece % (BN / 8);
    const int tok = table[row].x;
    if (tok < 0) continue;
    const int col = n0 + ch * 8;
    const uint4 v = *(const uint4*)(lds + row * OUT_ROWB + ch * 16);
    *(uint4*)((char*)a.out[which] + ((int64_t)tok * a.token_stride + (int64_t)(col / D) * a.head_stride + col % D) * 2) = v;
  }
}

// ---- at most 32 rows (a decode step): the work is reading both weight matrices once -------------
// One workgroup = 4 waves = one rotary pair of 16-column groups (16 features d, 16 features d + D/2)
// of one head of one matrix, all rows, all of K.  Wave w takes the k-steps of 32 congruent to w
// mod 4, so that a round of the four waves reads 256 contiguous bytes of every weight row.
// Operands go straight from global memory into v_mfma_f32_16x16x32_bf16 fragments (nothing is
// reused inside a workgroup: the rows of x are few and stay in L2 for the other workgroups); the
// four partial 32 x 32 results are added in a fixed order through LDS, rotated and stored.
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int D>
__global__ __launch_bounds__(256) void project_qk_skinny_kernel(ProjectArgs a, int n_rows) {
  constexpr int PAIR = D / 2, GROUPS = PAIR / 16;
  __shared__ float part[4][32][33];
  __shared__ int2 table[32];
  const int which = blockIdx.y;
  const int head = blockIdx.x / GROUPS, grp = blockIdx.x % GROUPS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;  // fragment row / column, and which 8 of the 32 k values

  if (tid < 32) {
    int tok = -1, pos = 0, base = 0;
    for (int s = 0; s < a.segs.n; ++s) {
      const int c = a.segs.count[s];
      if (tid >= base && tid < base + c) {
        tok = a.segs.tok_start[s] + (tid - base);
        pos = a.segs.pos_start[s] + (tid - base);
      }
      base += c;
    }
    table[tid] = make_int2(tok, pos);
  }
  __syncthreads();

  const int col_lo = head * D + grp * 16 + l16;
  const char* w_lo = (const char*)a.w[which] + ((int64_t)col_lo * a.w_stride + kq * 8) * 2;
  const char* w_hi = w_lo + (int64_t)PAIR * a.w_stride * 2;
  const char* x0 = (const char*)a.x + ((int64_t)max(table[l16].x, 0) * a.x_stride + kq * 8) * 2;
  const char* x1 = (const char*)a.x + ((int64_t)max(table[16 + l16].x, 0) * a.x_stride + kq * 8) * 2;
  const bool two = n_rows > 16;

  f32x4 acc[2][2];  // [row block][lo, hi]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int n_steps = a.d_model / 32;
  constexpr int UN = 8;  // k-steps in flight per wave
  for (int ks0 = wave; ks0 < n_steps; ks0 += 4 * UN) {
    bf16x8 bl[UN], bh[UN], a0[UN], a1[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int ks = ks0 + 4 * u;
      if (ks < n_steps) {
        const int64_t off = (int64_t)ks * 64;
        bl[u] = __builtin_bit_cast(bf16x8, *(const uint4*)(w_lo + off));
        bh[u] = __builtin_bit_cast(bf16x8, *(const uint4*)(w_hi + off));
        a0[u] = __builtin_bit_cast(bf16x8, *(const uint4*)(x0 + off));
        if (two) a1[u] = __builtin_bit_cast(bf16x8, *(const uint4*)(x1 + off));
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (ks0 + 4 * u < n_steps) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], bl[u], acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[u], bh[u], acc[0][1], 0, 0, 0);
        if (two) {
          acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], bl[u], acc[1][0], 0, 0, 0);
          acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[u], bh[u], acc[1][1], 0, 0, 0);
        }
      }
    }
  }
  // accumulator register i of block (rb, c) holds row rb*16 + kq*4 + i, column c*16 + l16
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) part[wave][rb * 16 + kq * 4 + i][c * 16 + l16] = acc[rb][c][i];
  __syncthreads();
  // 32 rows x 16 pairs: two items per thread; the four partials are added in wave order
  for (int item = tid; item < 32 * 16; item += 256) {
    const int row = item >> 4, j = item & 15;
    const int2 tp = table[row];
    if (tp.x < 0) continue;
    float lo = ((part[0][row][j] + part[1][row][j]) + part[2][row][j]) + part[3][row][j];
    float hi = ((part[0][row][16 + j] + part[1][row][16 + j]) + part[2][row][16 + j]) + part[3][row][16 + j];
    const int d = grp * 16 + j;
    if (a.rope_theta > 0.f) {
      const double rev = (double)tp.y * exp2(-2.0 * (double)d / (double)D * a.log2_theta) * 0.15915494309189535;
      const float frac = (float)(rev - rint(rev));
      const float sn = __builtin_amdgcn_sinf(frac), cs = __builtin_amdgcn_cosf(frac);
      const float nlo = lo * cs - hi * sn, nhi = hi * cs + lo * sn;
      lo = nlo;
      hi = nhi;
    }
    bf16_t* o = (bf16_t*)a.out[which] + (int64_t)tp.x * a.token_stride + (int64_t)head * a.head_stride + d;
    o[0] = (bf16_t)lo;
    o[PAIR] = (bf16_t)hi;
  }
}

// The same job when d_model is a multiple of 256, with longer contiguous reads: every visit to a
// weight row (and to a row of x) fetches 512 contiguous bytes instead of 64 (measured 12 % faster).
// K is walked in chunks of 256, each chunk of the 32 weight rows and of the rows of x goes
// to LDS by global_load_lds_dwordx4 (one instruction = two whole 512-byte row pieces), three
// chunks ahead of its use through a four-stage ring; fragments are then read from LDS (16-byte
// chunk c of row r sits at chunk c ^ (r & 15): conflict-free for the fragment pattern).
namespace sk {
constexpr int KC = 256, ROWB = KC * 2, ROWS = 32;
constexpr int TILE = ROWS * ROWB;          // 16 KB: the weight rows, or the rows of x
constexpr int STAGE = 2 * TILE, AHEAD = 3, STAGES = AHEAD + 1;
constexpr int LDS_BYTES = STAGES * STAGE;  // 128 KB
constexpr int LOADS = 2 * (TILE / 1024) / 4;  // load instructions per wave and chunk
}  // namespace sk

template <int D>
__global__ __launch_bounds__(256) void project_qk_skinny_staged_kernel(ProjectArgs a, int n_rows) {
  using namespace sk;
  constexpr int PAIR = D / 2, GROUPS = PAIR / 16;
  extern __shared__ __attribute__((aligned(16))) char ring[];
  __shared__ float part[4][32][33];
  __shared__ int2 table[32];
  const int which = blockIdx.y;
  const int head = blockIdx.x / GROUPS, grp = blockIdx.x % GROUPS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;

  if (tid < 32) {
    int tok = -1, pos = 0, base = 0;
    for (int s = 0; s < a.segs.n; ++s) {
      const int c = a.segs.count[s];
      if (tid >= base && tid < base + c) {
        tok = a.segs.tok_start[s] + (tid - base);
        pos = a.segs.pos_start[s] + (tid - base);
      }
      base += c;
    }
    table[tid] = make_int2(tok, pos);
  }
  __syncthreads();

  // ---- loader: wave w fills tile rows w*8 + p*2 + lane/32 (p < 4), lane%32 = physical 16-byte chunk.
  // Weight tile row r is feature d = grp*16 + (r & 15) of the head, plus D/2 for r >= 16.
  uint32_t off_w[4], off_x[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int r = wave * 8 + p * 2 + (lane >> 5);
    const int logical = (lane & 31) ^ (r & 15);
    const int wrow = head * D + grp * 16 + (r & 15) + (r >> 4) * PAIR;
    off_w[p] = (uint32_t)wrow * (uint32_t)(a.w_stride * 2) + logical * 16;
    off_x[p] = (uint32_t)max(table[r].x, 0) * (uint32_t)(a.x_stride * 2) + logical * 16;  // idle rows repeat token 0
  }
  const char* wbase = pj_uniform_ptr((const char*)a.w[which]);
  const char* xbase = pj_uniform_ptr((const char*)a.x);
  const uint32_t ring_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)ring;
  auto load_chunk = [&](int t) {
    const uint32_t st = ring_base + (t % STAGES) * STAGE;
    const uint32_t wb = __builtin_amdgcn_readfirstlane(st + wave * 8 * ROWB);
    const uint32_t xb = __builtin_amdgcn_readfirstlane(st + TILE + wave * 8 * ROWB);
    const char* ws = wbase + (uint64_t)t * ROWB;
    const char* xs = xbase + (uint64_t)t * ROWB;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      pj_async_copy16(ws, off_w[p], wb + p * 2 * ROWB);
      pj_async_copy16(xs, off_x[p], xb + p * 2 * ROWB);
    }
  };
  static_assert(LOADS == 8, "four weight and four x instructions per wave and chunk");

  const bool two = n_rows > 16;
  f32x4 acc[2][2];  // [row block][lo, hi]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int n_chunks = a.d_model / KC;
#pragma unroll
  for (int t = 0; t < AHEAD; ++t)
    if (t < n_chunks) load_chunk(t);
  for (int t = 0; t < n_chunks; ++t) {
    if (t + AHEAD <= n_chunks) pj_wait_vmcnt<(AHEAD - 1) * LOADS>();
    else pj_wait_vmcnt<0>();
    __syncthreads();  // chunk t visible; every wave is done with chunk t-1, whose stage is refilled next
    if (t + AHEAD < n_chunks) load_chunk(t + AHEAD);
    const char* sb = ring + (t % STAGES) * STAGE;
    // wave w takes the k-steps of 32 congruent to w mod 4 (two per chunk); fragment chunk = ks*4 + kq
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int phys = (((wave + 4 * j) * 4 + kq) ^ l16) * 16;
      const bf16x8 bl = *(const bf16x8*)(sb + l16 * ROWB + phys);
      const bf16x8 bh = *(const bf16x8*)(sb + (16 + l16) * ROWB + phys);
      const bf16x8 a0 = *(const bf16x8*)(sb + TILE + l16 * ROWB + phys);
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bl, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bh, acc[0][1], 0, 0, 0);
      if (two) {
        const bf16x8 a1 = *(const bf16x8*)(sb + TILE + (16 + l16) * ROWB + phys);
        acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bl, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bh, acc[1][1], 0, 0, 0);
      }
    }
  }
  // accumulator register i of block (rb, c) holds row rb*16 + kq*4 + i, column c*16 + l16
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) part[wave][rb * 16 + kq * 4 + i][c * 16 + l16] = acc[rb][c][i];
  __syncthreads();
  for (int item = tid; item < 32 * 16; item += 256) {
    const int row = item >> 4, j = item & 15;
    const int2 tp = table[row];
    if (tp.x < 0) continue;
    float lo = ((part[0][row][j] + part[1][row][j]) + part[2][row][j]) + part[3][row][j];
    float hi = ((part[0][row][16 + j] + part[1][row][16 + j]) + part[2][row][16 + j]) + part[3][row][16 + j];
    const int d = grp * 16 + j;
    if (a.rope_theta > 0.f) {
      const double rev = (double)tp.y * exp2(-2.0 * (double)d / (double)D * a.log2_theta) * 0.15915494309189535;
      const float frac = (float)(rev - rint(rev));
      const float sn = __builtin_amdgcn_sinf(frac), cs = __builtin_amdgcn_cosf(frac);
      const float nlo = lo * cs - hi * sn, nhi = hi * cs + lo * sn;
      lo = nlo;
      hi = nhi;
    }
    bf16_t* o = (bf16_t*)a.out[which] + (int64_t)tp.x * a.token_stride + (int64_t)head * a.head_stride + d;
    o[0] = (bf16_t)lo;
    o[PAIR] = (bf16_t)hi;
  }
}

template <int D> static hipError_t launch_skinny_staged_t(const ProjectArgs& a, int n_rows, hipStream_t stream) {
  static std::atomic<unsigned long long> attr_set{0};
  if (hipError_t e = ensure_dynamic_lds((const void*)project_qk_skinny_staged_kernel<D>, sk::LDS_BYTES, attr_set); e != hipSuccess) return e;
  hipLaunchKernelGGL(project_qk_skinny_staged_kernel<D>, dim3(a.n_heads * (D / 32), 2), dim3(256), sk::LDS_BYTES, stream, a, n_rows);
  return hipGetLastError();
}

hipError_t launch_project_qk_skinny(const ProjectArgs& a, int n_rows, hipStream_t stream) {
  if (a.d_model % sk::KC == 0)
    return a.head_dim == 128 ? launch_skinny_staged_t<128>(a, n_rows, stream) : launch_skinny_staged_t<64>(a, n_rows, stream);
  if (a.head_dim == 128) {
    hipLaunchKernelGGL(project_qk_skinny_kernel<128>, dim3(a.n_heads * 4, 2), dim3(256), 0, stream, a, n_rows);
  } else {
    hipLaunchKernelGGL(project_qk_skinny_kernel<64>, dim3(a.n_heads * 2, 2), dim3(256), 0, stream, a, n_rows);
  }
  return hipGetLastError();
}

template <int D, int MB>
static hipError_t launch_project_qk_t(const ProjectArgs& a, int rows, hipStream_t stream) {
  static std::atomic<unsigned long long> attr_set{0};
  constexpr int lds_bytes = pj::Shape<MB>::LDS_BYTES;
  if (hipError_t e = ensure_dynamic_lds((const void*)project_qk_kernel<D, MB>, lds_bytes, attr_set); e != hipSuccess) return e;
  const int m_tiles = (rows + pj::Shape<MB>::BM - 1) / pj::Shape<MB>::BM;
  const int nt2 = 2 * (a.n_heads * a.head_dim / pj::BN);
  hipLaunchKernelGGL((project_qk_kernel<D, MB>), dim3(m_tiles * nt2), dim3(512), lds_bytes, stream, a, m_tiles);
  return hipGetLastError();
}

// 256-row tiles when they fill the chip at least twice over, 128-row tiles for fewer rows (the text
// rows of a lazy layer): twice as many workgroups, each half as long.
hipError_t launch_project_qk(const ProjectArgs& a, int rows, hipStream_t stream) {
  const int nt2 = 2 * (a.n_heads * a.head_dim / pj::BN);
  const bool big = (int64_t)((rows + 255) / 256) * nt2 >= 512;
  if (a.head_dim == 128) return big ? launch_project_qk_t<128, 4>(a, rows, stream) : launch_project_qk_t<128, 2>(a, rows, stream);
  return big ? launch_project_qk_t<64, 4>(a, rows, stream) : launch_project_qk_t<64, 2>(a, rows, stream);
}

}  // namespace qc
