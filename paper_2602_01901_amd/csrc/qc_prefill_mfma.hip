// Prefill attention on the matrix cores: bf16 inputs, head_dim 128 (paper Eq. 1; Eq. 7 in a lazy
// layer).  Flash-style: the score matrix is never materialised; softmax runs online in fp32.
//
// Work split.  One workgroup of 4 waves takes BM = 128 consecutive query rows of one (sequence,
// head); each wave owns 32 of them for the whole kernel; two workgroups share a CU (their phases
// drift apart, so one's matrix work meets the other's vector work).  Keys/values are visited in
// tiles of BN = 64 rows, double buffered in LDS: the global->LDS loads of tile t+1 are in flight
// while tile t is multiplied.
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
// of the kernel is unchanged.
//
// Cache writes are fused: a workgroup stores the K/V rows of its own query range from the key
// tiles on its diagonal (which it has in LDS anyway) and the Q Cache rows from its Q fragments.
#include "qc_device.h"

namespace qc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

namespace pf {
constexpr int NW = 4;                  // waves per workgroup
constexpr int BM = NW * 32;            // query rows per workgroup
constexpr int STAGES = 2;              // LDS buffers per tile ring
constexpr int LPT = 16 / NW;           // load instructions per wave per tile and matrix (4 rows each)
constexpr int BN = 64, D = 128;
constexpr int ROWB = D * 2;            // bytes per row
constexpr int TILE = BN * ROWB;        // one K or V tile in LDS (no padding; XOR-swizzled 16-byte chunks)
constexpr int STAGE = 2 * TILE;        // one ring stage: K tile then V tile
constexpr float kRescaleThreshold = 8.0f;  // log2 units
}  // namespace pf

// LDS layout.  A tile row is 16 chunks of 16 bytes.  K rows store logical chunk c at physical
// chunk c ^ (row & 15): the 16-byte operand reads of 16 consecutive rows then cover all 64 banks.
// V rows store chunk c at c ^ ((row & 3) << 2): the 4-row transposing reads hit 4 distinct
// quarter-rows.  Tiles are filled by global_load_lds_dwordx4 (each lane's 16 bytes land at
// consecutive LDS addresses), so the swizzle is applied on the global side: lane i of an
// instruction that fills rows r0..r0+3 fetches logical chunk (i % 16) ^ swz(row).

// Page lists of one sequence (paged batches; null otherwise): positions, k_own's pool, q_cache's pool.
struct PfPages {
  const int32_t *seq, *k, *q;
};
// Up to two pages that a run of at most 64 consecutive rows of a pool touches, fetched by scalar loads:
// rows of page index `first` live on page p0, rows of the next index on p1.
struct PagePair {
  int first, p0, p1;
  __device__ __forceinline__ int64_t row(int r, int h, int n_heads) const {
    return ((int64_t)((r >> 6) == first ? p0 : p1) * n_heads + h) * kPageRows + (r & (kPageRows - 1));
  }
};
// `first` must be a wave-uniform index; both entries read lie inside the list (entries the sequence does
// not hold are fetched but never chosen by a row that exists).
__device__ __forceinline__ PagePair load_page_pair(const int32_t* list, int first, int list_len) {
  PagePair pp = {first, 0, 0};
  if (list_len > 0) {
    pp.first = min(first, list_len - 1);
    pp.p0 = uniform_load(list + pp.first);
    pp.p1 = uniform_load(list + min(pp.first + 1, list_len - 1));
  }
  return pp;
}
// qp: the Q Cache pages of the wave's query rows (paged batches).
template <bool PAGED>
__device__ __forceinline__ const char* pf_q_row(const PrefillArgs& a, const SeqMeta& sm, const RowBase& rb, const PagePair& qp, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len) {
    const int r = pos - sm.vis_start;
    return a.lv.q_cache + (PAGED ? qp.row(r, h, a.n_heads) : rb.q + r) * pf::ROWB;
  }
  return (const char*)a.q + ((int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride) * 2;
}
// page: the page that holds the positions of pos's key tile (paged batches; a tile is one page).
template <bool PAGED>
__device__ __forceinline__ const char* pf_k_row(const PrefillArgs& a, const SeqMeta& sm, const RowBase& rb, int page, int h, int pos) {
  if (a.is_lazy && pos >= sm.vis_start && pos < sm.vis_start + sm.vis_len)
    return a.lv.k_anchor + (PAGED ? ((int64_t)page * a.n_heads + h) * kPageRows + (pos & (kPageRows - 1)) : rb.anchor + pos) * pf::ROWB;
  return (const char*)a.k + ((int64_t)(sm.tok0 + pos) * a.token_stride + (int64_t)h * a.head_stride) * 2;
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// One global_load_lds_dwordx4: lane i's 16 bytes go to LDS byte offset lds_off + 16*i (lds_off is
// wave-uniform and travels in M0, which is saved and restored around the instruction).  Issued as
// inline asm so that the compiler does not tie later LDS reads of the OTHER buffer to these
// loads; the kernel waits for them itself (vmcnt(0)) before the barrier that publishes the tile.
__device__ __forceinline__ void async_copy16(const char* src, uint32_t lds_off) {
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(src), "s"(lds_off)
               : "memory");
}
// Same with a wave-uniform 64-bit base in SGPRs and a 32-bit per-lane byte offset.
__device__ __forceinline__ void async_copy16_sv(const char* sbase, uint32_t voff, uint32_t lds_off) {
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(voff), "s"(sbase), "s"(lds_off)
               : "memory");
}
// Pin a wave-uniform pointer into scalar registers.
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_offset_of(const char* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ bf16x8 lds_read_tr8(const char* p0, const char* p1) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p1));
  const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v8);
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {  // at most N vector-memory ops outstanding
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// PAGED: cache rows live on pages of 64 rows, which is also the key tile: a key tile read from the first
// layer's K cache and the tiles a workgroup stores are one page each.
template <bool PAGED>
__global__ __launch_bounds__(pf::NW * 64, 2) void prefill_mfma_kernel(PrefillArgs a, int n_qt, int xcd_map) {
  static_assert(pf::BN == kPageRows, "a key tile is one page");
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
  const SeqMeta sm = load_meta(a.lv, b, a.inherit_all);
  const int len = sm.len0;
  const int q0 = qt * BM;
  if (q0 >= len) return;
  const RowBase rb = PAGED ? RowBase{0, 0, 0, 0} : row_bases(a.lv, b, h, a.n_heads);
  PfPages pg = {nullptr, nullptr, nullptr};
  if constexpr (PAGED) {
    pg.seq = a.lv.pt_seq + (int64_t)b * a.lv.pt_seq_stride;
    pg.k = a.lv.pt_k + (int64_t)b * a.lv.pt_k_stride;
    pg.q = a.lv.pt_q + (int64_t)b * a.lv.pt_q_stride;
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int wrow0 = q0 + wave * 32;        // first query row of this wave
  const int qi = wrow0 + l32;              // this lane's query row
  const float c = a.scale * kLog2e;

  f32x16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  // ---- tile loader: wave w fills rows w*16 + p*4 + lane/16, p = 0..3, of the K and V tiles
  const int n_tiles = min((len + BN - 1) / BN, (q0 + BM + BN - 1) / BN);
  const int lrow = wave * (4 * LPT) + (lane >> 4), lchunk = lane & 15;
  const uint32_t lds_base = lds_offset_of(lds);
  // Fast path (tile fully inside the sequence and taken from one source): a wave-uniform 64-bit
  // base that already includes the tile offset, plus per-lane 32-bit offsets fixed for the kernel.
  const uint32_t ts2 = (uint32_t)(a.token_stride * 2);
  const char* kin_base = uniform_ptr((const char*)a.k + ((int64_t)sm.tok0 * a.token_stride + (int64_t)h * a.head_stride) * 2);
  const char* vin_base = uniform_ptr((const char*)a.v + ((int64_t)sm.tok0 * a.token_stride + (int64_t)h * a.head_stride) * 2);
  const char* kanc_base = uniform_ptr(a.is_lazy ? a.lv.k_anchor + (PAGED ? (int64_t)h * kPageRows : rb.anchor) * ROWB : nullptr);
  const int64_t page_bytes = (int64_t)a.n_heads * kPageRows * ROWB;   // one page of a region, all heads
  uint32_t off_kin[LPT], off_kanc[LPT], off_v[LPT];
#pragma unroll
  for (int p = 0; p < LPT; ++p) {
    const int r = lrow + 4 * p;
    off_kin[p] = r * ts2 + ((lchunk ^ (r & 15)) * 16);
    off_kanc[p] = r * ROWB + ((lchunk ^ (r & 15)) * 16);
    off_v[p] = r * ts2 + ((lchunk ^ ((r & 3) << 2)) * 16);
  }
  const int span_lo = a.is_lazy ? sm.vis_start : 0, span_hi = a.is_lazy ? sm.vis_start + sm.vis_len : 0;
  // `page`: paged batches, lazy layer: the page of the sequence that holds positions t*64 .. t*64+63
  auto load_tile = [&](int t, int page) {
    const uint32_t kb = __builtin_amdgcn_readfirstlane(lds_base + (t % STAGES) * STAGE + wave * (4 * LPT) * ROWB);
    const uint32_t vb = kb + TILE;
    const int k0 = __builtin_amdgcn_readfirstlane(t * BN);
    const bool inside = k0 >= span_lo && k0 + BN <= span_hi;
    const bool outside = k0 + BN <= span_lo || k0 >= span_hi;
    if (k0 + BN <= len && (inside || outside)) {
      const char* vsrc = vin_base + (uint64_t)k0 * ts2;
      if (inside) {
        const char* ksrc = PAGED ? kanc_base + (uint64_t)page * page_bytes : kanc_base + (uint64_t)k0 * ROWB;
#pragma unroll
        for (int p = 0; p < LPT; ++p) {
          async_copy16_sv(ksrc, off_kanc[p], kb + p * 4 * ROWB);
          async_copy16_sv(vsrc, off_v[p], vb + p * 4 * ROWB);
        }
      } else {
        const char* ksrc = kin_base + (uint64_t)k0 * ts2;
#pragma unroll
        for (int p = 0; p < LPT; ++p) {
          async_copy16_sv(ksrc, off_kin[p], kb + p * 4 * ROWB);
          async_copy16_sv(vsrc, off_v[p], vb + p * 4 * ROWB);
        }
      }
    } else {  // ragged last tile or a tile straddling a span boundary: per-row addresses
#pragma unroll
      for (int p = 0; p < LPT; ++p) {
        const int r = lrow + 4 * p;
        const int pos = min(k0 + r, len - 1);  // rows past the end repeat the last row; their scores are masked
        async_copy16(pf_k_row<PAGED>(a, sm, rb, page, h, pos) + ((lchunk ^ (r & 15)) * 16), kb + p * 4 * ROWB);
        async_copy16(vin_base + (int64_t)pos * ts2 + ((lchunk ^ ((r & 3) << 2)) * 16), vb + p * 4 * ROWB);
      }
    }
  };

  // Paged lazy layers: lane i keeps the page of key tile 64*block + i of the sequence, for the current
  // block of 64 tiles and the next one (one vector load per 64 tiles, long complete when first used);
  // a tile's page is then a lane read away, with no memory access in the tile loop.
  int pages_cur = 0, pages_next = 0;
  auto fetch_pages = [&](int block) -> int {
    if constexpr (PAGED)
      if (a.is_lazy) return pg.seq[min(block * 64 + lane, a.lv.pt_seq_stride - 1)];
    return 0;
  };
  auto page_of_tile = [&](int t) -> int {
    if constexpr (PAGED) return __builtin_amdgcn_readlane(pages_cur, t & 63);
    else return 0;
  };
  pages_cur = fetch_pages(0);
  pages_next = fetch_pages(1);
  load_tile(0, page_of_tile(0));  // issued before the Q loads below so that the two latencies overlap

  // ---- Q fragments (B operand of S^T = K Q^T): query qi, dims ks*16 + hf*8 .. +8
  bf16x8 qf[8];
  {
    // paged batches: the Q Cache rows of this wave's queries lie on at most two pages
    PagePair qpages = {0, 0, 0};
    if constexpr (PAGED)
      if (a.is_lazy || a.write_q)
        qpages = load_page_pair(pg.q, max(min(__builtin_amdgcn_readfirstlane(wrow0), len - 1) - sm.vis_start, 0) >> 6, a.lv.pt_q_stride);
    const char* qp = pf_q_row<PAGED>(a, sm, rb, qpages, h, min(qi, len - 1));
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + (ks * 16 + hf * 8) * 2));
    // Q Cache write (ordinary layer followed by a lazy one): the span rows of Q, straight from the
    // fragments this lane holds (the two lane halves of a row write alternate 16-byte pieces).
    if (a.write_q && qi < len && qi >= sm.vis_start && qi < sm.vis_start + sm.vis_len) {
      const int qr = qi - sm.vis_start;
      char* qc = a.lv.q_cache + (PAGED ? qpages.row(qr, h, a.n_heads) : rb.q + qr) * ROWB;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) *(uint4*)(qc + (ks * 16 + hf * 8) * 2) = __builtin_bit_cast(uint4, qf[ks]);
    }
  }


  // per-lane LDS read offsets that do not depend on the tile
  int k_off[8];  // K fragment of k-step ks: row l32 (+32 jb), logical chunk ks*2 + hf
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_off[ks] = l32 * ROWB + (((ks * 2 + hf) ^ (l32 & 15)) * 16);
  const int vq = (lane & 15) >> 2;
  const int v_base = (hf * 4 + vq) * ROWB + (l32 >> 4) * 32 + (lane & 3) * 8;
  int v_off[4];  // V fragment of output block db: chunk group db ^ (row & 3)
#pragma unroll
  for (int db = 0; db < 4; ++db) v_off[db] = v_base + ((db ^ vq) * 64);

  // ---- cache writes, fused: the key tiles at or after q0 hold exactly this workgroup's own rows.
  // Once such a tile is visible in LDS every thread copies a share of it to the K and V caches
  // (16-byte pieces, swizzle undone).  A lazy layer stores text rows only, moved down by vis_len
  // behind the span; its span rows in LDS are the anchor layer's and are not stored again.
  // Paged batches: a stored tile is one page of positions (its V rows, an ordinary layer's K rows, a lazy
  // layer's K rows ahead of the span); a lazy layer's K rows behind the span, moved down by vis_len, lie
  // on at most two pages of the text pool.  All fetched by scalar loads before the tile loop.
  struct StorePages {
    int v, k_pos;
    PagePair k_text;
  };
  auto store_pages = [&](int t) -> StorePages {
    StorePages sp = {0, 0, {0, 0, 0}};
    if constexpr (PAGED) {
      const int tt = min(t, n_tiles - 1);
      sp.v = uniform_load(pg.seq + tt);
      if (!a.is_lazy) {
        sp.k_pos = uniform_load(pg.k + tt);
      } else if (!a.inherit_all && a.lv.pt_k_stride > 0) {
        sp.k_pos = uniform_load(pg.k + min(tt, a.lv.pt_k_stride - 1));
        sp.k_text = load_page_pair(pg.k, max(max(tt * BN, sm.vis_start + sm.vis_len) - sm.vis_len, 0) >> 6, a.lv.pt_k_stride);
      }
    }
    return sp;
  };
  const int t_own = q0 / BN;   // the workgroup's own rows are key tiles t_own and t_own + 1
  const StorePages sp_a = store_pages(t_own), sp_b = store_pages(t_own + 1);
  auto store_tile_to_caches = [&](int t) {
    const char* kb = lds + (t % STAGES) * STAGE;
    const char* vb = kb + TILE;
    const int k0 = t * BN;
    char* kdst = a.lv.k_own + rb.k * ROWB;
    char* vdst = a.lv.v_own + rb.v * ROWB;
    const StorePages sp = t == t_own ? sp_a : sp_b;
    const int s0 = sm.vis_start, s1 = sm.vis_start + sm.vis_len;
    // row index of a row of this (sequence, head) in the region: run of rows, or page by page
    auto v_row = [&](int pos) -> int64_t {
      if constexpr (PAGED) return ((int64_t)sp.v * a.n_heads + h) * kPageRows + (pos & (kPageRows - 1));
      else return pos;
    };
    auto k_row = [&](int row, int pos) -> int64_t {   // row: where position pos is kept (pos, or pos - vis_len)
      if constexpr (PAGED) {
        if (a.is_lazy && pos >= s1) return sp.k_text.row(row, h, a.n_heads);
        return ((int64_t)sp.k_pos * a.n_heads + h) * kPageRows + (row & (kPageRows - 1));
      } else {
        return row;
      }
    };
#pragma unroll
    for (int p = 0; p < BN * 16 / (NW * 64); ++p) {
      const int idx = p * (NW * 64) + tid;
      const int r = idx >> 4, cp = idx & 15;  // row in tile, physical chunk
      const int pos = k0 + r;
      if (pos < len) {
        const uint4 vv = *(const uint4*)(vb + r * ROWB + cp * 16);
        *(uint4*)(vdst + v_row(pos) * ROWB + ((cp ^ ((r & 3) << 2)) * 16)) = vv;
        const bool in_span = a.is_lazy && pos >= s0 && pos < s1;
        if (!in_span) {
          const int row = (a.is_lazy && pos >= s1) ? pos - sm.vis_len : pos;
          const uint4 kv = *(const uint4*)(kb + r * ROWB + cp * 16);
          *(uint4*)(kdst + k_row(row, pos) * ROWB + ((cp ^ (r & 15)) * 16)) = kv;
        }
      }
    }
  };

  for (int t = 0; t < n_tiles; ++t) {
    // This wave's part of tile t has landed; after the barrier the whole tile is visible and every
    // wave is done with tile t-1, whose buffer is refilled next.
    wait_vmcnt<0>();
    __syncthreads();
    if (t + 1 < n_tiles) {
      if constexpr (PAGED)
        if (((t + 1) & 63) == 0) {
          pages_cur = pages_next;
          pages_next = fetch_pages(((t + 1) >> 6) + 1);
        }
      load_tile(t + 1, page_of_tile(t + 1));
    }
    const int k0 = t * BN;
    if (k0 >= q0) store_tile_to_caches(t);
    // wave-uniform: otherwise every key of the tile is above the diagonal, or (last query tile of a prompt
    // whose length is not a multiple of 128) the wave has no query row at all and only helps with the tiles
    if (k0 <= wrow0 + 31 && wrow0 < len) {
      const char* kb = lds + (t % STAGES) * STAGE;
      const char* vb = kb + TILE;
      f32x16 s[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[jb][r] = 0.f;
      {  // S^T = K Q^T, K fragments prefetched 4 MFMAs ahead
        bf16x8 kf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) kf[i] = *(const bf16x8*)(kb + k_off[i >> 1] + (i & 1) * 32 * ROWB);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qf[i >> 1], s[i & 1], 0, 0, 0);
          if (i + 4 < 16) kf[i & 3] = *(const bf16x8*)(kb + k_off[(i + 4) >> 1] + ((i + 4) & 1) * 32 * ROWB);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA ...
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // ... then the LDS read four steps ahead
        }
      }
      // The softmax section runs at raised wave priority and the matrix sections at the base one: the
      // SIMD then issues this wave's vector work ahead of the other workgroup's matrix instructions,
      // which keeps both pipes fed (measured 4 % faster than equal priorities).
      __builtin_amdgcn_s_setprio(3);
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
      {
        bf16x8 vf[4];
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) vf[i] = lds_read_tr8(vb + v_off[i & 3] + (i >> 2) * 16 * ROWB, vb + v_off[i & 3] + ((i >> 2) * 16 + 8) * ROWB);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i & 3], pb[i >> 2], o[i & 3], 0, 0, 0);
          if (i + 4 < 16) vf[i & 3] = lds_read_tr8(vb + v_off[i & 3] + ((i + 4) >> 2) * 16 * ROWB, vb + v_off[i & 3] + (((i + 4) >> 2) * 16 + 8) * ROWB);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
      }
    }
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

hipError_t launch_prefill_mfma_bf16_d128(const PrefillArgs& a, hipStream_t stream, KernelTimer* timer) {
  static std::atomic<unsigned long long> attr_set{0}, attr_set_paged{0};
  constexpr int lds_bytes = pf::STAGES * pf::STAGE;
  const bool paged = (a.lv.flags & LV_PAGED) != 0;
  if (hipError_t e = paged ? ensure_dynamic_lds((const void*)prefill_mfma_kernel<true>, lds_bytes, attr_set_paged)
                           : ensure_dynamic_lds((const void*)prefill_mfma_kernel<false>, lds_bytes, attr_set);
      e != hipSuccess)
    return e;
  const int n_qt = (a.max_len + pf::BM - 1) / pf::BM;
  const int nbh = a.batch * a.n_heads;
  if (timer) timer->begin(stream);
  if (paged) hipLaunchKernelGGL(prefill_mfma_kernel<true>, dim3(n_qt * nbh), dim3(pf::NW * 64), lds_bytes, stream, a, n_qt, (nbh % 8 == 0) ? 1 : 0);
  else hipLaunchKernelGGL(prefill_mfma_kernel<false>, dim3(n_qt * nbh), dim3(pf::NW * 64), lds_bytes, stream, a, n_qt, (nbh % 8 == 0) ? 1 : 0);
  if (timer) timer->end(stream);
  return hipGetLastError();
}

}  // namespace qc
