// Internal interface between the host-side C ABI (qc_api.cpp) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <utility>
#include <vector>

namespace qc {

// Per-sequence metadata rows in the arena's meta region: meta[row * max_batch + b].  The region holds
// META_BLOCKS such blocks of META_ROWS rows: block 0 describes the prompts as given, block 1 the
// prompts as the layers after a token-pruning boundary see them.
enum { META_TOK0 = 0, META_LEN0 = 1, META_VIS_START = 2, META_VIS_LEN = 3, META_ROWS = 4, META_BLOCKS = 2 };

// Capacity rows of the meta region (per-sequence capacities): meta layout is META_BLOCKS blocks of
// META_ROWS rows, META_COUNTER_WORDS counter words, then CAPS_ROWS rows of max_batch integers.
enum { CAP_SEQ = 0, BASE_SEQ = 1, CAP_TEXT = 2, BASE_TEXT = 3, CAP_VIS = 4, BASE_VIS = 5, CAPS_ROWS = 6 };
enum { META_COUNTER_WORDS = 64 };
// LayerView::flags
enum { LV_RAGGED = 1,    // capacities are per sequence: row bases come from the capacity rows
       LV_K_TEXT = 2,    // k_own holds text rows only (lazy layer, Visual Lazy Attention)
       LV_Q_VIS = 4,     // q_cache holds visual rows only (Visual Lazy Attention)
       LV_LATE = 8,      // meta points at block 1 (layer behind a pruning boundary)
       LV_PAGED = 16 };  // rows live on pages of kPageRows rows; the page lists below say which

// Paged batches: every region is [page][head][kPageRows][D]; a sequence holds a list of pages per pool
// (positions: V rows, K rows of ordinary layers, Q Cache rows under Global Lazy Attention; text rows: K rows
// of lazy layers; visual rows: Q Cache rows under Visual Lazy Attention).  Row r of head h sits at row
// index (list[r / kPageRows] * H + h) * kPageRows + r % kPageRows of its region.
enum { kPageRows = 64, kMaxPagesPerSeq = 1024 };

// Device addresses of everything one layer call touches.  Cache regions are
// [batch][head][cap][D] with the element type of the configuration (with per-sequence capacities:
// sequence after sequence, each [head][cap_b][D]).
struct LayerView {
  char* k_own;            // this layer's K rows
  char* v_own;            // this layer's V rows
  const char* k_anchor;   // K rows of the block's first layer (lazy layers only, else nullptr)
  char* q_cache;          // Q Cache rows (nullptr if the call neither reads nor writes it)
  const int32_t* meta;    // int32 [META_ROWS][max_batch]
  int32_t cap_k;          // row capacity per (b, h) of k_own
  int32_t cap_v;
  int32_t cap_k_anchor;
  int32_t cap_q;
  int32_t max_batch;
  int32_t flags;
  // page lists (LV_PAGED): sequence b's list of a pool starts at pt_x + b * pt_x_stride
  const int32_t* pt_seq;  // positions: v_own, k_anchor, k_own of an ordinary layer
  const int32_t* pt_k;    // the pool k_own's rows live in (pt_seq, or the text-row lists in a lazy layer)
  const int32_t* pt_q;    // the pool q_cache's rows live in
  int32_t pt_seq_stride, pt_k_stride, pt_q_stride;
};

struct PrefillArgs {
  LayerView lv;
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int64_t token_stride;   // elements
  int64_t head_stride;    // elements
  int32_t batch, n_heads, head_dim;
  int32_t is_lazy;        // substitute span rows of q/k, store text rows of k only
  int32_t write_q;        // store span rows of q into the Q Cache
  int32_t inherit_all;    // Global Lazy Attention: the inherited span is the whole prompt, [0, len)
  int32_t max_len;        // longest prompt in the batch
  float scale;            // softmax scale (already resolved, > 0)
};

struct DecodeArgs {
  LayerView lv;
  const void* q;          // [batch][H][D]
  const void* k;
  const void* v;
  void* out;
  float* workspace;       // [batch][H][max_chunks][D + 2] partial (o, m, l)
  const int32_t* generated_dev;  // nullptr, or where the number of completed decode steps lives in device memory
  int32_t batch, n_heads, head_dim;
  int32_t is_lazy;
  int32_t generated;      // decode steps completed before this one: len_b = len0_b + generated
  int32_t max_len;        // longest len_b in the batch (before this step)
  int32_t chunk_keys;     // key positions per workgroup
  int32_t max_chunks;     // ceil((max_len + 1) / chunk_keys)
  float scale;
  // Small batches carry their per-sequence integers in the kernel arguments (one dependent memory
  // round trip less per launch, which matters for launches of a few microseconds).
  enum { kInlineSeqs = 8 };
  int32_t inline_meta;                 // 1: the arrays below are valid (batch <= kInlineSeqs)
  int32_t len0_inline[kInlineSeqs];
  int32_t vis_start_inline[kInlineSeqs];
  int32_t vis_len_inline[kInlineSeqs];
};

struct SelectArgs {       // last-row attention of one ordinary layer (lazy-block selection, Eq. 3)
  LayerView lv;
  const void* q_last;     // [batch][H][D]: query of each sequence's last token
  float* scores;          // workspace: [batch][H][score_stride]
  float* row_stats;       // workspace: [batch][H][2] = (max, sum) of each score row
  float* probs;           // out: [batch][probs_stride], positions 0..len-1
  int64_t probs_stride;
  int32_t score_stride;
  int32_t batch, n_heads, head_dim;
  int32_t generated;
  float scale;
};

struct JsChunk {          // by-value payload of the similarity kernel: row lengths of up to N samples
  enum { N = 64 };
  int32_t len[N];
};

struct ProjectSegs {      // rows to project: contiguous token ranges, in order (by value in the kernel arguments)
  enum { N = 128 };
  int32_t tok_start[N];   // first token index of the range in the packed tensors
  int32_t count[N];
  int32_t pos_start[N];   // position of that token inside its sequence
  int32_t n;
};

struct ProjectArgs {
  const void* x;          // [tokens][d_model] bf16, row stride x_stride elements
  const void* w[2];       // W_Q, W_K: [H*D] rows of d_model bf16, row stride w_stride elements
  void* out[2];           // q, k: element (t, h, d) at t*token_stride + h*head_stride + d
  int64_t x_stride, w_stride, token_stride, head_stride;
  int32_t d_model, n_heads, head_dim;
  float rope_theta;       // 0: no rotary embedding
  double log2_theta;
  ProjectSegs segs;
};

// What a decode call needs in addition under Global Lazy Attention.  Kept out of DecodeArgs so that
// the kernel arguments of the ordinary path stay as small as they were (a few-microsecond launch
// notices an extra argument load).
struct DecodeGlaArgs {
  float* scores;          // [batch][H][score_stride] scaled scores of the current step
  int32_t score_stride;   // floats per (sequence, head) in `scores`
  int32_t mode;           // 0: no Global Lazy Attention work in this call; 1: first layer of a block:
                          // store the score of every position and the query at row len of the Q Cache;
                          // 2: lazy layer: take the scores from `scores` instead of reading keys
};

struct PruneChunk {       // by-value payload of the survivor selection kernel: up to N sequences
  enum { N = 64 };
  int32_t tok0[N];        // first packed token index of the sequence
  int32_t len[N];
  int32_t vis_start[N];
  int32_t vis_len[N];
  int32_t keep[N];
  int32_t out0[N];        // first entry of the sequence in the row map
};

struct MoveChunk {        // by-value payload of the row relocation kernel: up to N regions
  enum { N = 32 };
  int64_t src[N], dst[N];             // byte offsets of head 0's rows inside the arena
  int64_t src_stride[N], dst_stride[N];   // bytes from one head's rows to the next
  int32_t rows[N];                    // rows per head to move
  int32_t arena[N];                   // 0: K/V arena, 1: Q arena
};

struct TableChunk {       // by-value payload of the page-list upload kernel: up to N entries
  enum { N = 128 };
  int32_t at[N];          // index into the page-list buffer
  int32_t page[N];
};

struct MetaChunk {        // by-value payload of the metadata upload kernel: up to ROWS rows of N sequences
  enum { N = 64, ROWS = 6 };
  int32_t v[ROWS][N];
};

// Optional instrumentation: HIP events recorded on the call's stream around the dominant kernel
// of a layer call (prefill: the attention kernel; decode: the streaming kernel, not the merge).
struct KernelTimer {
  static constexpr size_t kMaxPairs = 131072;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
  size_t used = 0;
  int64_t dropped = 0;
  bool open = false;
  void begin(hipStream_t s) {
    open = false;
    if (used == pool.size()) {
      if (pool.size() >= kMaxPairs) { ++dropped; return; }
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) { ++dropped; return; }
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); ++dropped; return; }
      pool.emplace_back(a, b);
    }
    open = hipEventRecord(pool[used].first, s) == hipSuccess;
  }
  void end(hipStream_t s) {
    if (open && hipEventRecord(pool[used].second, s) == hipSuccess) ++used;
    open = false;
  }
  // Waits for the recorded events, sums their durations and starts over.
  hipError_t read(double* total_ms, int64_t* launches) {
    *total_ms = 0.0;
    *launches = 0;
    for (size_t i = 0; i < used; ++i) {
      hipError_t e = hipEventSynchronize(pool[i].second);
      float ms = 0.f;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, pool[i].first, pool[i].second);
      if (e != hipSuccess) { used = 0; return e; }
      *total_ms += ms;
      ++*launches;
    }
    used = 0;
    dropped = 0;
    return hipSuccess;
  }
  ~KernelTimer() {
    for (auto& p : pool) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
  }
};

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the
// kernel).  `done` holds one bit per device; concurrent callers at worst both set the same value.
inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) done.fetch_or(1ull << dev, std::memory_order_release);
  return e;
}

hipError_t launch_fill_zero(void* dev, size_t bytes, hipStream_t stream);
hipError_t launch_counter_update(int32_t* counter, int32_t value, int32_t add, hipStream_t stream);
hipError_t launch_meta_upload(int32_t* meta_dev, int32_t max_batch, int32_t first, int32_t count, int32_t rows,
                              const MetaChunk& chunk, hipStream_t stream);
hipError_t launch_table_upload(int32_t* tables, int32_t count, const TableChunk& chunk, hipStream_t stream);
hipError_t launch_move_rows(void* arena0, void* arena1, int32_t row_bytes, int32_t n_heads, int32_t count,
                            const MoveChunk& chunk, hipStream_t stream);
hipError_t launch_prefill(const PrefillArgs& a, int dtype, hipStream_t stream, KernelTimer* timer);
// Size of the library's own decode scratch array (one per GPU, held until the process ends).
constexpr size_t kStaticScratchBytes = 4u << 20;
// Device address and size of that array on the current device; allocates nothing.
hipError_t decode_static_scratch(void** ptr, size_t* bytes);
hipError_t launch_decode(const DecodeArgs& a, const DecodeGlaArgs& g, int dtype, hipStream_t stream, KernelTimer* timer);
hipError_t launch_last_row_attention(const SelectArgs& a, int dtype, int max_len, hipStream_t stream);
hipError_t launch_js(const float* pm, const float* pn, int64_t stride, int first, int count, const JsChunk& c,
                     float* js_out, hipStream_t stream);
hipError_t launch_mean(const float* x, int n, float* out, hipStream_t stream);
hipError_t launch_prune_select(const float* scores, int64_t stride, int first, int count, const PruneChunk& c,
                               int32_t* row_map, hipStream_t stream);
hipError_t launch_gather_rows(const void* src, int64_t src_stride, const int32_t* row_map, int64_t n_rows,
                              int64_t row_bytes, void* dst, int64_t dst_stride, hipStream_t stream);
hipError_t launch_project_qk(const ProjectArgs& a, int rows, hipStream_t stream);
hipError_t launch_project_qk_skinny(const ProjectArgs& a, int n_rows, hipStream_t stream);

}  // namespace qc
