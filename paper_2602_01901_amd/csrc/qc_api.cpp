// Host side of the C ABI declared in include/qcache.h: validation, lazy-block bookkeeping,
// arena address arithmetic and kernel dispatch.  All arithmetic of the method runs in the
// kernels; this file only decides which rows live where (integers).
#include "qcache.h"

#include <algorithm>
#include <array>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "qc_internal.h"

namespace {

thread_local char g_err[256] = "";

qc_status fail(qc_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Config {
  int32_t N = 0, H = 0, D = 0, dtype = 0;
  int32_t max_batch = 0, max_seq = 0, max_vis = 0, max_text = 0;
  int32_t mode = QC_VLA;
  // Smaller regions for the layers behind a pruning boundary fixed at creation: layers >= late_from
  // hold at most max_seq_late positions per sequence (late_from = 0: no such boundary).
  int32_t late_from = 0, max_seq_late = 0;
  std::vector<uint8_t> lazy;
  std::vector<int32_t> anchor;  // anchor[l] = first layer of l's block (l itself if not lazy)

  int e() const { return dtype == QC_BF16 ? 2 : 4; }
  bool gla() const { return mode == QC_GLA; }
  int64_t cap_v(int l) const { return (late_from > 0 && l >= late_from) ? max_seq_late : max_seq; }
  int64_t cap_k(int l) const { return lazy[l] ? (gla() ? 0 : max_text) : cap_v(l); }
  int64_t cap_q() const { return gla() ? max_seq : max_vis; }
  // An ordinary layer stores queries in the Q Cache exactly when the next layer is lazy.
  bool writes_q(int l) const { return !lazy[l] && l + 1 < N && lazy[l + 1]; }
  int64_t k_layer_bytes(int l) const { return (int64_t)max_batch * H * cap_k(l) * D * e(); }
  int64_t v_layer_bytes(int l) const { return (int64_t)max_batch * H * cap_v(l) * D * e(); }
  int64_t off_k(int l) const {
    int64_t o = 0;
    for (int i = 0; i < l; ++i) o += k_layer_bytes(i);
    return o;
  }
  int64_t off_v(int l) const {
    int64_t o = off_k(N);
    for (int i = 0; i < l; ++i) o += v_layer_bytes(i);
    return o;
  }
  int64_t off_meta() const { return round_up(off_v(N), 256); }
  // after the per-sequence integers: 256 bytes of device-side counters (int32 [0] = decode steps
  // completed, as maintained for replayed decode graphs)
  int64_t off_counters() const { return off_meta() + (int64_t)qc::META_BLOCKS * qc::META_ROWS * 4 * max_batch; }
  // then the capacity rows (per-sequence capacities; zero otherwise)
  int64_t off_caps() const { return off_counters() + 4 * qc::META_COUNTER_WORDS; }
  int64_t meta_bytes() const {
    return round_up((int64_t)qc::META_BLOCKS * qc::META_ROWS * 4 * max_batch + 4 * qc::META_COUNTER_WORDS +
                        (int64_t)qc::CAPS_ROWS * 4 * max_batch, 256);
  }
  int64_t kv_bytes() const { return off_meta() + meta_bytes(); }
  int64_t q_bytes() const { return (int64_t)max_batch * H * cap_q() * D * e(); }
  int64_t row_bytes() const { return (int64_t)D * e(); }
  // Paged batches: page lists per sequence and pool (POOL_SEQ positions, POOL_TEXT text rows of lazy layers,
  // POOL_VIS Q Cache rows under Visual Lazy Attention).  The last two exist only where rows are kept in them.
  int n_lazy() const { int n = 0; for (auto f : lazy) n += f ? 1 : 0; return n; }
  bool pool_used(int pool) const { return pool == 0 || (!gla() && n_lazy() > 0); }
  int64_t pool_pages(int pool) const {
    if (!pool_used(pool)) return 0;
    return (int64_t)max_batch * ((pool == 0 ? max_seq : pool == 1 ? max_text : max_vis) / qc::kPageRows);
  }
  // entries of one sequence's list = pages it may hold at most: the whole pool, up to what the kernels stage
  int32_t pool_stride(int pool) const { return (int32_t)std::min<int64_t>(pool_pages(pool), qc::kMaxPagesPerSeq); }
  int64_t table_off(int pool) const {     // first entry of the pool's lists in the page-list buffer
    int64_t o = 0;
    for (int i = 0; i < pool; ++i) o += (int64_t)max_batch * pool_stride(i);
    return o;
  }
  int64_t table_entries() const { return table_off(3); }
  bool pageable() const {
    return late_from == 0 && max_seq % qc::kPageRows == 0 &&
           (gla() || (max_text % qc::kPageRows == 0 && max_vis % qc::kPageRows == 0));
  }
  bool same(const Config& o) const {
    return N == o.N && H == o.H && D == o.D && dtype == o.dtype && max_batch == o.max_batch &&
           max_seq == o.max_seq && max_vis == o.max_vis && max_text == o.max_text && mode == o.mode &&
           late_from == o.late_from && max_seq_late == o.max_seq_late &&
           lazy == o.lazy;
  }
};

// Smallest key chunk a decode workgroup takes; fixes the workspace size.
constexpr int kMinChunkKeys = 64;

bool parse_config(const qc_config* c, Config* out) {
  if (!c || !c->lazy_mask) return false;
  if (c->n_layers < 1 || c->n_heads < 1 || c->max_batch < 1 || c->max_seq < 1 || c->max_vis < 0 ||
      c->max_text < 0)
    return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->dtype != QC_F32 && c->dtype != QC_BF16) return false;
  if ((c->mode != QC_VLA && c->mode != QC_GLA) || c->reserved != 0) return false;
  if (c->prune_before_layer != 0 &&
      (c->prune_before_layer < 1 || c->prune_before_layer >= c->n_layers || c->lazy_mask[c->prune_before_layer] ||
       c->max_seq_late < 1 || c->max_seq_late > c->max_seq))
    return false;
  if (c->prune_before_layer == 0 && c->max_seq_late != 0) return false;
  if (c->max_vis > c->max_seq || c->max_text > c->max_seq) return false;
  if (c->lazy_mask[0]) return false;
  out->N = c->n_layers;
  out->H = c->n_heads;
  out->D = c->head_dim;
  out->dtype = c->dtype;
  out->max_batch = c->max_batch;
  out->max_seq = c->max_seq;
  out->max_vis = c->max_vis;
  out->max_text = c->max_text;
  out->mode = c->mode;
  out->late_from = c->prune_before_layer;
  out->max_seq_late = c->max_seq_late;
  out->lazy.assign(c->lazy_mask, c->lazy_mask + c->n_layers);
  for (auto& f : out->lazy) f = f ? 1 : 0;
  out->anchor.resize(out->N);
  for (int l = 0; l < out->N; ++l) out->anchor[l] = out->lazy[l] ? out->anchor[l - 1] : l;
  return true;
}

enum Phase { PH_EMPTY = 0, PH_RESET = 1, PH_PREFILL = 2, PH_READY = 3, PH_DECODE = 4 };

}  // namespace

struct qc_kvcache {
  Config cfg;
  char* arena = nullptr;
  int phase = PH_EMPTY;
  int32_t batch = 0;
  int32_t next_layer = 0;
  int32_t generated = 0;
  std::vector<int32_t> vis_start, vis_len, len0, tok0;
  // Token pruning: layers >= first_late see sequence b with vis_len1[b] visual tokens and len1[b]
  // prompt tokens, packed from tok1[b] (the last two known once the first such layer has run).
  int32_t first_late = -1;
  int32_t units = 256;    // compute units of the device the handle was created on
  bool late_known = false;
  std::vector<int32_t> vis_len1, len1, tok1;
  bool late(int layer) const { return first_late >= 0 && layer >= first_late; }
  int32_t vis_len_of(int layer, int b) const { return late(layer) ? vis_len1[b] : vis_len[b]; }
  int32_t len_of(int layer, int b) const { return late(layer) ? len0[b] - vis_len[b] + vis_len1[b] : len0[b]; }
  // Per-sequence capacities (qc_reset_ragged): rows sequence b may use, and where they start.
  bool ragged = false;
  bool paged = false;     // rows on pages (qc_reset_paged), see below
  std::vector<int32_t> cap_seq, cap_text, base_seq, base_text, base_vis;
  int64_t cap_seq_of(int b) const { return ragged ? cap_seq[b] : cfg.max_seq; }
  // positions sequence b may reach in `layer` (smaller behind a configured pruning boundary; on a paged
  // batch as far as its page list reaches: the pools decide before that)
  int64_t cap_of(int layer, int b) const {
    if (paged) return (int64_t)cfg.pool_stride(0) * qc::kPageRows;
    return ragged ? cap_seq[b] : cfg.cap_v(layer);
  }
  int64_t cap_text_of(int b) const {
    if (paged) return cfg.pool_used(1) ? (int64_t)cfg.pool_stride(1) * qc::kPageRows : (int64_t)1 << 40;
    return ragged ? cap_text[b] : cfg.max_text;
  }
  int64_t longest_cap() const {
    int64_t m = ragged ? 0 : cfg.max_seq;
    if (ragged) for (int b = 0; b < batch; ++b) m = std::max<int64_t>(m, cap_seq[b]);
    // paged: a sequence has no capacity of its own; a recorded launch covers max_seq positions, or, once a
    // sequence is longer than that, the next multiple of max_seq above the longest one (and is recorded
    // again when a sequence outgrows it)
    if (paged)
      for (int b = 0; b < batch; ++b)
        if (live[b]) m = std::max<int64_t>(m, ((int64_t)len0[b] + steps_of(b) + 1 + cfg.max_seq - 1) / cfg.max_seq * cfg.max_seq);
    return m;
  }
  // Paged batches (qc_reset_paged): rows live on pages of kPageRows rows.  pages[pool][b] = the pages slot b
  // holds, in row order; free_pages[pool] ascending (the lowest free page is handed out first); `tables` is
  // the caller's device buffer the kernels read the lists from.
  int32_t* tables = nullptr;
  std::vector<std::vector<int32_t>> pages[3];
  std::vector<int32_t> free_pages[3];
  bool slots() const { return ragged || paged; }   // sequences may join and leave
  // Slots of the batch (qc_seq_join / qc_seq_leave): live[b] = slot b holds a sequence; joining[b] =
  // it is (to be) filled by the prefill pass that is open or about to open; joined_at[b] = value of
  // `generated` when its prefill pass ended.  Without joins and leaves every slot is live, every
  // sequence belongs to the one pass after qc_reset and joined_at is 0 throughout.
  std::vector<uint8_t> live, joining;
  std::vector<int32_t> joined_at;
  bool join_pass = false;   // the open (or pending) prefill pass fills joining slots beside settled sequences
  bool settled(int b) const { return live[b] && !joining[b]; }
  int32_t steps_of(int b) const { return generated - joined_at[b]; }
  // value the kernels add the step counter to: prompt length less the steps that ran before the sequence joined
  int32_t len_base(int layer, int b) const { return live[b] ? len_of(layer, b) - joined_at[b] : kFreeSlotLen; }
  bool all_live() const { for (int b = 0; b < batch; ++b) if (!live[b]) return false; return true; }
  static constexpr int32_t kFreeSlotLen = -(1 << 30);   // a free slot's length stays negative for any step count
  // Value the device-side step counter holds once everything enqueued so far has run (-1: not set).
  int64_t dev_generated = -1;
  bool timing = false;
  qc::KernelTimer prefill_timer, decode_timer, decode_shared_timer;
  const void* score_workspace = nullptr;  // workspace the current block's scores were written to (GLA)
};

struct qc_qcache {
  Config cfg;
  char* arena = nullptr;
  int32_t owner = -1;
};

struct qc_decode_graph {
  qc_kvcache* kv = nullptr;
  qc_qcache* qc = nullptr;
  hipGraphExec_t exec = nullptr;
  int32_t batch = 0, first_late = -1;
  bool ragged = false;                   // recorded with per-sequence capacities
  bool paged = false;                    // recorded on a paged batch
  int64_t covered = 0;                   // positions the recorded launch grids cover
  int32_t final_owner = -1;              // Q Cache owner after a step (Global Lazy Attention)
  const void* score_workspace = nullptr;
};

extern "C" {

const char* qc_status_str(qc_status s) {
  switch (s) {
    case QC_OK: return "QC_OK";
    case QC_EINVAL: return "QC_EINVAL";
    case QC_EORDER: return "QC_EORDER";
    case QC_ECAPACITY: return "QC_ECAPACITY";
    case QC_EDEVICE: return "QC_EDEVICE";
  }
  return "QC_UNKNOWN";
}

const char* qc_last_error(void) { return g_err; }

size_t qc_kv_arena_bytes(const qc_config* cfg) {
  Config c;
  return parse_config(cfg, &c) ? (size_t)c.kv_bytes() : 0;
}

size_t qc_q_arena_bytes(const qc_config* cfg) {
  Config c;
  return parse_config(cfg, &c) ? (size_t)c.q_bytes() : 0;
}

// Decode workspace: the split partials, then (Global Lazy Attention only) one float per position
// of every (sequence, head): the scaled scores of the block whose first layer ran last.
// The score rows are read and written 16 bytes at a time in runs of 8 positions: the row stride is
// max_seq rounded up to 8 floats and the region starts 256-byte aligned.
static int64_t partial_bytes(const Config& c) {
  int64_t chunks = (c.max_seq + kMinChunkKeys - 1) / kMinChunkKeys;
  // a call never uses more than 1024 + batch*H partial slots, whatever the lengths (the key axis is
  // split only until about 1024 workgroups exist): that bound also covers per-sequence capacities
  // beyond max_seq
  int64_t slots = std::max<int64_t>((int64_t)c.max_batch * c.H * chunks, 1024 + (int64_t)c.max_batch * c.H);
  int64_t b = slots * (c.D + 2) * 4;
  return c.gla() ? round_up(b, 256) : b;
}
static int64_t score_stride(const Config& c) { return round_up(c.max_seq, 8); }
static int64_t score_bytes(const Config& c) { return c.gla() ? (int64_t)c.max_batch * c.H * score_stride(c) * 4 : 0; }

size_t qc_decode_workspace_bytes(const qc_config* cfg) {
  Config c;
  if (!parse_config(cfg, &c)) return 0;
  return (size_t)(partial_bytes(c) + score_bytes(c));
}

// Compute units of the current device (cached per device; 256 if the runtime does not say).
static int compute_units() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

qc_status qc_kvcache_create(const qc_config* cfg, void* dev_arena, size_t arena_bytes, qc_kvcache** out) {
  if (!out) return fail(QC_EINVAL, "qc_kvcache_create: out is null");
  *out = nullptr;
  Config c;
  if (!parse_config(cfg, &c)) return fail(QC_EINVAL, "qc_kvcache_create: invalid configuration");
  if (!dev_arena || ((uintptr_t)dev_arena & 255)) return fail(QC_EINVAL, "qc_kvcache_create: arena null or not 256-byte aligned");
  if ((int64_t)arena_bytes < c.kv_bytes())
    return fail(QC_ECAPACITY, "qc_kvcache_create: arena holds %zu bytes, %lld needed", arena_bytes, (long long)c.kv_bytes());
  qc_kvcache* kv = new (std::nothrow) qc_kvcache;
  if (!kv) return fail(QC_ECAPACITY, "qc_kvcache_create: out of host memory");
  kv->cfg = c;
  kv->arena = (char*)dev_arena;
  kv->units = compute_units();   // asked once, here: not from inside a call that a caller may be capturing
  *out = kv;
  return QC_OK;
}

qc_status qc_qcache_create(const qc_config* cfg, void* dev_arena, size_t arena_bytes, qc_qcache** out) {
  if (!out) return fail(QC_EINVAL, "qc_qcache_create: out is null");
  *out = nullptr;
  Config c;
  if (!parse_config(cfg, &c)) return fail(QC_EINVAL, "qc_qcache_create: invalid configuration");
  if (c.q_bytes() > 0 && (!dev_arena || ((uintptr_t)dev_arena & 255)))
    return fail(QC_EINVAL, "qc_qcache_create: arena null or not 256-byte aligned");
  if ((int64_t)arena_bytes < c.q_bytes())
    return fail(QC_ECAPACITY, "qc_qcache_create: arena holds %zu bytes, %lld needed", arena_bytes, (long long)c.q_bytes());
  qc_qcache* q = new (std::nothrow) qc_qcache;
  if (!q) return fail(QC_ECAPACITY, "qc_qcache_create: out of host memory");
  q->cfg = c;
  q->arena = (char*)dev_arena;
  *out = q;
  return QC_OK;
}

void qc_kvcache_destroy(qc_kvcache* kv) { delete kv; }
void qc_qcache_destroy(qc_qcache* qc) { delete qc; }

struct PagedInit {
  const uint8_t* present;   // batch flags (0 = the slot starts free), or null: every slot holds a sequence
  void* tables;             // device buffer for the page lists
  size_t table_bytes;
};

static qc_status reset_impl(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                            const int32_t* vis_len, const int32_t* cap_seq, const int32_t* cap_text,
                            int32_t zero_fill, void* stream, const PagedInit* paged = nullptr) {
  if (!kv || !qc) return fail(QC_EINVAL, "qc_reset: null handle");
  if (!kv->cfg.same(qc->cfg)) return fail(QC_EINVAL, "qc_reset: K/V cache and Q Cache were created with different configurations");
  if (!vis_start || !vis_len) return fail(QC_EINVAL, "qc_reset: null span arrays");
  const Config& c = kv->cfg;
  if (batch < 1) return fail(QC_EINVAL, "qc_reset: batch %d", batch);
  if (batch > c.max_batch) return fail(QC_ECAPACITY, "qc_reset: batch %d exceeds max_batch %d", batch, c.max_batch);
  const bool ragged = cap_seq != nullptr;
  if (ragged && !cap_text) return fail(QC_EINVAL, "qc_reset_ragged: null capacity array");
  if (paged) {
    if (!c.pageable()) return fail(QC_EINVAL, "qc_reset_paged: the configuration cannot be paged (max_seq, max_text and max_vis must be multiples of %d, max_seq at most %d, no separately sized late layers)", qc::kPageRows, qc::kPageRows * qc::kMaxPagesPerSeq);
    if (!paged->tables || ((uintptr_t)paged->tables & 15)) return fail(QC_EINVAL, "qc_reset_paged: page-list buffer null or not 16-byte aligned");
    if ((int64_t)paged->table_bytes < c.table_entries() * 4) return fail(QC_ECAPACITY, "qc_reset_paged: page-list buffer holds %zu bytes, %lld needed", paged->table_bytes, (long long)c.table_entries() * 4);
  }
  if (ragged && c.late_from > 0) return fail(QC_EINVAL, "qc_reset_ragged: per-sequence capacities cannot be combined with a configuration that sizes the layers behind a pruning boundary separately");
  int64_t sum_seq = 0, sum_text = 0, sum_vis = 0;
  for (int b = 0; b < batch; ++b) {
    if (ragged && cap_seq[b] == 0) continue;
    if (paged && paged->present && !paged->present[b]) continue;
    if (vis_start[b] < 0 || vis_len[b] < 0) return fail(QC_EINVAL, "qc_reset: negative span for sequence %d", b);
    if (paged) {
      if (c.pool_used(2) && vis_len[b] > (int64_t)c.pool_stride(2) * qc::kPageRows) return fail(QC_ECAPACITY, "qc_reset_paged: sequence %d has %d visual tokens, a sequence may hold %lld", b, vis_len[b], (long long)c.pool_stride(2) * qc::kPageRows);
      if ((int64_t)vis_start[b] + vis_len[b] > (int64_t)c.pool_stride(0) * qc::kPageRows) return fail(QC_ECAPACITY, "qc_reset_paged: span of sequence %d exceeds what a sequence may hold", b);
      continue;
    }
    if (!ragged) {
      if (!c.gla() && vis_len[b] > c.max_vis) return fail(QC_ECAPACITY, "qc_reset: sequence %d has %d visual tokens, max_vis %d", b, vis_len[b], c.max_vis);
      if ((int64_t)vis_start[b] + vis_len[b] > c.max_seq) return fail(QC_ECAPACITY, "qc_reset: span of sequence %d exceeds max_seq", b);
      continue;
    }
    if (cap_seq[b] < 8 || cap_seq[b] % 8 || cap_text[b] < 0)
      return fail(QC_EINVAL, "qc_reset_ragged: cap_seq[%d] must be 0 (a free slot) or a positive multiple of 8, cap_text[%d] not negative", b, b);
    if ((int64_t)vis_start[b] + vis_len[b] > cap_seq[b]) return fail(QC_ECAPACITY, "qc_reset_ragged: span of sequence %d exceeds its %d positions", b, cap_seq[b]);
    sum_seq += cap_seq[b];
    sum_text += cap_text[b];
    sum_vis += vis_len[b];
  }
  if (ragged) {
    if (sum_seq > (int64_t)c.max_batch * c.max_seq) return fail(QC_ECAPACITY, "qc_reset_ragged: %lld positions asked for, the arena holds max_batch*max_seq = %lld", (long long)sum_seq, (long long)c.max_batch * c.max_seq);
    if (!c.gla() && sum_text > (int64_t)c.max_batch * c.max_text) return fail(QC_ECAPACITY, "qc_reset_ragged: %lld text rows asked for, the arena holds max_batch*max_text = %lld", (long long)sum_text, (long long)c.max_batch * c.max_text);
    if (!c.gla() && sum_vis > (int64_t)c.max_batch * c.max_vis) return fail(QC_ECAPACITY, "qc_reset_ragged: %lld visual tokens, the Q arena holds max_batch*max_vis = %lld", (long long)sum_vis, (long long)c.max_batch * c.max_vis);
  }
  if (zero_fill) {
    hipError_t e = qc::launch_fill_zero(kv->arena, (size_t)c.kv_bytes(), (hipStream_t)stream);
    if (e == hipSuccess && c.q_bytes() > 0) e = qc::launch_fill_zero(qc->arena, (size_t)c.q_bytes(), (hipStream_t)stream);
    if (e != hipSuccess) return fail(QC_EDEVICE, "qc_reset: %s", hipGetErrorString(e));
  }
  kv->batch = batch;
  kv->vis_start.assign(vis_start, vis_start + batch);
  kv->vis_len.assign(vis_len, vis_len + batch);
  kv->len0.assign(batch, 0);
  kv->tok0.assign(batch, 0);
  kv->phase = PH_RESET;
  kv->next_layer = 0;
  kv->generated = 0;
  kv->score_workspace = nullptr;
  kv->first_late = -1;
  kv->late_known = false;
  kv->dev_generated = -1;
  qc->owner = -1;
  kv->ragged = ragged;
  kv->live.assign(batch, 1);
  kv->joining.assign(batch, 1);
  kv->joined_at.assign(batch, 0);
  kv->join_pass = false;
  kv->paged = paged != nullptr;
  kv->tables = paged ? (int32_t*)paged->tables : nullptr;
  for (int pool = 0; pool < 3; ++pool) {
    kv->pages[pool].assign(paged ? batch : 0, std::vector<int32_t>());
    kv->free_pages[pool].clear();
    if (paged)
      for (int64_t pg = 0; pg < c.pool_pages(pool); ++pg) kv->free_pages[pool].push_back((int32_t)pg);
  }
  if (paged && paged->present)
    for (int b = 0; b < batch; ++b)
      if (!paged->present[b]) {   // free slot: no rows, nothing to fill
        kv->live[b] = kv->joining[b] = 0;
        kv->vis_start[b] = kv->vis_len[b] = 0;
      }
  if (ragged) {
    kv->cap_seq.assign(cap_seq, cap_seq + batch);
    kv->cap_text.assign(cap_text, cap_text + batch);
    kv->base_seq.assign(batch, 0);
    kv->base_text.assign(batch, 0);
    kv->base_vis.assign(batch, 0);
    int64_t next_seq = 0, next_text = 0, next_vis = 0;
    for (int b = 0; b < batch; ++b) {
      if (cap_seq[b] == 0) {   // free slot: no rows, nothing to fill
        kv->live[b] = kv->joining[b] = 0;
        kv->cap_text[b] = kv->vis_start[b] = kv->vis_len[b] = 0;
        continue;
      }
      kv->base_seq[b] = (int32_t)next_seq;
      kv->base_text[b] = c.gla() ? 0 : (int32_t)next_text;   // Global Lazy Attention keeps nothing in these two pools
      kv->base_vis[b] = c.gla() ? 0 : (int32_t)next_vis;
      next_seq += cap_seq[b];
      next_text += cap_text[b];
      next_vis += vis_len[b];
    }
    // the capacity rows the kernels read (after the optional clear above, on the same stream)
    for (int first = 0; first < batch; first += qc::MetaChunk::N) {
      qc::MetaChunk mc;
      memset(&mc, 0, sizeof(mc));
      const int count = batch - first < qc::MetaChunk::N ? batch - first : qc::MetaChunk::N;
      for (int i = 0; i < count; ++i) {
        const int b = first + i;
        mc.v[qc::CAP_SEQ][i] = kv->cap_seq[b];
        mc.v[qc::BASE_SEQ][i] = kv->base_seq[b];
        mc.v[qc::CAP_TEXT][i] = kv->cap_text[b];
        mc.v[qc::BASE_TEXT][i] = kv->base_text[b];
        mc.v[qc::CAP_VIS][i] = kv->vis_len[b];
        mc.v[qc::BASE_VIS][i] = kv->base_vis[b];
      }
      hipError_t e = qc::launch_meta_upload((int32_t*)(kv->arena + c.off_caps()), c.max_batch, first, count, qc::CAPS_ROWS, mc, (hipStream_t)stream);
      if (e != hipSuccess) return fail(QC_EDEVICE, "qc_reset_ragged: %s", hipGetErrorString(e));
    }
  }
  return QC_OK;
}

qc_status qc_reset(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                   const int32_t* vis_len, int32_t zero_fill, void* stream) {
  return reset_impl(kv, qc, batch, vis_start, vis_len, nullptr, nullptr, zero_fill, stream);
}

qc_status qc_reset_ragged(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                          const int32_t* vis_len, const int32_t* cap_seq, const int32_t* cap_text,
                          int32_t zero_fill, void* stream) {
  if (!cap_seq || !cap_text) return fail(QC_EINVAL, "qc_reset_ragged: null capacity array");
  return reset_impl(kv, qc, batch, vis_start, vis_len, cap_seq, cap_text, zero_fill, stream);
}

static_assert(QC_PAGE_ROWS == qc::kPageRows, "header and library disagree on the page size");

size_t qc_page_table_bytes(const qc_config* cfg) {
  Config c;
  if (!parse_config(cfg, &c) || !c.pageable()) return 0;
  return (size_t)round_up(c.table_entries() * 4, 256);
}

qc_status qc_reset_paged(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                         const int32_t* vis_len, const uint8_t* present, void* page_lists,
                         size_t page_list_bytes, int32_t zero_fill, void* stream) {
  const PagedInit init = {present, page_lists, page_list_bytes};
  return reset_impl(kv, qc, batch, vis_start, vis_len, nullptr, nullptr, zero_fill, stream, &init);
}

// Pages the sequences need beyond what they hold.  want[b][pool] = rows slot b must be able to hold in the
// pool (negative: leave the slot's list of that pool alone).  Checks every pool first (QC_ECAPACITY, nothing
// changed), then hands pages out lowest number first, slot after slot and pool after pool, and enqueues
// the new list entries for the kernels.
static qc_status paged_reserve(qc_kvcache* kv, const std::vector<std::array<int64_t, 3>>& want, const char* who, hipStream_t st) {
  const Config& c = kv->cfg;
  int64_t need[3] = {0, 0, 0};
  for (int b = 0; b < kv->batch; ++b)
    for (int pool = 0; pool < 3; ++pool) {
      if (want[b][pool] < 0 || !c.pool_used(pool)) continue;
      const int64_t pages = (want[b][pool] + qc::kPageRows - 1) / qc::kPageRows;
      if (pages > c.pool_stride(pool)) return fail(QC_ECAPACITY, "%s: sequence %d needs %lld pages of pool %d, a sequence may hold %d", who, b, (long long)pages, pool, c.pool_stride(pool));
      need[pool] += std::max<int64_t>(0, pages - (int64_t)kv->pages[pool][b].size());
    }
  for (int pool = 0; pool < 3; ++pool)
    if (need[pool] > (int64_t)kv->free_pages[pool].size())
      return fail(QC_ECAPACITY, "%s: %lld pages of pool %d needed, %zu free", who, (long long)need[pool], pool, kv->free_pages[pool].size());
  // host side first (complete and consistent whatever the uploads below return), then the new entries
  // go to the device lists, TableChunk::N per launch
  std::vector<std::pair<int32_t, int32_t>> entries;   // (index in the page-list buffer, page)
  size_t taken[3] = {0, 0, 0};
  for (int b = 0; b < kv->batch; ++b)
    for (int pool = 0; pool < 3; ++pool) {
      if (want[b][pool] < 0 || !c.pool_used(pool)) continue;
      const int64_t pages = (want[b][pool] + qc::kPageRows - 1) / qc::kPageRows;
      while ((int64_t)kv->pages[pool][b].size() < pages) {
        const int32_t pg = kv->free_pages[pool][taken[pool]++];
        entries.emplace_back((int32_t)(c.table_off(pool) + (int64_t)b * c.pool_stride(pool) + (int64_t)kv->pages[pool][b].size()), pg);
        kv->pages[pool][b].push_back(pg);
      }
    }
  for (int pool = 0; pool < 3; ++pool)
    kv->free_pages[pool].erase(kv->free_pages[pool].begin(), kv->free_pages[pool].begin() + taken[pool]);
  qc::TableChunk tc;
  for (size_t first = 0; first < entries.size(); first += qc::TableChunk::N) {
    const int n = (int)std::min<size_t>(qc::TableChunk::N, entries.size() - first);
    for (int i = 0; i < n; ++i) {
      tc.at[i] = entries[first + i].first;
      tc.page[i] = entries[first + i].second;
    }
    hipError_t e = qc::launch_table_upload(kv->tables, n, tc, st);
    if (e != hipSuccess) return fail(QC_EDEVICE, "%s: page-list upload: %s", who, hipGetErrorString(e));
  }
  return QC_OK;
}

static qc::LayerView make_view(const qc_kvcache* kv, const qc_qcache* qc, int layer) {
  const Config& c = kv->cfg;
  qc::LayerView lv;
  lv.k_own = kv->arena + c.off_k(layer);
  lv.v_own = kv->arena + c.off_v(layer);
  lv.cap_k = (int32_t)c.cap_k(layer);
  lv.cap_v = (int32_t)c.cap_v(layer);
  int a = c.anchor[layer];
  lv.k_anchor = c.lazy[layer] ? kv->arena + c.off_k(a) : nullptr;
  lv.cap_k_anchor = (int32_t)c.cap_k(a);
  lv.q_cache = qc ? qc->arena : nullptr;
  lv.cap_q = (int32_t)c.cap_q();
  lv.meta = (const int32_t*)(kv->arena + c.off_meta()) + (kv->late(layer) ? qc::META_ROWS * c.max_batch : 0);
  lv.max_batch = c.max_batch;
  lv.flags = (kv->ragged ? qc::LV_RAGGED : 0) | ((c.lazy[layer] && !c.gla()) ? qc::LV_K_TEXT : 0) |
             (c.gla() ? 0 : qc::LV_Q_VIS) | (kv->late(layer) ? qc::LV_LATE : 0) | (kv->paged ? qc::LV_PAGED : 0);
  lv.pt_seq = lv.pt_k = lv.pt_q = nullptr;
  lv.pt_seq_stride = lv.pt_k_stride = lv.pt_q_stride = 0;
  if (kv->paged) {
    const int k_pool = (c.lazy[layer] && !c.gla()) ? 1 : 0, q_pool = c.gla() ? 0 : 2;
    lv.pt_seq = kv->tables + c.table_off(0);
    lv.pt_seq_stride = c.pool_stride(0);
    lv.pt_k = kv->tables + c.table_off(k_pool);
    lv.pt_k_stride = c.pool_stride(k_pool);
    lv.pt_q = kv->tables + c.table_off(q_pool);
    lv.pt_q_stride = c.pool_stride(q_pool);
  }
  return lv;
}

static qc_status check_spans(const char* who, const qc_kvcache* kv, int layer, const int32_t* vis_start, const int32_t* vis_len, bool prefill) {
  if (!vis_start || !vis_len) return fail(QC_EINVAL, "%s: null span arrays", who);
  for (int b = 0; b < kv->batch; ++b)
    if ((prefill ? kv->joining[b] : kv->live[b]) && (vis_start[b] != kv->vis_start[b] || vis_len[b] != kv->vis_len_of(layer, b)))
      return fail(QC_EINVAL, "%s: span of sequence %d differs from the one given to %s", who, b,
                  kv->late(layer) ? "qc_reset and qc_prune" : "qc_reset");
  return QC_OK;
}

// Per-sequence integers as the decode kernels want them, for slots [first, first + count): a
// sequence's length is its entry plus the step counter; a free slot's stays negative.
static qc_status upload_decode_meta(qc_kvcache* kv, int first, int count, hipStream_t st) {
  const Config& c = kv->cfg;
  int32_t* meta = (int32_t*)(kv->arena + c.off_meta());
  for (int f = first; f < first + count; f += qc::MetaChunk::N) {
    qc::MetaChunk mc;
    memset(&mc, 0, sizeof(mc));
    const int n = first + count - f < qc::MetaChunk::N ? first + count - f : qc::MetaChunk::N;
    for (int i = 0; i < n; ++i) {
      const int b = f + i;
      mc.v[qc::META_TOK0][i] = kv->tok0[b];
      mc.v[qc::META_LEN0][i] = kv->len_base(0, b);
      mc.v[qc::META_VIS_START][i] = kv->vis_start[b];
      mc.v[qc::META_VIS_LEN][i] = kv->vis_len[b];
    }
    hipError_t e = qc::launch_meta_upload(meta, c.max_batch, f, n, qc::META_ROWS, mc, st);
    if (e != hipSuccess) return fail(QC_EDEVICE, "metadata upload: %s", hipGetErrorString(e));
  }
  return QC_OK;
}

qc_status qc_prefill(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                     const void* k, const void* v, void* out, const int32_t* cu_seqlens,
                     int64_t token_stride, int64_t head_stride, const int32_t* vis_start,
                     const int32_t* vis_len, float softmax_scale, void* stream) {
  if (!kv || !qc) return fail(QC_EINVAL, "qc_prefill: null handle");
  const Config& c = kv->cfg;
  if (!c.same(qc->cfg)) return fail(QC_EINVAL, "qc_prefill: handles were created with different configurations");
  if (layer < 0 || layer >= c.N) return fail(QC_EINVAL, "qc_prefill: layer %d out of range", layer);
  if ((is_lazy != 0) != (c.lazy[layer] != 0)) return fail(QC_EINVAL, "qc_prefill: is_lazy=%d contradicts the configured mask for layer %d", is_lazy, layer);
  // Global Lazy Attention: a lazy layer has no q and k of its own, the two arguments are ignored.
  const bool qk_unused = c.gla() && c.lazy[layer];
  if (qk_unused) q = k = nullptr;
  if ((!qk_unused && (!q || !k)) || !v || !out || !cu_seqlens) return fail(QC_EINVAL, "qc_prefill: null tensor or cu_seqlens");
  const int e = c.e();
  if (head_stride < c.D || token_stride < c.D || (head_stride * e) % 16 || (token_stride * e) % 16)
    return fail(QC_EINVAL, "qc_prefill: strides must be >= head_dim and keep rows 16-byte aligned");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15)
    return fail(QC_EINVAL, "qc_prefill: tensors must be 16-byte aligned");
  if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return fail(QC_EINVAL, "qc_prefill: bad softmax_scale");
  if (kv->phase != PH_RESET && kv->phase != PH_PREFILL)
    return fail(QC_EORDER, "qc_prefill: no prefill pass is open (call qc_reset first)");
  if (layer != kv->next_layer) return fail(QC_EORDER, "qc_prefill: expected layer %d, got %d", kv->next_layer, layer);
  if (qc_status s = check_spans("qc_prefill", kv, layer, vis_start, vis_len, true)) return s;
  // The first layer of the pass, and the first layer after a pruning boundary, fix the packing.
  const bool opens = layer == 0 || layer == kv->first_late;
  if (cu_seqlens[0] != 0) return fail(QC_EINVAL, "qc_prefill: cu_seqlens[0] must be 0");
  int32_t max_len = 0;
  int participants = 0;
  for (int b = 0; b < kv->batch; ++b) {
    int64_t len = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
    if (!kv->joining[b]) {   // a free slot, or a sequence that is already decoding: not part of this pass
      if (len != 0) return fail(QC_EINVAL, "qc_prefill: slot %d is not filled by this pass, it must have no tokens in cu_seqlens", b);
      continue;
    }
    ++participants;
    if (len < 1) return fail(QC_EINVAL, "qc_prefill: sequence %d is empty", b);
    const int32_t vn = kv->vis_len_of(layer, b);
    if (layer > 0 && len != kv->len_of(layer, b))
      return fail(QC_EINVAL, "qc_prefill: sequence %d has %lld tokens, layer %d expects %d", b, (long long)len, layer, kv->len_of(layer, b));
    if (kv->vis_start[b] + vn > len) return fail(QC_EINVAL, "qc_prefill: span of sequence %d exceeds its %lld tokens", b, (long long)len);
    if (len > kv->cap_of(layer, b)) return fail(QC_ECAPACITY, "qc_prefill: sequence %d has %lld tokens, its capacity in layer %d is %lld", b, (long long)len, layer, (long long)kv->cap_of(layer, b));
    if (!c.gla() && len - vn > kv->cap_text_of(b)) return fail(QC_ECAPACITY, "qc_prefill: sequence %d has %lld text tokens, its capacity is %lld", b, (long long)(len - vn), (long long)kv->cap_text_of(b));
    if (!opens && cu_seqlens[b] != (kv->late(layer) ? kv->tok1[b] : kv->tok0[b]))
      return fail(QC_EINVAL, "qc_prefill: cu_seqlens changed between layers");
    if (len > max_len) max_len = (int32_t)len;
  }
  if (participants == 0) return fail(QC_EORDER, "qc_prefill: no slot of the batch is waiting to be filled");
  if ((int64_t)max_len * token_stride * e >= ((int64_t)1 << 31))
    return fail(QC_EINVAL, "qc_prefill: one sequence spans %lld bytes of the input tensors, the limit is 2 GiB", (long long)((int64_t)max_len * token_stride * e));
  if (c.lazy[layer] && qc->owner != c.anchor[layer])
    return fail(QC_EORDER, "qc_prefill: Q Cache belongs to layer %d, layer %d inherits from %d", qc->owner, layer, c.anchor[layer]);

  hipStream_t st = (hipStream_t)stream;
  if (kv->paged && layer == 0) {   // the prompts of this pass get their pages
    std::vector<std::array<int64_t, 3>> want(kv->batch, std::array<int64_t, 3>{-1, -1, -1});
    for (int b = 0; b < kv->batch; ++b)
      if (kv->joining[b]) {
        const int64_t len = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        want[b] = {len, len - kv->vis_len[b], kv->vis_len[b]};
      }
    if (qc_status s = paged_reserve(kv, want, "qc_prefill", st)) return s;
  }
  qc::LayerView lv = make_view(kv, qc, layer);
  if (opens) {
    for (int first = 0; first < kv->batch; first += qc::MetaChunk::N) {
      qc::MetaChunk mc;
      memset(&mc, 0, sizeof(mc));
      int count = kv->batch - first < qc::MetaChunk::N ? kv->batch - first : qc::MetaChunk::N;
      for (int i = 0; i < count; ++i) {
        int b = first + i;
        mc.v[qc::META_TOK0][i] = cu_seqlens[b];
        mc.v[qc::META_LEN0][i] = cu_seqlens[b + 1] - cu_seqlens[b];   // 0 outside the pass: the kernels skip the slot
        mc.v[qc::META_VIS_START][i] = kv->vis_start[b];
        mc.v[qc::META_VIS_LEN][i] = kv->vis_len_of(layer, b);
      }
      hipError_t e2 = qc::launch_meta_upload(const_cast<int32_t*>(lv.meta), c.max_batch, first, count, qc::META_ROWS, mc, st);
      if (e2 != hipSuccess) return fail(QC_EDEVICE, "qc_prefill: metadata upload: %s", hipGetErrorString(e2));
    }
  }
  qc::PrefillArgs a;
  a.lv = lv;
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.token_stride = token_stride;
  a.head_stride = head_stride;
  a.batch = kv->batch; a.n_heads = c.H; a.head_dim = c.D;
  a.is_lazy = c.lazy[layer];
  a.write_q = c.writes_q(layer) ? 1 : 0;
  a.inherit_all = c.gla() ? 1 : 0;
  a.max_len = max_len;
  a.scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)c.D);
  hipError_t err = qc::launch_prefill(a, c.dtype, st, kv->timing ? &kv->prefill_timer : nullptr);
  if (err != hipSuccess) return fail(QC_EDEVICE, "qc_prefill: %s", hipGetErrorString(err));

  if (layer == 0) {
    for (int b = 0; b < kv->batch; ++b)
      if (kv->joining[b]) {
        kv->tok0[b] = cu_seqlens[b];
        kv->len0[b] = cu_seqlens[b + 1] - cu_seqlens[b];
      }
  } else if (opens) {
    for (int b = 0; b < kv->batch; ++b) kv->tok1[b] = cu_seqlens[b];
    kv->late_known = true;
  }
  if (a.write_q) qc->owner = layer;
  kv->next_layer = layer + 1;
  kv->phase = PH_PREFILL;
  if (kv->next_layer == c.N) {
    // The pass is over: its sequences decode from the next step on.  When slots are free, or sequences
    // that were decoding already sat the pass out, the per-sequence integers the decode kernels read
    // are written again: the pass had the lengths of the slots outside it at zero.
    const bool rewrite = kv->join_pass || !kv->all_live();
    for (int b = 0; b < kv->batch; ++b)
      if (kv->joining[b]) {
        kv->joining[b] = 0;
        kv->joined_at[b] = kv->generated;
      }
    kv->join_pass = false;
    kv->phase = PH_READY;
    kv->next_layer = 0;
    if (rewrite)
      if (qc_status s = upload_decode_meta(kv, 0, kv->batch, st)) return s;
  }
  return QC_OK;
}

// ---- sequences joining and leaving a running batch ----------------------------------------------
// Lowest start of `want` free rows in a pool of `pool` rows, given the extents (start, rows) in use;
// -1 when no gap is wide enough.  A request for no rows is placed at 0.
static int64_t first_fit(std::vector<std::pair<int64_t, int64_t>> used, int64_t want, int64_t pool) {
  if (want == 0) return 0;
  std::sort(used.begin(), used.end());
  int64_t at = 0;
  for (const auto& u : used) {
    if (u.second == 0) continue;
    if (u.first - at >= want) return at;
    at = std::max(at, u.first + u.second);
  }
  return pool - at >= want ? at : -1;
}

qc_status qc_seq_leave(qc_kvcache* kv, qc_qcache* qc, int32_t b, void* stream) {
  if (!kv || !qc) return fail(QC_EINVAL, "qc_seq_leave: null handle");
  if (!kv->slots()) return fail(QC_EORDER, "qc_seq_leave: needs a batch set up with per-sequence capacities (qc_reset_ragged) or with pages (qc_reset_paged)");
  if (b < 0 || b >= kv->batch) return fail(QC_EINVAL, "qc_seq_leave: slot %d out of range", b);
  if (kv->phase != PH_READY) return fail(QC_EORDER, "qc_seq_leave: allowed between two decode steps only");
  if (!kv->live[b]) return fail(QC_EINVAL, "qc_seq_leave: slot %d holds no sequence", b);
  kv->live[b] = 0;
  if (kv->paged) {   // its pages are free again (lowest numbers first at the next hand-out)
    for (int pool = 0; pool < 3; ++pool) {
      auto& fr = kv->free_pages[pool];
      fr.insert(fr.end(), kv->pages[pool][b].begin(), kv->pages[pool][b].end());
      std::sort(fr.begin(), fr.end());
      kv->pages[pool][b].clear();
    }
  } else {
    kv->cap_seq[b] = kv->cap_text[b] = 0;
    kv->base_seq[b] = kv->base_text[b] = kv->base_vis[b] = 0;
  }
  kv->vis_start[b] = kv->vis_len[b] = 0;
  kv->len0[b] = kv->tok0[b] = kv->joined_at[b] = 0;
  return upload_decode_meta(kv, b, 1, (hipStream_t)stream);
}

qc_status qc_seq_join(qc_kvcache* kv, qc_qcache* qc, int32_t b, int32_t vis_start, int32_t vis_len,
                      int32_t cap_seq, int32_t cap_text, void* stream) {
  if (!kv || !qc) return fail(QC_EINVAL, "qc_seq_join: null handle");
  const Config& c = kv->cfg;
  if (!kv->slots()) return fail(QC_EORDER, "qc_seq_join: needs a batch set up with per-sequence capacities (qc_reset_ragged) or with pages (qc_reset_paged)");
  if (b < 0 || b >= kv->batch) return fail(QC_EINVAL, "qc_seq_join: slot %d out of range", b);
  // between two decode steps, or before the prefill pass that follows (more joins, or the reset) has begun
  if (kv->phase != PH_READY && kv->phase != PH_RESET) return fail(QC_EORDER, "qc_seq_join: allowed between two decode steps, or before a prefill pass has begun");
  if (kv->first_late >= 0) return fail(QC_EORDER, "qc_seq_join: not available on a batch with a pruning boundary");
  if (kv->live[b]) return fail(QC_EINVAL, "qc_seq_join: slot %d is taken", b);
  if (vis_start < 0 || vis_len < 0) return fail(QC_EINVAL, "qc_seq_join: negative span");
  if (kv->paged) {   // pages are handed out when the sequence's prefill pass begins; capacities are not used
    if (cap_seq != 0 || cap_text != 0) return fail(QC_EINVAL, "qc_seq_join: a paged batch takes no capacities (pass 0)");
    if (c.pool_used(2) && vis_len > (int64_t)c.pool_stride(2) * qc::kPageRows) return fail(QC_ECAPACITY, "qc_seq_join: %d visual tokens, a sequence may hold %lld", vis_len, (long long)c.pool_stride(2) * qc::kPageRows);
    if ((int64_t)vis_start + vis_len > (int64_t)c.pool_stride(0) * qc::kPageRows) return fail(QC_ECAPACITY, "qc_seq_join: the span exceeds what a sequence may hold");
    kv->live[b] = kv->joining[b] = 1;
    kv->joined_at[b] = 0;
    kv->vis_start[b] = vis_start;
    kv->vis_len[b] = vis_len;
    kv->len0[b] = kv->tok0[b] = 0;
    if (kv->phase == PH_READY) {
      kv->join_pass = true;
      kv->phase = PH_RESET;
      kv->next_layer = 0;
    }
    return QC_OK;
  }
  if (cap_seq < 8 || cap_seq % 8 || cap_text < 0) return fail(QC_EINVAL, "qc_seq_join: cap_seq must be a positive multiple of 8, cap_text not negative");
  if ((int64_t)vis_start + vis_len > cap_seq) return fail(QC_ECAPACITY, "qc_seq_join: the span exceeds the sequence's %d positions", cap_seq);
  std::vector<std::pair<int64_t, int64_t>> seq, text, vis;
  for (int i = 0; i < kv->batch; ++i)
    if (kv->live[i]) {
      seq.emplace_back(kv->base_seq[i], kv->cap_seq[i]);
      text.emplace_back(kv->base_text[i], kv->cap_text[i]);
      vis.emplace_back(kv->base_vis[i], kv->vis_len[i]);
    }
  const int64_t at_seq = first_fit(seq, cap_seq, (int64_t)c.max_batch * c.max_seq);
  const int64_t at_text = c.gla() ? 0 : first_fit(text, cap_text, (int64_t)c.max_batch * c.max_text);
  const int64_t at_vis = c.gla() ? 0 : first_fit(vis, vis_len, (int64_t)c.max_batch * c.max_vis);
  if (at_seq < 0) return fail(QC_ECAPACITY, "qc_seq_join: no run of %d free positions among max_batch*max_seq = %lld", cap_seq, (long long)c.max_batch * c.max_seq);
  if (at_text < 0) return fail(QC_ECAPACITY, "qc_seq_join: no run of %d free text rows among max_batch*max_text = %lld", cap_text, (long long)c.max_batch * c.max_text);
  if (at_vis < 0) return fail(QC_ECAPACITY, "qc_seq_join: no run of %d free Q Cache rows among max_batch*max_vis = %lld", vis_len, (long long)c.max_batch * c.max_vis);
  qc::MetaChunk mc;
  memset(&mc, 0, sizeof(mc));
  mc.v[qc::CAP_SEQ][0] = cap_seq;
  mc.v[qc::BASE_SEQ][0] = (int32_t)at_seq;
  mc.v[qc::CAP_TEXT][0] = cap_text;
  mc.v[qc::BASE_TEXT][0] = (int32_t)at_text;
  mc.v[qc::CAP_VIS][0] = vis_len;
  mc.v[qc::BASE_VIS][0] = (int32_t)at_vis;
  hipError_t e = qc::launch_meta_upload((int32_t*)(kv->arena + c.off_caps()), c.max_batch, b, 1, qc::CAPS_ROWS, mc, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_seq_join: %s", hipGetErrorString(e));
  kv->live[b] = kv->joining[b] = 1;
  kv->joined_at[b] = 0;
  kv->cap_seq[b] = cap_seq;
  kv->cap_text[b] = cap_text;
  kv->base_seq[b] = (int32_t)at_seq;
  kv->base_text[b] = (int32_t)at_text;
  kv->base_vis[b] = (int32_t)at_vis;
  kv->vis_start[b] = vis_start;
  kv->vis_len[b] = vis_len;
  kv->len0[b] = kv->tok0[b] = 0;
  if (kv->phase == PH_READY) {   // opens a pass of its own: the sequences that are decoding sit it out
    kv->join_pass = true;
    kv->phase = PH_RESET;
    kv->next_layer = 0;
  }
  return QC_OK;
}

qc_status qc_seq_grow(qc_kvcache* kv, qc_qcache* qc, int32_t b, int32_t cap_seq, int32_t cap_text, void* stream) {
  if (!kv || !qc) return fail(QC_EINVAL, "qc_seq_grow: null handle");
  const Config& c = kv->cfg;
  if (kv->paged) return fail(QC_EORDER, "qc_seq_grow: a paged batch grows page by page on its own");
  if (!kv->ragged) return fail(QC_EORDER, "qc_seq_grow: needs a batch set up with per-sequence capacities (qc_reset_ragged)");
  if (b < 0 || b >= kv->batch) return fail(QC_EINVAL, "qc_seq_grow: slot %d out of range", b);
  if (kv->phase != PH_READY) return fail(QC_EORDER, "qc_seq_grow: allowed between two decode steps only");
  if (!kv->live[b]) return fail(QC_EINVAL, "qc_seq_grow: slot %d holds no sequence", b);
  if (kv->first_late >= 0) return fail(QC_EORDER, "qc_seq_grow: not available on a batch with a pruning boundary");
  const int64_t len = (int64_t)kv->len0[b] + kv->steps_of(b), text = len - kv->vis_len[b];
  if (cap_seq < 8 || cap_seq % 8 || cap_text < 0) return fail(QC_EINVAL, "qc_seq_grow: cap_seq must be a positive multiple of 8, cap_text not negative");
  if (cap_seq < len || (!c.gla() && cap_text < text))
    return fail(QC_ECAPACITY, "qc_seq_grow: the sequence already holds %lld positions and %lld text rows", (long long)len, (long long)text);
  // New extents beside everybody's current ones, the sequence's own included: rows are copied, never
  // shifted in place.  A pool whose capacity does not change keeps its extent.
  std::vector<std::pair<int64_t, int64_t>> seq, txt;
  for (int i = 0; i < kv->batch; ++i)
    if (kv->live[i]) {
      seq.emplace_back(kv->base_seq[i], kv->cap_seq[i]);
      txt.emplace_back(kv->base_text[i], kv->cap_text[i]);
    }
  const bool move_seq = cap_seq != kv->cap_seq[b], move_text = !c.gla() && cap_text != kv->cap_text[b];
  const int64_t at_seq = move_seq ? first_fit(seq, cap_seq, (int64_t)c.max_batch * c.max_seq) : kv->base_seq[b];
  const int64_t at_text = move_text ? first_fit(txt, cap_text, (int64_t)c.max_batch * c.max_text) : kv->base_text[b];
  if (at_seq < 0) return fail(QC_ECAPACITY, "qc_seq_grow: no run of %d free positions among max_batch*max_seq = %lld", cap_seq, (long long)c.max_batch * c.max_seq);
  if (at_text < 0) return fail(QC_ECAPACITY, "qc_seq_grow: no run of %d free text rows among max_batch*max_text = %lld", cap_text, (long long)c.max_batch * c.max_text);
  const int64_t rb = c.row_bytes();
  qc::MoveChunk mc;
  int n = 0;
  auto flush = [&]() -> hipError_t {
    hipError_t e = qc::launch_move_rows(kv->arena, qc->arena, (int32_t)rb, c.H, n, mc, (hipStream_t)stream);
    n = 0;
    return e;
  };
  auto add = [&](int arena, int64_t region, int64_t base_old, int64_t cap_old, int64_t base_new, int64_t cap_new, int64_t rows) -> hipError_t {
    if (rows == 0) return hipSuccess;
    mc.arena[n] = arena;
    mc.src[n] = region + base_old * c.H * rb;
    mc.dst[n] = region + base_new * c.H * rb;
    mc.src_stride[n] = cap_old * rb;
    mc.dst_stride[n] = cap_new * rb;
    mc.rows[n] = (int32_t)rows;
    return ++n == qc::MoveChunk::N ? flush() : hipSuccess;
  };
  hipError_t e = hipSuccess;
  for (int l = 0; l < c.N && e == hipSuccess; ++l) {
    if (move_seq) e = add(0, c.off_v(l), kv->base_seq[b], kv->cap_seq[b], at_seq, cap_seq, len);
    if (e != hipSuccess) break;
    const bool text_rows = c.lazy[l] && !c.gla();
    if (text_rows) { if (move_text) e = add(0, c.off_k(l), kv->base_text[b], kv->cap_text[b], at_text, cap_text, text); }
    else if (c.cap_k(l) > 0 && move_seq) e = add(0, c.off_k(l), kv->base_seq[b], kv->cap_seq[b], at_seq, cap_seq, len);
  }
  // Global Lazy Attention: the Q Cache holds one row per position, laid out like the position rows
  if (e == hipSuccess && c.gla() && move_seq && qc->owner >= 0) e = add(1, 0, kv->base_seq[b], kv->cap_seq[b], at_seq, cap_seq, len);
  if (e == hipSuccess) e = flush();
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_seq_grow: %s", hipGetErrorString(e));
  qc::MetaChunk caps;
  memset(&caps, 0, sizeof(caps));
  caps.v[qc::CAP_SEQ][0] = cap_seq;
  caps.v[qc::BASE_SEQ][0] = (int32_t)at_seq;
  caps.v[qc::CAP_TEXT][0] = c.gla() ? kv->cap_text[b] : cap_text;
  caps.v[qc::BASE_TEXT][0] = (int32_t)at_text;
  caps.v[qc::CAP_VIS][0] = kv->vis_len[b];
  caps.v[qc::BASE_VIS][0] = kv->base_vis[b];
  e = qc::launch_meta_upload((int32_t*)(kv->arena + c.off_caps()), c.max_batch, b, 1, qc::CAPS_ROWS, caps, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_seq_grow: %s", hipGetErrorString(e));
  kv->cap_seq[b] = cap_seq;
  kv->base_seq[b] = (int32_t)at_seq;
  if (!c.gla()) kv->cap_text[b] = cap_text;
  kv->base_text[b] = (int32_t)at_text;
  return QC_OK;
}

qc_status qc_seq_pages(const qc_kvcache* kv, int32_t b, int32_t pool, int32_t* pages, int32_t capacity, int32_t* count) {
  if (!kv || !count) return fail(QC_EINVAL, "qc_seq_pages: null argument");
  if (!kv->paged) return fail(QC_EORDER, "qc_seq_pages: needs a paged batch (qc_reset_paged)");
  if (b < 0 || b >= kv->batch || pool < 0 || pool > 2) return fail(QC_EINVAL, "qc_seq_pages: slot or pool out of range");
  const auto& list = kv->pages[pool][b];
  *count = (int32_t)list.size();
  if (pages)
    for (int i = 0; i < capacity && i < (int)list.size(); ++i) pages[i] = list[i];
  return QC_OK;
}

qc_status qc_pool_pages(const qc_kvcache* kv, int32_t pool, int32_t* total, int32_t* free_pages) {
  if (!kv || !total || !free_pages) return fail(QC_EINVAL, "qc_pool_pages: null argument");
  if (!kv->paged) return fail(QC_EORDER, "qc_pool_pages: needs a paged batch (qc_reset_paged)");
  if (pool < 0 || pool > 2) return fail(QC_EINVAL, "qc_pool_pages: pool out of range");
  *total = (int32_t)kv->cfg.pool_pages(pool);
  *free_pages = (int32_t)kv->free_pages[pool].size();
  return QC_OK;
}

qc_status qc_pages_needed(const qc_config* cfg, int32_t len, int32_t vis_len, int32_t* pages) {
  Config c;
  if (!pages) return fail(QC_EINVAL, "qc_pages_needed: null argument");
  if (!parse_config(cfg, &c)) return fail(QC_EINVAL, "qc_pages_needed: invalid configuration");
  if (!c.pageable()) return fail(QC_EINVAL, "qc_pages_needed: the configuration cannot be paged");
  if (len < 0 || vis_len < 0 || vis_len > len) return fail(QC_EINVAL, "qc_pages_needed: need 0 <= vis_len <= len");
  const int64_t rows[3] = {len, (int64_t)len - vis_len, vis_len};
  for (int pool = 0; pool < 3; ++pool)
    pages[pool] = c.pool_used(pool) ? (int32_t)((rows[pool] + qc::kPageRows - 1) / qc::kPageRows) : 0;
  return QC_OK;
}

qc_status qc_seq_extent(const qc_kvcache* kv, int32_t b, int32_t* live, int32_t* base_seq, int32_t* base_text, int32_t* base_vis) {
  if (!kv || !live || !base_seq || !base_text || !base_vis) return fail(QC_EINVAL, "qc_seq_extent: null argument");
  if (kv->paged) return fail(QC_EORDER, "qc_seq_extent: a paged batch has no extents (see qc_seq_pages)");
  if (!kv->ragged) return fail(QC_EORDER, "qc_seq_extent: needs a batch set up with per-sequence capacities (qc_reset_ragged)");
  if (b < 0 || b >= kv->batch) return fail(QC_EINVAL, "qc_seq_extent: slot %d out of range", b);
  *live = kv->live[b];
  *base_seq = kv->base_seq[b];
  *base_text = kv->base_text[b];
  *base_vis = kv->base_vis[b];
  return QC_OK;
}

// How a decode launch splits the key axis of its (sequence, head) pairs: *chunk key positions per workgroup,
// *max_chunks workgroups for the longest sequence (positions 0 .. max_len).
// Split only as far as needed to give every compute unit a few workgroups: each extra chunk costs a
// partial result and the merge pass.  With many pairs there is no split and the kernel writes the output
// directly.
static void split_plan(int64_t pairs, int64_t max_len, int64_t units, int32_t* chunk, int32_t* max_chunks) {
  constexpr int64_t kTargetGroups = 1024;
  int64_t want = (kTargetGroups + pairs - 1) / pairs;
  if (want < 1) want = 1;
  // Where the chunks stay long (the bandwidth-bound launches), the number of chunks is the one between
  // 3 and 6 workgroups per compute unit (all resident at once) that spreads them most evenly: the launch
  // lasts as long as its fullest unit.  Measured at 160 pairs on 256 units, 5 to 9 chunks: 5.53, 6.11,
  // 5.88, 6.16, 6.10 TB/s for 3.1, 3.75, 4.4, 5.0, 5.6 workgroups per unit.
  int64_t best = 0;
  double best_ratio = 0.0;
  for (int64_t n = std::max<int64_t>(1, (3 * units + pairs - 1) / pairs); n * pairs <= 6 * units; ++n) {
    if ((max_len + 1) / n < 2 * kMinChunkKeys) break;
    const double per_unit = (double)(n * pairs) / (double)units;
    const double ratio = std::ceil(per_unit) / per_unit;   // fullest unit against the mean
    if (best == 0 || ratio < best_ratio - 1e-9) {
      best = n;
      best_ratio = ratio;
    }
  }
  if (best > 0) want = best;
  const int64_t per = (max_len + 1 + want - 1) / want;
  // chunks of (nearly) equal length: a chunk rounded up to a multiple of 64 left up to a tenth more rows
  // in six chunks than in the seventh at cfg5 (+2.5 % time)
  *chunk = (int32_t)(per < kMinChunkKeys ? kMinChunkKeys : round_up(per, 8));
  *max_chunks = (int32_t)((max_len + 1 + *chunk - 1) / *chunk);
}

qc_status qc_decode_split(int32_t pairs, int32_t max_len, int32_t compute_units_, int32_t* chunk_keys, int32_t* chunks) {
  if (!chunk_keys || !chunks) return fail(QC_EINVAL, "qc_decode_split: null argument");
  if (pairs < 1 || max_len < 0 || compute_units_ < 1) return fail(QC_EINVAL, "qc_decode_split: need pairs >= 1, max_len >= 0, compute_units >= 1");
  split_plan(pairs, max_len, compute_units_, chunk_keys, chunks);
  return QC_OK;
}

// Launch geometry of a decode call that is being recorded into a graph: fixed for every later replay.
struct GraphGeom {
  int32_t chunk, max_chunks;
  const int32_t* generated_dev;
};

static qc_status decode_impl(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                             const void* k, const void* v, void* out, const int32_t* vis_start,
                             const int32_t* vis_len, float softmax_scale, void* workspace,
                             size_t workspace_bytes, void* stream, const GraphGeom* geom,
                             bool static_scratch = false) {
  if (!kv) return fail(QC_EINVAL, "qc_decode: null handle");
  const Config& c = kv->cfg;
  // Visual Lazy Attention never touches the Q Cache while decoding; Global Lazy Attention does.
  if (c.gla()) {
    if (!qc) return fail(QC_EINVAL, "qc_decode: Global Lazy Attention needs the Q Cache handle");
    if (!c.same(qc->cfg)) return fail(QC_EINVAL, "qc_decode: handles were created with different configurations");
  }
  if (layer < 0 || layer >= c.N) return fail(QC_EINVAL, "qc_decode: layer %d out of range", layer);
  if ((is_lazy != 0) != (c.lazy[layer] != 0)) return fail(QC_EINVAL, "qc_decode: is_lazy=%d contradicts the configured mask for layer %d", is_lazy, layer);
  const bool qk_unused = c.gla() && c.lazy[layer];
  if (qk_unused) q = k = nullptr;
  if ((!qk_unused && (!q || !k)) || !v || !out || !workspace) return fail(QC_EINVAL, "qc_decode: null tensor or workspace");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)workspace) & 15)
    return fail(QC_EINVAL, "qc_decode: tensors and workspace must be 16-byte aligned");
  if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return fail(QC_EINVAL, "qc_decode: bad softmax_scale");
  if (kv->phase != PH_READY && kv->phase != PH_DECODE) return fail(QC_EORDER, "qc_decode: prefill has not finished");
  if (layer != kv->next_layer) return fail(QC_EORDER, "qc_decode: expected layer %d, got %d", kv->next_layer, layer);
  if (!geom)
    if (qc_status s = check_spans("qc_decode", kv, layer, vis_start, vis_len, false)) return s;
  int32_t max_len = 0;
  for (int b = 0; b < kv->batch; ++b) {
    if (!kv->live[b]) continue;
    int64_t len = (int64_t)kv->len_of(layer, b) + kv->steps_of(b);
    const int32_t vn = kv->vis_len_of(layer, b);
    if (len + 1 > kv->cap_of(layer, b)) return fail(QC_ECAPACITY, "qc_decode: sequence %d would reach %lld positions, its capacity in layer %d is %lld", b, (long long)(len + 1), layer, (long long)kv->cap_of(layer, b));
    if (!c.gla() && len + 1 - vn > kv->cap_text_of(b)) return fail(QC_ECAPACITY, "qc_decode: sequence %d would reach %lld text rows, its capacity is %lld", b, (long long)(len + 1 - vn), (long long)kv->cap_text_of(b));
    if (len > max_len) max_len = (int32_t)len;
  }
  if (qk_unused && qc->owner != c.anchor[layer])
    return fail(QC_EORDER, "qc_decode: Q Cache belongs to layer %d, layer %d inherits from %d", qc->owner, layer, c.anchor[layer]);
  const int64_t pairs = (int64_t)kv->batch * c.H;
  int32_t chunk = 0, max_chunks = 0;
  split_plan(pairs, max_len, kv->units, &chunk, &max_chunks);
  if (geom) {
    chunk = geom->chunk;
    max_chunks = geom->max_chunks;
  }
  size_t need = (size_t)kv->batch * c.H * max_chunks * (c.D + 2) * 4;
  if (c.gla()) need = (size_t)(partial_bytes(c) + score_bytes(c));
  if (workspace_bytes < need)
    return static_scratch ? fail(QC_ECAPACITY, "qc_decode_static: the call needs %zu bytes of scratch, the library's array holds %zu; use qc_decode with a workspace", need, workspace_bytes)
                          : fail(QC_ECAPACITY, "qc_decode: workspace holds %zu bytes, %zu needed", workspace_bytes, need);
  if (qk_unused && kv->score_workspace != workspace)
    return fail(QC_EINVAL, "qc_decode: layer %d needs the workspace its block's first layer was called with", layer);

  if (kv->paged && layer == 0 && !geom) {   // the row this step appends may open a page (a replayed step: at its launch)
    std::vector<std::array<int64_t, 3>> want(kv->batch, std::array<int64_t, 3>{-1, -1, -1});
    for (int b = 0; b < kv->batch; ++b)
      if (kv->live[b]) {
        const int64_t len = (int64_t)kv->len_of(0, b) + kv->steps_of(b);
        want[b] = {len + 1, len + 1 - kv->vis_len[b], -1};
      }
    if (qc_status s = paged_reserve(kv, want, "qc_decode", (hipStream_t)stream)) return s;
  }
  qc::DecodeArgs a;
  a.lv = make_view(kv, c.gla() ? qc : nullptr, layer);
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.workspace = (float*)workspace;
  a.generated_dev = geom ? geom->generated_dev : nullptr;
  a.batch = kv->batch; a.n_heads = c.H; a.head_dim = c.D;
  a.is_lazy = c.lazy[layer];
  qc::DecodeGlaArgs g;
  g.scores = c.gla() ? (float*)((char*)workspace + partial_bytes(c)) : nullptr;
  g.score_stride = (int32_t)score_stride(c);
  g.mode = qk_unused ? 2 : ((c.gla() && c.writes_q(layer)) ? 1 : 0);
  a.generated = kv->generated;
  a.max_len = max_len;
  a.chunk_keys = chunk;
  a.max_chunks = max_chunks;
  a.scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)c.D);
  // a recorded launch reads everything per-sequence from device memory: it then serves any batch of this size
  a.inline_meta = (!geom && !kv->paged && kv->batch <= qc::DecodeArgs::kInlineSeqs) ? 1 : 0;
  for (int b = 0; b < qc::DecodeArgs::kInlineSeqs; ++b) {
    const bool ok = a.inline_meta && b < kv->batch;
    a.len0_inline[b] = ok ? kv->len_base(layer, b) : 0;
    a.vis_start_inline[b] = ok ? kv->vis_start[b] : 0;
    a.vis_len_inline[b] = ok ? kv->vis_len_of(layer, b) : 0;
  }
  qc::KernelTimer* timer = (!kv->timing || geom) ? nullptr : (g.mode == 2 ? &kv->decode_shared_timer : &kv->decode_timer);
  hipError_t err = qc::launch_decode(a, g, c.dtype, (hipStream_t)stream, timer);
  if (err != hipSuccess) return fail(QC_EDEVICE, "qc_decode: %s", hipGetErrorString(err));

  if (g.mode == 1) {
    qc->owner = layer;
    kv->score_workspace = workspace;
  }
  kv->next_layer = layer + 1;
  kv->phase = PH_DECODE;
  if (kv->next_layer == c.N) {
    kv->next_layer = 0;
    kv->generated += 1;
    kv->phase = PH_READY;
  }
  return QC_OK;
}

qc_status qc_decode(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                    const void* k, const void* v, void* out, const int32_t* vis_start,
                    const int32_t* vis_len, float softmax_scale, void* workspace,
                    size_t workspace_bytes, void* stream) {
  return decode_impl(kv, qc, layer, is_lazy, q, k, v, out, vis_start, vis_len, softmax_scale, workspace,
                     workspace_bytes, stream, nullptr);
}

qc_status qc_decode_static(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                           const void* k, const void* v, void* out, const int32_t* vis_start,
                           const int32_t* vis_len, float softmax_scale, void* stream) {
  static_assert(QC_STATIC_SCRATCH_BYTES == qc::kStaticScratchBytes, "header and library disagree on the scratch size");
  void* scratch_ptr = nullptr;
  size_t scratch_bytes = 0;
  hipError_t e = qc::decode_static_scratch(&scratch_ptr, &scratch_bytes);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_decode_static: %s", hipGetErrorString(e));
  return decode_impl(kv, qc, layer, is_lazy, q, k, v, out, vis_start, vis_len, softmax_scale, scratch_ptr,
                     scratch_bytes, stream, nullptr, true);
}

// ---- one whole decode step as a replayable graph -------------------------------------------------
// Capacity checks of a step about to be replayed: every layer's appended row must fit.
static qc_status step_fits(const char* who, const qc_kvcache* kv) {
  const Config& c = kv->cfg;
  for (int stage = 0; stage < 2; ++stage) {
    const int layer = stage ? (kv->first_late >= 0 ? kv->first_late : (c.late_from > 0 ? c.late_from : -1)) : 0;
    if (layer < 0) break;
    for (int b = 0; b < kv->batch; ++b) {
      if (!kv->live[b]) continue;
      const int64_t len = (int64_t)kv->len_of(layer, b) + kv->steps_of(b);
      if (len + 1 > kv->cap_of(layer, b)) return fail(QC_ECAPACITY, "%s: sequence %d would reach %lld positions, its capacity in layer %d is %lld", who, b, (long long)(len + 1), layer, (long long)kv->cap_of(layer, b));
      if (!c.gla() && len + 1 - kv->vis_len_of(layer, b) > kv->cap_text_of(b))
        return fail(QC_ECAPACITY, "%s: sequence %d would reach %lld text rows, its capacity is %lld", who, b, (long long)(len + 1 - kv->vis_len_of(layer, b)), (long long)kv->cap_text_of(b));
    }
  }
  return QC_OK;
}

qc_status qc_decode_graph_create(qc_kvcache* kv, qc_qcache* qc, const void* const* q, const void* const* k,
                                 const void* const* v, void* const* out, float softmax_scale, void* workspace,
                                 size_t workspace_bytes, qc_decode_graph** out_graph) {
  if (!out_graph) return fail(QC_EINVAL, "qc_decode_graph_create: out_graph is null");
  *out_graph = nullptr;
  if (!kv || !qc || !q || !k || !v || !out) return fail(QC_EINVAL, "qc_decode_graph_create: null argument");
  const Config& c = kv->cfg;
  if (!c.same(qc->cfg)) return fail(QC_EINVAL, "qc_decode_graph_create: handles were created with different configurations");
  if (kv->phase != PH_READY) return fail(QC_EORDER, "qc_decode_graph_create: needs a finished prefill pass and no decode step in flight");
  if (qc_status s = step_fits("qc_decode_graph_create", kv)) return s;
  // Launch geometry for any length up to the capacity (workgroups past a sequence's end leave at once).
  constexpr int64_t kTargetGroups = 1024;
  const int64_t pairs = (int64_t)kv->batch * c.H;
  const int64_t want = std::max<int64_t>(1, (kTargetGroups + pairs - 1) / pairs);
  const int64_t longest = kv->longest_cap();
  const int64_t per = (longest + want - 1) / want;
  GraphGeom geom;
  geom.chunk = (int32_t)round_up(per < kMinChunkKeys ? kMinChunkKeys : per, kMinChunkKeys);
  geom.max_chunks = (int32_t)((longest + geom.chunk - 1) / geom.chunk);
  geom.generated_dev = (const int32_t*)(kv->arena + c.off_counters());

  hipStream_t cap = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&cap, hipStreamNonBlocking);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_decode_graph_create: %s", hipGetErrorString(e));
  // Recording runs the ordinary call sequence of a step, which moves the bookkeeping forward as if
  // the step had happened; it is put back afterwards (nothing executes while recording).
  const int saved_phase = kv->phase, saved_next = kv->next_layer, saved_gen = kv->generated, saved_owner = qc->owner;
  const void* saved_score_ws = kv->score_workspace;
  qc_status st = QC_OK;
  hipGraph_t graph = nullptr;
  e = hipStreamBeginCapture(cap, hipStreamCaptureModeThreadLocal);
  if (e == hipSuccess) {
    for (int l = 0; l < c.N && st == QC_OK; ++l)
      st = decode_impl(kv, qc, l, c.lazy[l], q[l], k[l], v[l], out[l], nullptr, nullptr, softmax_scale, workspace,
                       workspace_bytes, cap, &geom);
    if (st == QC_OK) {
      hipError_t e2 = qc::launch_counter_update((int32_t*)(kv->arena + c.off_counters()), 1, 1, cap);
      if (e2 != hipSuccess) st = fail(QC_EDEVICE, "qc_decode_graph_create: %s", hipGetErrorString(e2));
    }
    hipError_t e3 = hipStreamEndCapture(cap, &graph);
    if (st == QC_OK && e3 != hipSuccess) st = fail(QC_EDEVICE, "qc_decode_graph_create: %s", hipGetErrorString(e3));
  } else {
    st = fail(QC_EDEVICE, "qc_decode_graph_create: %s", hipGetErrorString(e));
  }
  const int final_owner = qc->owner;
  const void* final_score_ws = kv->score_workspace;
  kv->phase = saved_phase; kv->next_layer = saved_next; kv->generated = saved_gen; qc->owner = saved_owner;
  kv->score_workspace = saved_score_ws;
  (void)hipStreamDestroy(cap);
  if (st != QC_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return st;
  }
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_decode_graph_create: %s", hipGetErrorString(e));
  qc_decode_graph* g = new (std::nothrow) qc_decode_graph;
  if (!g) {
    (void)hipGraphExecDestroy(exec);
    return fail(QC_ECAPACITY, "qc_decode_graph_create: out of host memory");
  }
  g->kv = kv; g->qc = qc; g->exec = exec;
  g->batch = kv->batch; g->first_late = kv->first_late;
  g->ragged = kv->ragged; g->paged = kv->paged; g->covered = (int64_t)geom.chunk * geom.max_chunks;
  g->final_owner = final_owner; g->score_workspace = final_score_ws;
  *out_graph = g;
  return QC_OK;
}

qc_status qc_decode_graph_launch(qc_decode_graph* g, void* stream) {
  if (!g) return fail(QC_EINVAL, "qc_decode_graph_launch: null handle");
  qc_kvcache* kv = g->kv;
  const Config& c = kv->cfg;
  if (kv->phase != PH_READY) return fail(QC_EORDER, "qc_decode_graph_launch: needs a finished prefill pass and no decode step in flight");
  if (kv->batch != g->batch || kv->first_late != g->first_late)
    return fail(QC_EORDER, "qc_decode_graph_launch: the graph was recorded for %d sequences (pruning boundary %d), the cache now holds %d (%d)", g->batch, g->first_late, kv->batch, kv->first_late);
  if (kv->ragged != g->ragged || kv->paged != g->paged || kv->longest_cap() > g->covered)
    return fail(QC_EORDER, "qc_decode_graph_launch: the graph was recorded for another kind of capacities, or for at most %lld positions", (long long)g->covered);
  if (qc_status s = step_fits("qc_decode_graph_launch", kv)) return s;
  if (kv->paged) {   // the row this step appends may open a page: host work ahead of the replay, on its stream
    std::vector<std::array<int64_t, 3>> want(kv->batch, std::array<int64_t, 3>{-1, -1, -1});
    for (int b = 0; b < kv->batch; ++b)
      if (kv->live[b]) {
        const int64_t len = (int64_t)kv->len_of(0, b) + kv->steps_of(b);
        want[b] = {len + 1, len + 1 - kv->vis_len[b], -1};
      }
    if (qc_status s = paged_reserve(kv, want, "qc_decode_graph_launch", (hipStream_t)stream)) return s;
  }
  if (kv->dev_generated != kv->generated) {  // first replay, or ordinary qc_decode steps ran in between
    hipError_t e = qc::launch_counter_update((int32_t*)(kv->arena + c.off_counters()), kv->generated, 0, (hipStream_t)stream);
    if (e != hipSuccess) return fail(QC_EDEVICE, "qc_decode_graph_launch: %s", hipGetErrorString(e));
    kv->dev_generated = kv->generated;
  }
  hipError_t e = hipGraphLaunch(g->exec, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_decode_graph_launch: %s", hipGetErrorString(e));
  kv->generated += 1;
  kv->dev_generated += 1;
  if (g->final_owner >= 0) g->qc->owner = g->final_owner;
  kv->score_workspace = g->score_workspace;
  return QC_OK;
}

void qc_decode_graph_destroy(qc_decode_graph* g) {
  if (!g) return;
  (void)hipGraphExecDestroy(g->exec);
  delete g;
}

// Rows resident in `layer` for sequence b, given how far the current pass has come.
static void rows_of(const qc_kvcache* kv, int layer, int b, int64_t* rk, int64_t* rv) {
  const Config& c = kv->cfg;
  int64_t len = 0;
  if (kv->phase == PH_EMPTY || !kv->live[b]) len = 0;
  else if (kv->joining[b]) len = (kv->phase == PH_PREFILL && layer < kv->next_layer) ? kv->len_of(layer, b) : 0;
  else len = (int64_t)kv->len_of(layer, b) + kv->steps_of(b) + ((kv->phase == PH_DECODE && layer < kv->next_layer) ? 1 : 0);
  *rv = len;
  if (c.gla()) *rk = c.lazy[layer] ? 0 : len;
  else *rk = len ? len - (c.lazy[layer] ? kv->vis_len_of(layer, b) : 0) : 0;
}

qc_status qc_stats(const qc_kvcache* kv, const qc_qcache* qc, qc_stats_t* out) {
  if (!kv || !out) return fail(QC_EINVAL, "qc_stats: null argument");
  const Config& c = kv->cfg;
  memset(out, 0, sizeof(*out));
  const int64_t per_row = (int64_t)c.H * c.D * c.e();
  for (int b = 0; b < kv->batch; ++b) {
    for (int l = 0; l < c.N; ++l) {
      int64_t rk, rv;
      rows_of(kv, l, b, &rk, &rv);
      out->k_bytes += rk * per_row;
      out->v_bytes += rv * per_row;
    }
    if (!kv->live[b]) continue;
    // a sequence waiting for a pass that has not reached layer 0 yet has nothing resident
    const bool started = !kv->joining[b] || kv->phase == PH_PREFILL;
    if (qc && qc->owner >= 0 && started) {
      // rows of the layer that wrote the Q Cache last (after a pruning boundary: of the shortened sequence)
      int64_t q_rows = kv->vis_len_of(qc->owner, b);
      if (c.gla()) {  // one row per position; the row of the token in flight once a block's first layer has run
        q_rows = kv->len_of(qc->owner, b);
        if (!kv->joining[b]) q_rows += kv->steps_of(b);
        if (kv->phase == PH_DECODE && qc->owner < kv->next_layer) q_rows += 1;
      }
      out->q_bytes += q_rows * per_row;
    }
    if (kv->joining[b]) out->tokens += kv->phase == PH_PREFILL ? kv->len0[b] : 0;
    else out->tokens += (int64_t)kv->len0[b] + kv->steps_of(b);
  }
  out->batch = kv->batch;
  out->q_owner = qc ? qc->owner : -1;
  out->generated = kv->generated;
  out->next_layer = kv->next_layer;
  return QC_OK;
}

// ---- query/key projection (Eq. 7: text rows only in a lazy layer) ----------------------------------
qc_status qc_project_qk(const void* x, int64_t x_stride, const void* w_q, const void* w_k, int64_t w_stride,
                        void* q, void* k, int64_t token_stride, int64_t head_stride, int32_t d_model, int32_t n_heads,
                        int32_t head_dim, int32_t batch, const int32_t* cu_seqlens, const int32_t* pos0,
                        const int32_t* vis_start, const int32_t* vis_len, int32_t skip_span,
                        float rope_theta, void* stream) {
  if (!x || !w_q || !w_k || !q || !k || !cu_seqlens) return fail(QC_EINVAL, "qc_project_qk: null argument");
  if (skip_span && (!vis_start || !vis_len)) return fail(QC_EINVAL, "qc_project_qk: skip_span needs the span arrays");
  if (head_dim != 64 && head_dim != 128) return fail(QC_EINVAL, "qc_project_qk: head_dim must be 64 or 128");
  if (batch < 1 || n_heads < 1 || d_model < 64 || d_model % 64) return fail(QC_EINVAL, "qc_project_qk: d_model must be a positive multiple of 64, batch and n_heads positive");
  const int64_t n_out = (int64_t)n_heads * head_dim;
  if (n_out % 256) return fail(QC_EINVAL, "qc_project_qk: n_heads*head_dim must be a multiple of 256");
  if (x_stride < d_model || (x_stride * 2) % 16 || w_stride < d_model || (w_stride * 2) % 16 ||
      head_stride < head_dim || token_stride < head_dim)
    return fail(QC_EINVAL, "qc_project_qk: bad strides");
  if (((uintptr_t)x | (uintptr_t)w_q | (uintptr_t)w_k) & 15) return fail(QC_EINVAL, "qc_project_qk: x and the weights must be 16-byte aligned");
  if ((((uintptr_t)q | (uintptr_t)k) & 15) || (token_stride * 2) % 16 || (head_stride * 2) % 16)
    return fail(QC_EINVAL, "qc_project_qk: q and k and their strides must keep rows 16-byte aligned");
  if (!(rope_theta >= 0.0f) || !std::isfinite(rope_theta)) return fail(QC_EINVAL, "qc_project_qk: bad rope_theta");
  if (cu_seqlens[0] != 0) return fail(QC_EINVAL, "qc_project_qk: cu_seqlens[0] must be 0");
  for (int b = 0; b < batch; ++b) {
    if (cu_seqlens[b + 1] < cu_seqlens[b]) return fail(QC_EINVAL, "qc_project_qk: cu_seqlens must not decrease");
    if (pos0 && pos0[b] < 0) return fail(QC_EINVAL, "qc_project_qk: negative position");
    if (skip_span && (vis_start[b] < 0 || vis_len[b] < 0)) return fail(QC_EINVAL, "qc_project_qk: negative span");
  }
  const int64_t tokens = cu_seqlens[batch];
  if (tokens * x_stride * 2 >= ((int64_t)1 << 31) || n_out * w_stride * 2 >= ((int64_t)1 << 31))
    return fail(QC_EINVAL, "qc_project_qk: x or a weight matrix spans 2 GiB or more");

  qc::ProjectArgs a;
  a.x = x;
  a.w[0] = w_q; a.w[1] = w_k;
  a.out[0] = q; a.out[1] = k;
  a.x_stride = x_stride; a.w_stride = w_stride; a.token_stride = token_stride; a.head_stride = head_stride;
  a.d_model = d_model; a.n_heads = n_heads; a.head_dim = head_dim;
  a.rope_theta = rope_theta;
  a.log2_theta = rope_theta > 0.0f ? std::log2((double)rope_theta) : 0.0;
  // Up to two token ranges per sequence; a launch takes as many sequences as fit its range list.
  int b = 0;
  while (b < batch) {
    memset(&a.segs, 0, sizeof(a.segs));
    int64_t rows = 0;
    while (b < batch && a.segs.n + 2 <= qc::ProjectSegs::N) {
      const int64_t t0 = cu_seqlens[b], len = cu_seqlens[b + 1] - t0, p0 = pos0 ? pos0[b] : 0;
      int64_t cut_lo = p0 + len, cut_hi = p0 + len;   // positions [cut_lo, cut_hi) are skipped
      if (skip_span && vis_len[b] > 0) {
        cut_lo = std::min<int64_t>(std::max<int64_t>(vis_start[b], p0), p0 + len);
        cut_hi = std::min<int64_t>(std::max<int64_t>((int64_t)vis_start[b] + vis_len[b], p0), p0 + len);
      }
      const int64_t ranges[2][2] = {{p0, cut_lo}, {cut_hi, p0 + len}};
      for (auto& r : ranges)
        if (r[1] > r[0]) {
          const int i = a.segs.n++;
          a.segs.tok_start[i] = (int32_t)(t0 + (r[0] - p0));
          a.segs.count[i] = (int32_t)(r[1] - r[0]);
          a.segs.pos_start[i] = (int32_t)r[0];
          rows += r[1] - r[0];
        }
      ++b;
    }
    if (rows == 0) continue;
    // A handful of rows (a decode step) is a matter of streaming the weights once: separate kernel.
    hipError_t e = rows <= 32 ? qc::launch_project_qk_skinny(a, (int)rows, (hipStream_t)stream)
                              : qc::launch_project_qk(a, (int)rows, (hipStream_t)stream);
    if (e != hipSuccess) return fail(QC_EDEVICE, "qc_project_qk: %s", hipGetErrorString(e));
  }
  return QC_OK;
}

// ---- lazy-block selection (Eq. 3 / Eq. 4) --------------------------------------------------------
static int64_t select_score_stride(const Config& c) { return round_up(c.max_seq, 4); }

size_t qc_select_workspace_bytes(const qc_config* cfg) {
  Config c;
  if (!parse_config(cfg, &c)) return 0;
  return (size_t)round_up((int64_t)c.max_batch * c.H * (select_score_stride(c) + 2) * 4, 256);
}

qc_status qc_last_row_attention(qc_kvcache* kv, int32_t layer, const void* q_last, float* probs,
                                int64_t probs_stride, float softmax_scale, void* workspace,
                                size_t workspace_bytes, void* stream) {
  if (!kv) return fail(QC_EINVAL, "qc_last_row_attention: null handle");
  const Config& c = kv->cfg;
  if (layer < 0 || layer >= c.N) return fail(QC_EINVAL, "qc_last_row_attention: layer %d out of range", layer);
  if (c.lazy[layer]) return fail(QC_EINVAL, "qc_last_row_attention: layer %d is lazy and does not hold all of its keys", layer);
  if (!q_last || !probs || !workspace) return fail(QC_EINVAL, "qc_last_row_attention: null tensor or workspace");
  if (((uintptr_t)q_last | (uintptr_t)workspace) & 15) return fail(QC_EINVAL, "qc_last_row_attention: q_last and workspace must be 16-byte aligned");
  if ((uintptr_t)probs & 3) return fail(QC_EINVAL, "qc_last_row_attention: probs must be 4-byte aligned");
  if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return fail(QC_EINVAL, "qc_last_row_attention: bad softmax_scale");
  if (kv->phase != PH_READY && !(kv->phase == PH_PREFILL && layer < kv->next_layer))
    return fail(QC_EORDER, "qc_last_row_attention: needs a prefill pass in which layer %d has run and no decode step in flight", layer);
  int32_t max_len = 0;
  // inside a prefill pass the kernels see the prompts of the pass; afterwards every live sequence
  for (int b = 0; b < kv->batch; ++b) {
    if (kv->phase == PH_PREFILL ? !kv->joining[b] : !kv->live[b]) continue;
    int32_t len = kv->len_of(layer, b) + (kv->phase == PH_PREFILL ? 0 : kv->steps_of(b));
    if (len > max_len) max_len = len;
  }
  if (probs_stride < max_len) return fail(QC_EINVAL, "qc_last_row_attention: probs_stride %lld is shorter than the longest sequence (%d)", (long long)probs_stride, max_len);
  const int64_t need = round_up((int64_t)c.max_batch * c.H * (select_score_stride(c) + 2) * 4, 256);
  if ((int64_t)workspace_bytes < need) return fail(QC_ECAPACITY, "qc_last_row_attention: workspace holds %zu bytes, %lld needed", workspace_bytes, (long long)need);
  qc::SelectArgs a;
  a.lv = make_view(kv, nullptr, layer);
  a.q_last = q_last;
  a.scores = (float*)workspace;
  a.row_stats = (float*)workspace + (int64_t)c.max_batch * c.H * select_score_stride(c);
  a.probs = probs;
  a.probs_stride = probs_stride;
  a.score_stride = (int32_t)select_score_stride(c);
  a.batch = kv->batch; a.n_heads = c.H; a.head_dim = c.D;
  a.generated = kv->phase == PH_PREFILL ? 0 : kv->generated;
  a.scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)c.D);
  hipError_t e = qc::launch_last_row_attention(a, c.dtype, max_len, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_last_row_attention: %s", hipGetErrorString(e));
  return QC_OK;
}

qc_status qc_attention_similarity(const float* probs_m, const float* probs_n, int64_t stride,
                                  int32_t n_samples, const int32_t* lens, float* js_out, float* s_out,
                                  void* stream) {
  if (!probs_m || !probs_n || !lens || !js_out || !s_out) return fail(QC_EINVAL, "qc_attention_similarity: null argument");
  if (n_samples < 1 || stride < 1) return fail(QC_EINVAL, "qc_attention_similarity: needs at least one sample and a positive stride");
  if (((uintptr_t)probs_m | (uintptr_t)probs_n | (uintptr_t)js_out | (uintptr_t)s_out) & 3) return fail(QC_EINVAL, "qc_attention_similarity: pointers must be 4-byte aligned");
  for (int i = 0; i < n_samples; ++i)
    if (lens[i] < 1 || lens[i] > stride) return fail(QC_EINVAL, "qc_attention_similarity: length of sample %d out of range", i);
  for (int first = 0; first < n_samples; first += qc::JsChunk::N) {
    qc::JsChunk ch;
    memset(&ch, 0, sizeof(ch));
    const int count = n_samples - first < qc::JsChunk::N ? n_samples - first : qc::JsChunk::N;
    for (int i = 0; i < count; ++i) ch.len[i] = lens[first + i];
    hipError_t e = qc::launch_js(probs_m, probs_n, stride, first, count, ch, js_out, (hipStream_t)stream);
    if (e != hipSuccess) return fail(QC_EDEVICE, "qc_attention_similarity: %s", hipGetErrorString(e));
  }
  hipError_t e = qc::launch_mean(js_out, n_samples, s_out, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_attention_similarity: %s", hipGetErrorString(e));
  return QC_OK;
}

qc_status qc_lazy_mask_from_similarity(const float* adjacent, int32_t n_layers, float eps, uint8_t* mask_out) {
  if (!mask_out || n_layers < 1 || (n_layers > 1 && !adjacent)) return fail(QC_EINVAL, "qc_lazy_mask_from_similarity: null argument or no layers");
  if (!(eps > 0.0f) || !(eps <= 1.0f)) return fail(QC_EINVAL, "qc_lazy_mask_from_similarity: eps must lie in (0, 1]");
  mask_out[0] = 0;
  for (int i = 1; i < n_layers; ++i) mask_out[i] = adjacent[i - 1] < eps ? 1 : 0;
  return QC_OK;
}

// ---- token-wise pruning between two layers ("Compatibility" paragraph) ---------------------------
qc_status qc_prune_select(const float* scores, int64_t stride, int32_t batch, const int32_t* cu_seqlens,
                          const int32_t* vis_start, const int32_t* vis_len, const int32_t* keep,
                          int32_t* row_map, void* stream) {
  if (!scores || !cu_seqlens || !vis_start || !vis_len || !keep || !row_map) return fail(QC_EINVAL, "qc_prune_select: null argument");
  if (((uintptr_t)scores | (uintptr_t)row_map) & 3) return fail(QC_EINVAL, "qc_prune_select: scores and row_map must be 4-byte aligned");
  if (batch < 1 || stride < 1) return fail(QC_EINVAL, "qc_prune_select: batch and stride must be positive");
  if (cu_seqlens[0] != 0) return fail(QC_EINVAL, "qc_prune_select: cu_seqlens[0] must be 0");
  int64_t survivors = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t len = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
    if (len < 1 || len > stride) return fail(QC_EINVAL, "qc_prune_select: sequence %d has %lld tokens, stride %lld", b, (long long)len, (long long)stride);
    if (vis_start[b] < 0 || vis_len[b] < 0 || (int64_t)vis_start[b] + vis_len[b] > len)
      return fail(QC_EINVAL, "qc_prune_select: span of sequence %d lies outside its %lld tokens", b, (long long)len);
    if (keep[b] < 0 || keep[b] > vis_len[b]) return fail(QC_EINVAL, "qc_prune_select: keep[%d] = %d outside 0..%d", b, keep[b], vis_len[b]);
    survivors += len - vis_len[b] + keep[b];
  }
  if (survivors >= ((int64_t)1 << 31)) return fail(QC_EINVAL, "qc_prune_select: too many tokens");
  int64_t out0 = 0;
  for (int first = 0; first < batch; first += qc::PruneChunk::N) {
    qc::PruneChunk ch;
    memset(&ch, 0, sizeof(ch));
    const int count = batch - first < qc::PruneChunk::N ? batch - first : qc::PruneChunk::N;
    for (int i = 0; i < count; ++i) {
      const int b = first + i;
      ch.tok0[i] = cu_seqlens[b];
      ch.len[i] = cu_seqlens[b + 1] - cu_seqlens[b];
      ch.vis_start[i] = vis_start[b];
      ch.vis_len[i] = vis_len[b];
      ch.keep[i] = keep[b];
      ch.out0[i] = (int32_t)out0;
      out0 += ch.len[i] - vis_len[b] + keep[b];
    }
    hipError_t e = qc::launch_prune_select(scores, stride, first, count, ch, row_map, (hipStream_t)stream);
    if (e != hipSuccess) return fail(QC_EDEVICE, "qc_prune_select: %s", hipGetErrorString(e));
  }
  return QC_OK;
}

qc_status qc_gather_rows(const void* src, int64_t src_stride, const int32_t* row_map, int64_t n_rows,
                         int64_t row_bytes, void* dst, int64_t dst_stride, void* stream) {
  if (n_rows < 0) return fail(QC_EINVAL, "qc_gather_rows: negative row count");
  if (n_rows == 0) return QC_OK;
  if (!src || !row_map || !dst) return fail(QC_EINVAL, "qc_gather_rows: null argument");
  if (row_bytes < 16 || row_bytes % 16 || src_stride < row_bytes || dst_stride < row_bytes || src_stride % 16 || dst_stride % 16)
    return fail(QC_EINVAL, "qc_gather_rows: rows and strides must be multiples of 16 bytes, strides >= row_bytes");
  if ((((uintptr_t)src | (uintptr_t)dst) & 15) || ((uintptr_t)row_map & 3)) return fail(QC_EINVAL, "qc_gather_rows: misaligned pointer");
  if (row_bytes / 16 >= ((int64_t)1 << 31) || n_rows >= ((int64_t)1 << 31)) return fail(QC_EINVAL, "qc_gather_rows: too large");
  hipError_t e = qc::launch_gather_rows(src, src_stride, row_map, n_rows, row_bytes, dst, dst_stride, (hipStream_t)stream);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_gather_rows: %s", hipGetErrorString(e));
  return QC_OK;
}

qc_status qc_prune(qc_kvcache* kv, qc_qcache* qc, const int32_t* keep) {
  if (!kv || !qc || !keep) return fail(QC_EINVAL, "qc_prune: null argument");
  const Config& c = kv->cfg;
  if (!c.same(qc->cfg)) return fail(QC_EINVAL, "qc_prune: handles were created with different configurations");
  if (kv->phase != PH_PREFILL) return fail(QC_EORDER, "qc_prune: allowed only inside a prefill pass, between two layers");
  if (kv->first_late >= 0) return fail(QC_EORDER, "qc_prune: this pass already has a pruning boundary (before layer %d)", kv->first_late);
  if (kv->join_pass || !kv->all_live()) return fail(QC_EORDER, "qc_prune: not available on a batch with free slots or with sequences that joined later");
  if (c.lazy[kv->next_layer]) return fail(QC_EINVAL, "qc_prune: layer %d is lazy: a boundary cannot fall inside a lazy block", kv->next_layer);
  if (c.late_from > 0 && kv->next_layer != c.late_from) return fail(QC_EINVAL, "qc_prune: the configuration sizes the layers from %d on for a boundary there, not before layer %d", c.late_from, kv->next_layer);
  for (int b = 0; b < kv->batch; ++b) {
    if (keep[b] < 0 || keep[b] > kv->vis_len[b]) return fail(QC_EINVAL, "qc_prune: keep[%d] = %d outside 0..%d", b, keep[b], kv->vis_len[b]);
    if (kv->len0[b] - kv->vis_len[b] + keep[b] < 1) return fail(QC_EINVAL, "qc_prune: sequence %d would be left without a token", b);
  }
  kv->vis_len1.assign(keep, keep + kv->batch);
  kv->tok1.assign(kv->batch, 0);
  kv->late_known = false;
  kv->first_late = kv->next_layer;
  return QC_OK;
}

// ---- capacity planning ---------------------------------------------------------------------------
qc_status qc_plan_max_batch(const qc_config* cfg, size_t budget_bytes, int32_t what, int32_t* max_batch) {
  if (!cfg || !max_batch) return fail(QC_EINVAL, "qc_plan_max_batch: null argument");
  if (what <= 0 || (what & ~(QC_PLAN_KV | QC_PLAN_Q | QC_PLAN_WORKSPACE))) return fail(QC_EINVAL, "qc_plan_max_batch: what must be a sum of QC_PLAN_ values");
  qc_config probe = *cfg;
  probe.max_batch = 1;
  Config c;
  if (!parse_config(&probe, &c)) return fail(QC_EINVAL, "qc_plan_max_batch: invalid configuration");
  auto need = [&](int64_t batch) {
    c.max_batch = (int32_t)batch;
    int64_t n = 0;
    if (what & QC_PLAN_KV) n += c.kv_bytes();
    if (what & QC_PLAN_Q) n += c.q_bytes();
    if (what & QC_PLAN_WORKSPACE) n += partial_bytes(c) + score_bytes(c);
    return n;
  };
  // Every size grows with the batch: bisect on the largest batch that fits.
  const int64_t budget = budget_bytes > (size_t)INT64_MAX ? INT64_MAX : (int64_t)budget_bytes;
  int64_t lo = 0, hi = 1;
  while (hi < ((int64_t)1 << 24) && need(hi) <= budget) { lo = hi; hi *= 2; }
  while (hi - lo > 1) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (need(mid) <= budget) lo = mid; else hi = mid;
  }
  *max_batch = (int32_t)lo;
  return QC_OK;
}

qc_status qc_timing_enable(qc_kvcache* kv, int32_t enable) {
  if (!kv) return fail(QC_EINVAL, "qc_timing_enable: null handle");
  kv->timing = enable != 0;
  return QC_OK;
}

qc_status qc_timing_read(qc_kvcache* kv, int32_t which, double* total_ms, int64_t* launches) {
  if (!kv || !total_ms || !launches) return fail(QC_EINVAL, "qc_timing_read: null argument");
  if (which < 0 || which > 2) return fail(QC_EINVAL, "qc_timing_read: which must be 0 (prefill), 1 (decode) or 2 (decode, score-sharing lazy layers)");
  qc::KernelTimer& t = which == 0 ? kv->prefill_timer : which == 1 ? kv->decode_timer : kv->decode_shared_timer;
  hipError_t e = t.read(total_ms, launches);
  if (e != hipSuccess) return fail(QC_EDEVICE, "qc_timing_read: %s", hipGetErrorString(e));
  return QC_OK;
}

qc_status qc_layer_rows(const qc_kvcache* kv, int32_t layer, int64_t* rows_k, int64_t* rows_v) {
  if (!kv || !rows_k || !rows_v) return fail(QC_EINVAL, "qc_layer_rows: null argument");
  if (layer < 0 || layer >= kv->cfg.N) return fail(QC_EINVAL, "qc_layer_rows: layer %d out of range", layer);
  *rows_k = *rows_v = 0;
  for (int b = 0; b < kv->batch; ++b) {
    int64_t rk, rv;
    rows_of(kv, layer, b, &rk, &rv);
    *rows_k += rk;
    *rows_v += rv;
  }
  return QC_OK;
}

qc_status qc_seq_len(const qc_kvcache* kv, int32_t b, int32_t* len) {
  if (!kv || !len) return fail(QC_EINVAL, "qc_seq_len: null argument");
  if (b < 0 || b >= kv->batch) return fail(QC_EINVAL, "qc_seq_len: sequence %d out of range", b);
  *len = kv->settled(b) ? kv->len0[b] + kv->steps_of(b) : 0;
  return QC_OK;
}

qc_status qc_locate(const qc_kvcache* kv, int32_t which, int32_t layer, int32_t b, int32_t h,
                    int32_t pos, int32_t* src_layer, int64_t* byte_offset) {
  if (!kv || !src_layer || !byte_offset) return fail(QC_EINVAL, "qc_locate: null argument");
  const Config& c = kv->cfg;
  if (which != QC_K && which != QC_V) return fail(QC_EINVAL, "qc_locate: which must be QC_K or QC_V");
  if (layer < 0 || layer >= c.N || b < 0 || b >= kv->batch || h < 0 || h >= c.H || pos < 0)
    return fail(QC_EINVAL, "qc_locate: index out of range");
  if (!kv->ragged && pos >= c.max_seq) return fail(QC_EINVAL, "qc_locate: index out of range");
  if (!kv->live[b]) return fail(QC_EINVAL, "qc_locate: slot %d holds no sequence", b);
  const int64_t rb = c.row_bytes();
  if (kv->paged) {
    auto on_page = [&](int pool, int64_t row, int64_t* index) {
      const auto& list = kv->pages[pool][b];
      if (row / qc::kPageRows >= (int64_t)list.size()) return false;
      *index = ((int64_t)list[row / qc::kPageRows] * c.H + h) * qc::kPageRows + row % qc::kPageRows;
      return true;
    };
    int64_t index = 0;
    if (which == QC_V) {
      if (!on_page(0, pos, &index)) return fail(QC_ECAPACITY, "qc_locate: position %d lies on no page of the sequence", pos);
      *src_layer = layer;
      *byte_offset = c.off_v(layer) + index * rb;
      return QC_OK;
    }
    const int32_t s = kv->vis_start[b], vn = kv->vis_len_of(layer, b);
    int src = layer;
    int64_t row = pos;
    if (c.lazy[layer]) {
      if (c.gla() || (pos >= s && pos < s + vn)) src = c.anchor[layer];
      else if (pos >= s + vn) row = pos - vn;
    }
    if (!on_page((c.lazy[src] && !c.gla()) ? 1 : 0, row, &index)) return fail(QC_ECAPACITY, "qc_locate: position %d lies on no page of the sequence", pos);
    *src_layer = src;
    *byte_offset = c.off_k(src) + index * rb;
    return QC_OK;
  }
  // row index of (b, h, row 0) in a region of full-length rows / of a lazy layer's text rows
  auto seq0_of = [&](int l) {
    return kv->ragged ? (int64_t)kv->base_seq[b] * c.H + (int64_t)h * kv->cap_seq[b] : ((int64_t)b * c.H + h) * c.cap_v(l);
  };
  const int64_t seq0 = seq0_of(layer);
  if (pos >= kv->cap_of(layer, b)) return fail(QC_ECAPACITY, "qc_locate: position %d is beyond the sequence's capacity", pos);
  if (which == QC_V) {
    *src_layer = layer;
    *byte_offset = c.off_v(layer) + (seq0 + pos) * rb;
    return QC_OK;
  }
  const int32_t s = kv->vis_start[b], vn = kv->vis_len_of(layer, b);
  int src = layer;
  int64_t row = pos;
  if (c.lazy[layer]) {
    if (c.gla() || (pos >= s && pos < s + vn)) src = c.anchor[layer];
    else if (pos >= s + vn) row = pos - vn;
  }
  const bool text_rows = c.lazy[src] && !c.gla();
  const int64_t cap = text_rows ? kv->cap_text_of(b) : (c.cap_k(src) ? kv->cap_of(src, b) : 0);
  if (row >= cap) return fail(QC_ECAPACITY, "qc_locate: position %d has no row within the layer's capacity", pos);
  const int64_t row0 = !text_rows ? seq0_of(src) : (kv->ragged ? (int64_t)kv->base_text[b] * c.H + (int64_t)h * kv->cap_text[b] : ((int64_t)b * c.H + h) * c.max_text);
  *src_layer = src;
  *byte_offset = c.off_k(src) + (row0 + row) * rb;
  return QC_OK;
}

}  // extern "C"
