/*
 * qcache.h - C ABI of the Lazy Attention / Q Cache attention library for AMD MI355X (gfx950).
 *
 * The library implements the per-layer decoder attention of a multimodal LLM under
 * Visual Lazy Attention (VLA): ordinary layers compute causal softmax attention
 * (paper Eq. 1 for prefill, Eq. 2 for decode); lazy layers inherit the queries and keys
 * of the visual-token span from the first layer of their lazy block through the
 * layer-shared Q Cache (paper Eq. 7 for prefill, Eq. 8 for decode; Q Cache definition at
 * the end of the "Lazy Attention" subsection) and therefore keep only their text keys
 * ("Efficiency Analysis", KV Cache paragraph).
 *
 * Conventions common to every entry point
 *   - Every pointer is tagged below as HOST or DEVICE memory.  The caller owns all device
 *     memory (arenas, Q/K/V/O tensors, workspace) and the stream; the library owns only the
 *     host-side handles.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - Compute entry points are asynchronous on `stream`; host metadata is updated at call time.
 *   - Every call returns a qc_status and never throws or aborts.  Arguments are validated
 *     before anything is launched or changed: on any status other than QC_OK no cache state
 *     (host or device) has changed.  qc_last_error() returns a text for the calling thread's
 *     most recent failure.
 *   - Handles are not thread-safe; use one stream at a time per handle pair.
 *   - Layers must be visited in order 0..n_layers-1 within a prefill pass and within each
 *     decode step: that order is what makes "the Q Cache updates as the block changes"
 *     well defined.
 *   - Multi-head attention with as many K/V heads as query heads; head h of a lazy layer
 *     inherits from head h of its block's first layer.
 *   - Each sequence has one contiguous visual span [vis_start, vis_start + vis_len) at its
 *     true token positions; text may precede and follow it; generated tokens are text.
 *
 * Global Lazy Attention (GLA, qc_config.mode = QC_GLA; paper Eq. 5 for prefill, Eq. 6 for decode)
 * is the paper's coarser variant: a lazy layer inherits the queries and keys of EVERY token from
 * the first layer of its block, computes none of its own and stores no K rows; only its values are
 * its own.  The Q Cache then holds one row per token position (prompt and generated).  Where GLA
 * changes an entry point's behaviour the comment of that entry point says so; everything else
 * (state machine, layouts of the ordinary layers, error behaviour) is shared with VLA.
 */
#ifndef QCACHE_H
#define QCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QC_OK = 0,
  QC_EINVAL = 1,    /* null pointer, bad shape/dtype/stride, span out of range, lazy flag differs from
                       the configured mask, layer 0 marked lazy */
  QC_EORDER = 2,    /* layer called out of sequence; decode before prefill has finished; lazy layer
                       while the Q Cache belongs to another block */
  QC_ECAPACITY = 3, /* sequence, text-row or batch capacity exceeded; arena or workspace too small */
  QC_EDEVICE = 4    /* a HIP call failed (launch error, or an earlier asynchronous fault surfacing) */
} qc_status;

typedef enum { QC_F32 = 0, QC_BF16 = 1 } qc_dtype;
typedef enum { QC_VLA = 0, QC_GLA = 1 } qc_mode;

enum { QC_K = 0, QC_V = 1 };

/* Static description of the decoder stack and cache capacities.
 * lazy_mask: HOST, n_layers bytes, non-zero = lazy layer; copied by the create calls.  Layer 0
 * must be 0.  The first layer of the block a lazy layer l belongs to (its "anchor", l_c in the
 * paper) is the nearest preceding layer whose flag is 0.
 * max_seq  : most positions (prompt + generated) any sequence may reach.
 * max_vis  : most visual tokens in any sequence.
 * max_text : most text rows (prompt text + generated) any sequence may reach; this is the row
 *            capacity of a lazy layer's K cache, which is what makes its allocation smaller.
 * head_dim : 64 or 128.  dtype: element type of Q/K/V/O and of all caches.
 * prune_before_layer, max_seq_late: both 0, or a token-pruning boundary known when the caches are
 *            created: the layers from prune_before_layer on (an ordinary layer, 1..n_layers-1) then get
 *            regions of max_seq_late instead of max_seq rows per head, so that dropping tokens also
 *            shrinks the allocation, not only the rows in use.  qc_prune must then be called at exactly
 *            that boundary (QC_EINVAL elsewhere); without it the later layers still run, within their
 *            smaller capacity.  Not combinable with qc_reset_ragged.
 * mode     : QC_VLA or QC_GLA.  Under QC_GLA max_vis and max_text size nothing (a lazy layer has
 *            no K rows, the Q Cache has max_seq rows) but must still be valid (0..max_seq). */
typedef struct qc_config {
  int32_t n_layers;
  int32_t n_heads;
  int32_t head_dim;
  int32_t dtype; /* qc_dtype */
  int32_t max_batch;
  int32_t max_seq;
  int32_t max_vis;
  int32_t max_text;
  int32_t mode;     /* qc_mode */
  int32_t reserved; /* must be 0 */
  int32_t prune_before_layer; /* 0, or the layer a qc_prune boundary will precede (see max_seq_late) */
  int32_t max_seq_late;       /* 0, or the most positions a sequence may reach in the layers from
                                 prune_before_layer on (1..max_seq) */
  const uint8_t* lazy_mask;
} qc_config;

typedef struct qc_kvcache qc_kvcache; /* opaque host objects: metadata only */
typedef struct qc_qcache qc_qcache;

/* Resident-byte accounting ("Efficiency Analysis", KV Cache paragraph): bytes of cache rows that
 * currently hold data, not capacity.  k_bytes = sum over sequences and layers of
 * (len - lazy[l]*vis_len) * H * D * e; v_bytes = sum of n_layers * len * H * D * e; q_bytes = sum
 * of vis_len * H * D * e once a layer has written the Q Cache (0 before).  tokens = sum of len.
 * Under QC_GLA a lazy layer contributes no k_bytes, and q_bytes counts one row per position the
 * Q Cache holds: len rows, plus the row of the token being decoded once a block's first layer
 * has stored its query in the current step. */
typedef struct qc_stats_t {
  int64_t k_bytes;
  int64_t v_bytes;
  int64_t q_bytes;
  int64_t tokens;
  int32_t batch;
  int32_t q_owner;     /* layer whose visual queries the Q Cache holds, -1 if none */
  int32_t generated;   /* decode steps completed since prefill */
  int32_t next_layer;  /* layer the next qc_prefill / qc_decode call must name */
} qc_stats_t;

/* ---- sizes ------------------------------------------------------------------------------------
 * Exact byte sizes of the caller-allocated device buffers; 0 if the configuration is invalid.
 * K/V arena layout (all offsets in bytes, e = element size):
 *   K region: layers in order, layer l is [max_batch][n_heads][capK(l)][head_dim],
 *             capK(l) = max_text if lazy else max_seq;
 *   V region: layers in order, each [max_batch][n_heads][max_seq][head_dim] (max_seq_late in place of
 *             max_seq, here and in capK, for the layers from prune_before_layer on, if configured);
 *   meta    : at the next multiple of 256: int32 [2][4][max_batch]; block 0 = {first packed token
 *             index, prompt length, vis_start, vis_len} per sequence; block 1 = the same rows as the
 *             layers after a qc_prune boundary see them (zero without one); then 256 bytes of
 *             counters (int32 [0]: decode steps completed, kept for replayed decode graphs); then
 *             int32 [6][max_batch] = {cap_seq, first row, cap_text, first row, vis_len, first row}
 *             per sequence after qc_reset_ragged (zero otherwise); padded to a multiple of 256.
 * Q arena: [max_batch][n_heads][max_vis][head_dim] (one layer's worth, visual rows only).
 * Under QC_GLA: capK(l) = 0 for a lazy layer, and the Q arena is
 *   [max_batch][n_heads][max_seq][head_dim] with row = token position.
 * Decode workspace: split partial results, fp32; under QC_GLA followed (256-byte aligned) by one
 *   fp32 score per position, [max_batch][n_heads][max_seq rounded up to a multiple of 8]. */
size_t qc_kv_arena_bytes(const qc_config* cfg);
size_t qc_q_arena_bytes(const qc_config* cfg);
size_t qc_decode_workspace_bytes(const qc_config* cfg);

/* ---- handles ----------------------------------------------------------------------------------
 * cfg: HOST.  dev_arena: DEVICE, 256-byte aligned, at least the size reported above (else
 * QC_ECAPACITY); it stays owned by the caller and must outlive the handle.  *out receives a new
 * handle on QC_OK.  The create calls touch no device memory and make no HIP call. */
qc_status qc_kvcache_create(const qc_config* cfg, void* dev_arena, size_t arena_bytes, qc_kvcache** out);
qc_status qc_qcache_create(const qc_config* cfg, void* dev_arena, size_t arena_bytes, qc_qcache** out);
void qc_kvcache_destroy(qc_kvcache* kv);
void qc_qcache_destroy(qc_qcache* qc);

/* Start a new batch of `batch` sequences (1..max_batch): lengths 0, Q Cache unowned.
 * vis_start, vis_len: HOST, `batch` entries each (vis_len may be 0: pure-text sequence).
 * zero_fill != 0 additionally clears both arenas on `stream` (fill kernel), so that bytes never
 * written stay zero and whole-arena comparisons are meaningful; with 0 the call is host-only. */
qc_status qc_reset(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                   const int32_t* vis_len, int32_t zero_fill, void* stream);

/* The same with capacities per sequence, for batches of unequal lengths: sequence b may reach
 * cap_seq[b] positions and cap_text[b] text rows, instead of max_seq and max_text for everyone.  The
 * regions keep their sizes; inside each, the sequences' rows follow one another (sequence b's rows of
 * head h start at row (sum of the capacities before b)*n_heads + h*cap[b]; the Q arena is split by
 * vis_len[b] in the same way), so nothing is reserved for lengths a sequence cannot reach.
 * Equal capacities reproduce the layout described under "sizes".
 *   cap_seq, cap_text: HOST, `batch` entries; cap_seq[b] a positive multiple of 8 (or 0: a free slot,
 *   see qc_seq_join), cap_text[b] >= 0 (QC_EINVAL otherwise).  QC_ECAPACITY unless sum cap_seq <= max_batch*max_seq and, under QC_VLA,
 *   sum cap_text <= max_batch*max_text and sum vis_len <= max_batch*max_vis; batch <= max_batch.
 * The capacities are written to the arena's meta region on `stream` (the call is never host-only).
 * A workspace from qc_decode_workspace_bytes / qc_select_workspace_bytes is large enough for any
 * split of the pools.  qc_reset returns to equal capacities. */
qc_status qc_reset_ragged(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                          const int32_t* vis_len, const int32_t* cap_seq, const int32_t* cap_text,
                          int32_t zero_fill, void* stream);

/* ---- sequences joining and leaving a running batch ----------------------------------------------
 * The paper's Table 5 measures the largest batch that fits at a fixed prompt length; a server also
 * has to take a finished sequence out of a running batch and put a new one in its place.  On a batch
 * set up by qc_reset_ragged, `batch` is a number of slots: a slot holds a sequence or is free
 * (cap_seq[b] = 0 at qc_reset_ragged makes slot b free from the start; its other entries are
 * ignored).  Every call that takes per-sequence arrays or [batch]-shaped tensors keeps taking one
 * entry or row per slot; the entries and rows of a free slot are ignored and its `out` rows are
 * left untouched.
 *
 * qc_seq_leave: slot b becomes free and its rows in the three pools can be given to a later join.
 *   Allowed between two decode steps (QC_EORDER otherwise).  Nothing is cleared.
 * qc_seq_join: puts a new sequence into free slot b (QC_EINVAL if taken), with its span and its
 *   capacities as in qc_reset_ragged.  Its rows are placed first-fit: at the lowest row index of
 *   each pool (positions: max_batch*max_seq rows per head-layer; text rows: max_batch*max_text; Q
 *   Cache rows: max_batch*max_vis) where a run of the wanted length is free; QC_ECAPACITY if a pool
 *   has no such run (nothing is moved to make one).  Allowed between two decode steps, and between
 *   qc_reset_ragged and the first qc_prefill.  After joins between decode steps the next calls must
 *   be one prefill pass, qc_prefill for layers 0..n_layers-1, in which the sequences that are
 *   already decoding take no part: their slots have no tokens in cu_seqlens (QC_EINVAL otherwise)
 *   and their caches and lengths stay as they are; decoding then goes on with everybody.
 *   Not available on a batch with a qc_prune boundary, and qc_prune is not available on a batch with
 *   free or later-joined slots (QC_EORDER).  qc_stats_t.generated keeps counting the batch's steps.
 * qc_seq_grow: gives the sequence in slot b other capacities (larger, or smaller down to what it
 *   holds: QC_ECAPACITY below that), between two decode steps.  A pool whose capacity changes gets a new
 *   extent for the sequence, placed first-fit beside every extent in use including the old one, and
 *   the rows the sequence holds are copied there on `stream` (every layer's K and V rows, under QC_GLA
 *   also its Q Cache rows); the old extent is then free.  QC_ECAPACITY if no gap is wide enough; nothing
 *   changes then.  Not available on a batch with a qc_prune boundary.
 * The three calls enqueue their device work on `stream`, ordered like every other call.  A decode
 * graph (qc_decode_graph_create) recorded on the batch stays valid across them: it reads lengths,
 * spans, extents and the step count from device memory.
 * qc_seq_extent: where slot b's rows start in the three pools (first row index as used in the
 *   formula under qc_reset_ragged), and whether the slot holds a sequence; HOST outputs. */
qc_status qc_seq_leave(qc_kvcache* kv, qc_qcache* qc, int32_t b, void* stream);
qc_status qc_seq_join(qc_kvcache* kv, qc_qcache* qc, int32_t b, int32_t vis_start, int32_t vis_len,
                      int32_t cap_seq, int32_t cap_text, void* stream);
qc_status qc_seq_grow(qc_kvcache* kv, qc_qcache* qc, int32_t b, int32_t cap_seq, int32_t cap_text, void* stream);
qc_status qc_seq_extent(const qc_kvcache* kv, int32_t b, int32_t* live, int32_t* base_seq,
                        int32_t* base_text, int32_t* base_vis);

/* ---- paged batches ("Efficiency Evaluation", the maximum-batch paragraph: what limits the batch is the
 * memory the caches of all sequences take together) ------------------------------------------------
 * On a batch set up by qc_reset_paged the rows of a sequence live on pages of QC_PAGE_ROWS rows that it
 * is handed as it needs them, so the arena holds whatever mix of lengths fits in total, a sequence grows
 * without a copy, and a page freed by one sequence serves any other.  The regions keep their sizes and
 * places; each is read as [page][head][QC_PAGE_ROWS][head_dim], and row r of head h of a sequence sits at
 * row index (list[r / QC_PAGE_ROWS]*n_heads + h)*QC_PAGE_ROWS + r % QC_PAGE_ROWS, where `list` is the
 * sequence's page list of the pool the region belongs to: QC_POOL_SEQ (one row per position: V rows of
 * every layer, K rows of ordinary layers, Q Cache rows under QC_GLA; max_batch*max_seq/QC_PAGE_ROWS
 * pages), QC_POOL_TEXT (K rows of lazy layers under QC_VLA; max_batch*max_text/QC_PAGE_ROWS pages) and
 * QC_POOL_VIS (Q Cache rows under QC_VLA; max_batch*max_vis/QC_PAGE_ROWS pages).  One list per sequence
 * and pool serves every layer and head.  The last two pools are in use only under QC_VLA with at least
 * one lazy layer.  Pages are handed out lowest free number first, for the slots in order and for each
 * slot in the order of the pools above: by qc_prefill of layer 0 for the prompts of its pass, and by
 * qc_decode of layer 0 when the row the step appends opens a page (QC_ECAPACITY, and nothing changed,
 * when a pool has too few free pages).  max_seq, max_text and max_vis only size the pools: a sequence
 * may hold any share of a pool, up to 1024 pages (65536 rows) of it.
 *   The configuration must have max_seq, max_text and max_vis multiples of QC_PAGE_ROWS and no
 *   prune_before_layer (QC_EINVAL; qc_page_table_bytes returns 0).
 *   page_lists: DEVICE, 16-byte aligned, at least qc_page_table_bytes(cfg) bytes, owned by the caller and
 *   left alone by it until the next qc_reset*: the lists as the kernels read them.
 *   present: HOST, `batch` flags or NULL (every slot holds a sequence); 0 makes slot b free from the start.
 * Slots work as after qc_reset_ragged: qc_seq_leave gives the sequence's pages back (lowest numbers are
 * handed out first again; nothing is cleared), qc_seq_join takes no capacities (pass 0 for both) and
 * its sequence gets pages when its prefill pass begins.  Not available on a paged batch (QC_EORDER):
 * qc_seq_grow and qc_seq_extent (nothing to grow or to place).  qc_prune works as elsewhere; the layers
 * behind its boundary use the first rows of the same lists, so the pages keep following the unpruned
 * lengths (a configuration with prune_before_layer, which sizes those layers apart, cannot be paged).
 * A decode graph recorded on
 * a paged batch covers max_seq positions (or the next multiple of max_seq above the longest sequence at
 * the time); qc_decode_graph_launch hands out the pages its step opens before it launches the graph, and
 * returns QC_EORDER once a sequence has outgrown what the graph covers (record a new one then).
 * qc_locate answers through the lists.  qc_reset and qc_reset_ragged return to rows in runs.
 * qc_seq_pages: HOST query: *count = pages slot b holds in `pool`; the first min(capacity, *count) page
 *   numbers are written to `pages` if it is not NULL.
 * qc_pool_pages: HOST query: pages of `pool` in all and free at this moment (0 and 0 for a pool the
 *   configuration does not use).  QC_EORDER unless the batch is paged.
 * qc_pages_needed: HOST arithmetic, no handle: pages[QC_POOL_*] = pages a sequence holds in each pool once
 *   `len` positions of it are stored, vis_len of them visual: ceil(len/QC_PAGE_ROWS) of QC_POOL_SEQ,
 *   ceil((len - vis_len)/QC_PAGE_ROWS) of QC_POOL_TEXT and ceil(vis_len/QC_PAGE_ROWS) of QC_POOL_VIS (0 for
 *   a pool the configuration does not use).  With qc_pool_pages this is what admission needs: a sequence
 *   whose prompt and planned decode steps need no more than the free pages can join and will not run dry.
 *   QC_EINVAL for a configuration that cannot be paged or unless 0 <= vis_len <= len. */
#define QC_PAGE_ROWS 64
enum { QC_POOL_SEQ = 0, QC_POOL_TEXT = 1, QC_POOL_VIS = 2 };
size_t qc_page_table_bytes(const qc_config* cfg);
qc_status qc_reset_paged(qc_kvcache* kv, qc_qcache* qc, int32_t batch, const int32_t* vis_start,
                         const int32_t* vis_len, const uint8_t* present, void* page_lists,
                         size_t page_list_bytes, int32_t zero_fill, void* stream);
qc_status qc_seq_pages(const qc_kvcache* kv, int32_t b, int32_t pool, int32_t* pages, int32_t capacity,
                       int32_t* count);
qc_status qc_pool_pages(const qc_kvcache* kv, int32_t pool, int32_t* total, int32_t* free_pages);
qc_status qc_pages_needed(const qc_config* cfg, int32_t len, int32_t vis_len, int32_t* pages /* 3 entries */);

/* ---- prefill: one layer over the packed prompts (paper Eq. 1; Eq. 7 in a lazy layer) -----------
 * q, k, v, out: DEVICE, element (token t, head h, dim d) at t*token_stride + h*head_stride + d
 *   (strides in elements, shared by all four tensors; head_stride >= head_dim, 16-byte aligned
 *   rows; the rows of one sequence must span less than 2 GiB: len * token_stride * e < 2^31).
 *   Sequence b owns tokens cu_seqlens[b] .. cu_seqlens[b+1]-1.
 * cu_seqlens: HOST, batch+1 entries, cu_seqlens[0] = 0.  vis_start, vis_len: HOST, must repeat
 *   the values given to qc_reset.  is_lazy must equal the configured flag of `layer`.
 * softmax_scale: 0 selects 1/sqrt(head_dim).
 * Effects, ordinary layer: out = causal softmax attention of (q, k, v); all k and v rows are
 *   stored; if layer+1 is lazy the span rows of q are stored in the Q Cache, which now belongs
 *   to `layer`.
 * Effects, lazy layer: span rows of q are taken from the Q Cache and span rows of k from the
 *   anchor layer's K cache (the span rows of the q and k arguments are never read and may be
 *   left unwritten by the caller); attention as above with the layer's own v; only text rows of
 *   k are stored (compacted: positions after the span move down by vis_len), all rows of v.
 * Under QC_GLA (paper Eq. 5) an ordinary layer followed by a lazy one stores every row of q in the
 *   Q Cache; a lazy layer takes every row of q from the Q Cache and every row of k from the K cache
 *   of its block's first layer, stores all rows of v and nothing else; its q and k arguments are
 *   ignored and may be NULL. */
qc_status qc_prefill(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                     const void* k, const void* v, void* out, const int32_t* cu_seqlens,
                     int64_t token_stride, int64_t head_stride, const int32_t* vis_start,
                     const int32_t* vis_len, float softmax_scale, void* stream);

/* ---- decode: one generated token per sequence through one layer (paper Eq. 2; Eq. 8 if lazy) ---
 * q, k, v, out: DEVICE, [batch][n_heads][head_dim] contiguous.
 * The new k row is appended at row len (ordinary layer) or len - vis_len (lazy layer), the new
 * v row at row len; the query attends positions 0..len, where a lazy layer reads the span
 * positions from its anchor layer's K cache.  The Q Cache is neither read nor written (the
 * decode query is a text token); qc may be NULL.  After layer n_layers-1 every length grows by 1.
 * workspace: DEVICE, at least qc_decode_workspace_bytes(cfg), contents undefined between calls.
 * Under QC_GLA (paper Eq. 6) qc is required.  An ordinary layer followed by a lazy one also stores
 *   its query at row len of the Q Cache, which from then on belongs to it, and its scaled scores
 *   q.k of positions 0..len in the workspace.  A lazy layer attends with that query and with the
 *   K cache of its block's first layer, that is with exactly those scores: it reads them back
 *   instead of the keys (the product of Eq. 6 is formed once per block), streams only its own V
 *   cache and appends only its v row; its q and k arguments are ignored and may be NULL.  The
 *   layers of a block must therefore be given the same workspace on the same stream (QC_EINVAL
 *   otherwise), and nothing else may write to it between them.  QC_EORDER if the Q Cache belongs
 *   to another block. */
qc_status qc_decode(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                    const void* k, const void* v, void* out, const int32_t* vis_start,
                    const int32_t* vis_len, float softmax_scale, void* workspace,
                    size_t workspace_bytes, void* stream);

/* qc_decode_split: HOST arithmetic, no handle: how an ordinary qc_decode call (not a recorded one) divides
 * the key positions 0..max_len of `pairs` = batch * n_heads (sequence, head) pairs among workgroups on a
 * device of `compute_units` units: *chunk_keys positions per workgroup, *chunks workgroups for the longest
 * sequence (1: no split, no merge pass).  Stated here because the decode rate depends on it: the workgroups
 * are spread as evenly over the compute units as the pair count allows.  QC_EINVAL for non-positive
 * arguments (max_len may be 0). */
qc_status qc_decode_split(int32_t pairs, int32_t max_len, int32_t compute_units, int32_t* chunk_keys, int32_t* chunks);

/* ---- decode for callers that cannot allocate ------------------------------------------------------
 * For callers that must not call hipMalloc (code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation) and therefore cannot bring a workspace: qc_decode with the
 * workspace replaced by an array of QC_STATIC_SCRATCH_BYTES bytes that the library itself holds in
 * device memory, one copy per GPU, from load until the process ends.  Same kernels, same results,
 * same arguments and errors as qc_decode otherwise.  The call allocates nothing, on the host or on
 * the device (leave qc_timing_enable off: event creation allocates).
 *   QC_ECAPACITY if the call needs more scratch than the array holds.  Under QC_VLA a call needs at
 *   most 2047 partial results of head_dim + 2 floats (about 1 MiB), so it always fits; under QC_GLA
 *   it needs qc_decode_workspace_bytes(cfg), which fits only small configurations.
 *   The device that is current at the call must be the one `stream` and the arenas belong to.
 *   All calls on one GPU share that GPU's array, from every handle and every thread: calls that
 *   overlap on one GPU (two streams, two threads) race.  Nothing in it has to start at zero: each
 *   call writes every partial result it later reads.  Under QC_GLA the layers of a block must all use
 *   this entry point (or all qc_decode with one workspace). */
enum { QC_STATIC_SCRATCH_BYTES = 4194304 };
qc_status qc_decode_static(qc_kvcache* kv, qc_qcache* qc, int32_t layer, int32_t is_lazy, const void* q,
                           const void* k, const void* v, void* out, const int32_t* vis_start,
                           const int32_t* vis_len, float softmax_scale, void* stream);

/* ---- a whole decode step as one replayable HIP graph --------------------------------------------
 * At batch sizes where a layer call lasts a few microseconds, a decode step is bound by the gaps
 * between dependent launches on a stream (about 4 us each here); replayed from a graph the same
 * launches follow each other in under 2 us.  qc_decode_graph_create records the n_layers calls
 * qc_decode would make for one step, in layer order, into a HIP graph: same kernels, same
 * arithmetic, but they take the number of completed steps from a counter in the arena's meta
 * region (which the graph itself advances) and every per-sequence integer from device memory, so
 * one graph serves step after step, and any later batch of the same size on these handles.
 *   q, k, v, out: HOST arrays of n_layers DEVICE pointers, [batch][n_heads][head_dim] each: the
 *     buffers layer l reads and writes at EVERY replay (the caller refills q/k/v between replays; under
 *     QC_GLA the q and k entries of lazy layers are ignored and may be NULL).
 *   workspace: as for qc_decode, sized by qc_decode_workspace_bytes; used by every replay.
 * Requires a finished prefill pass with no decode step in flight (QC_EORDER otherwise).  Creation
 * records on a stream of its own and instantiates the graph: it allocates (host and runtime memory)
 * and must not itself be called under stream capture.
 * qc_decode_graph_launch replays the step on `stream` and moves the bookkeeping forward exactly as
 * n_layers qc_decode calls would; steps made with qc_decode and replays may alternate.  QC_EORDER if
 * no step may start now, or if the cache holds another number of sequences or another pruning
 * boundary than at creation; QC_ECAPACITY as qc_decode.  The graph holds the device pointers given
 * at creation; it must be destroyed before the handles it was made from. */
typedef struct qc_decode_graph qc_decode_graph;
qc_status qc_decode_graph_create(qc_kvcache* kv, qc_qcache* qc, const void* const* q, const void* const* k,
                                 const void* const* v, void* const* out, float softmax_scale, void* workspace,
                                 size_t workspace_bytes, qc_decode_graph** out_graph);
qc_status qc_decode_graph_launch(qc_decode_graph* graph, void* stream);
void qc_decode_graph_destroy(qc_decode_graph* graph);

/* ---- bookkeeping queries (host only, no HIP call) ---------------------------------------------- */
qc_status qc_stats(const qc_kvcache* kv, const qc_qcache* qc, qc_stats_t* out);
/* Rows of layer `layer` currently resident, summed over the batch. */
qc_status qc_layer_rows(const qc_kvcache* kv, int32_t layer, int64_t* rows_k, int64_t* rows_v);
qc_status qc_seq_len(const qc_kvcache* kv, int32_t b, int32_t* len);
/* Where layer `layer` reads the key (which = QC_K) or value (QC_V) of position `pos` of head h of
 * sequence b: *src_layer is `layer` itself, or the anchor layer for a span position of a lazy
 * layer; *byte_offset is the offset of that row in the K/V arena.  pos must be < max_seq.
 * Under QC_GLA every key position of a lazy layer resolves to the block's first layer. */
qc_status qc_locate(const qc_kvcache* kv, int32_t which, int32_t layer, int32_t b, int32_t h,
                    int32_t pos, int32_t* src_layer, int64_t* byte_offset);

/* ---- query/key projection feeding qc_prefill and qc_decode (paper Eq. 7: X_[T] W_Q, X_[T] W_K) -----
 * q[t][h][:] = rope(x[t] . W_Q[h*D .. h*D+D-1][:]) and the same for k with W_K, for every token t of the
 * batch that is not skipped.  With skip_span != 0 (a lazy layer under Visual Lazy Attention) the
 * tokens inside each sequence's visual span are neither computed nor written: this is the projector
 * work the method omits ("Efficiency Analysis", FLOPs and Latency).  bf16 only.
 *   x: DEVICE, bf16, token t at x + t*x_stride (elements), d_model values; 16-byte aligned rows.
 *   w_q, w_k: DEVICE, bf16, [n_heads*head_dim] rows (row = output feature) of d_model values, row r at
 *     w + r*w_stride (elements), 16-byte aligned rows.  q, k: DEVICE, bf16, element (t, h, d) at t*token_stride + h*head_stride + d: the
 *     tensors qc_prefill / qc_decode take.
 *   cu_seqlens: HOST, batch+1 entries: sequence b owns tokens cu_seqlens[b] .. cu_seqlens[b+1]-1.
 *   pos0: HOST, batch entries or NULL (= all 0): position of sequence b's first token (0 for a prompt,
 *     the current length for a decode step, where every sequence contributes one token).
 *   vis_start, vis_len: HOST, spans in positions; read only if skip_span != 0.
 *   rope_theta: base of the rotary embedding applied at each token's position (rotate-half
 *     convention: element d < D/2 of a head pairs with d + D/2, angle pos * theta^(-2d/D));
 *     0 = no rotation.
 * Limits (QC_EINVAL): head_dim 64 or 128; d_model a multiple of 64; n_heads*head_dim a multiple of
 * 256; tokens*x_stride*2 and n_heads*head_dim*w_stride*2 below 2^31 bytes. */
qc_status qc_project_qk(const void* x, int64_t x_stride, const void* w_q, const void* w_k, int64_t w_stride,
                        void* q, void* k, int64_t token_stride, int64_t head_stride, int32_t d_model, int32_t n_heads,
                        int32_t head_dim, int32_t batch, const int32_t* cu_seqlens, const int32_t* pos0,
                        const int32_t* vis_start, const int32_t* vis_len, int32_t skip_span,
                        float rope_theta, void* stream);

/* ---- lazy-block selection (paper Eq. 3 and Eq. 4; offline analysis, not part of serving) ---------
 * Run the model with a mask of zeros (every layer ordinary), and after the prefill pass ask every
 * layer for the last row of its attention matrix:
 * qc_last_row_attention: probs[b][pos], pos = 0..len_b-1, = mean over heads of
 *   Softmax(q_last[b][h] . K^layer[b][h][0..len_b-1] * scale) (the paper averages over heads; base of
 *   the softmax as in qc_prefill, softmax_scale 0 selects 1/sqrt(head_dim)).
 *   q_last: DEVICE, [batch][n_heads][head_dim], element type of the configuration: the query of each
 *   sequence's last token at `layer`.  probs: DEVICE, fp32, row b starts at b*probs_stride
 *   (probs_stride >= longest sequence); entries at and beyond len_b are not written.
 *   workspace: DEVICE, at least qc_select_workspace_bytes(cfg).  Requires a finished prefill pass, or
 *   an open one in which `layer` has already run (QC_EORDER otherwise; not between the layers of a
 *   decode step), and an ordinary `layer` (QC_EINVAL: a lazy layer does not hold all its keys).
 * qc_attention_similarity: js_out[i] = JS(probs_m row i, probs_n row i) over lens[i] entries, in nats
 *   (JS = (KL(p||m) + KL(q||m))/2, m = (p+q)/2, natural logarithm so that JS <= ln 2, terms with zero
 *   probability contribute zero), and
 *   *s_out = their mean over the n_samples rows = S(l_m, l_n) of Eq. 3.  probs_m, probs_n, js_out,
 *   s_out: DEVICE fp32; lens: HOST, n_samples entries, each 1..stride.
 * qc_lazy_mask_from_similarity (host only): Eq. 4.  adjacent[i] = S(l_i, l_i+1), i = 0..n_layers-2;
 *   layer i >= 1 becomes lazy exactly when adjacent[i-1] < eps, so that blocks are the maximal runs
 *   whose adjacent pairs all stay below eps and every block starts with an ordinary layer.
 *   0 < eps <= 1 (QC_EINVAL otherwise).  adjacent, mask_out: HOST. */
size_t qc_select_workspace_bytes(const qc_config* cfg);
qc_status qc_last_row_attention(qc_kvcache* kv, int32_t layer, const void* q_last, float* probs,
                                int64_t probs_stride, float softmax_scale, void* workspace,
                                size_t workspace_bytes, void* stream);
qc_status qc_attention_similarity(const float* probs_m, const float* probs_n, int64_t stride,
                                  int32_t n_samples, const int32_t* lens, float* js_out, float* s_out,
                                  void* stream);
qc_status qc_lazy_mask_from_similarity(const float* adjacent, int32_t n_layers, float eps, uint8_t* mask_out);

/* ---- token-wise pruning on top of Lazy Attention ("Compatibility" paragraph and its table) ---------
 * The paper states that a token pruning method (it names FastV) can run on a model that already uses
 * Lazy Attention and says no more.  Here pruning is one boundary inside a prefill pass: the layers
 * before it see the whole prompt, the layers after it, in this pass and in every later decode step,
 * see each sequence without the visual tokens that were dropped.  For those later layers the
 * sequence simply is shorter: their cache rows, their span [vis_start, vis_start + keep) and their
 * lazy blocks are those of the shortened sequence, so a boundary may not fall inside a lazy block.
 *
 * qc_prune_select: which tokens survive.  scores: DEVICE fp32, row b at b*stride, entry p ranks
 *   position p of sequence b (the rows qc_last_row_attention writes serve as they are: the attention
 *   the last prompt token pays to every position, which is the ranking FastV-style methods use).  Of
 *   each sequence's span the keep[b] positions of highest score survive, a tie going to the lower
 *   position (NaN scores: unspecified choice); text tokens always survive.  row_map: DEVICE int32,
 *   sum over b of (len_b - vis_len[b] + keep[b]) entries: the packed-prompt index
 *   (cu_seqlens[b] + position) of every surviving token, sequence after sequence in position order.
 *   cu_seqlens, vis_start, vis_len, keep: HOST.  QC_EINVAL unless 0 <= keep[b] <= vis_len[b] and the
 *   span lies inside the sequence and stride >= every length.
 * qc_gather_rows: dst row i = src row row_map[i], i = 0..n_rows-1: drops the pruned rows of any packed
 *   per-token tensor (hidden states, or q/k/v).  src, dst: DEVICE, rows of row_bytes bytes (a multiple
 *   of 16) at multiples of src_stride / dst_stride bytes (multiples of 16, >= row_bytes), 16-byte
 *   aligned, not overlapping.  row_map: DEVICE int32, entries must index rows of src (not checked).
 * qc_prune: moves the boundary into the cache state.  Allowed once per prefill pass, after at least
 *   one layer has run and before the last (QC_EORDER otherwise), and only if the next layer is an
 *   ordinary one (QC_EINVAL).  keep: HOST, batch entries, 0 <= keep[b] <= vis_len[b], and every
 *   sequence must keep at least one token (QC_EINVAL).  Host only.
 *   From then on every call that names a layer at or after the boundary takes vis_len = keep in its
 *   span arrays and, in qc_prefill, cu_seqlens of the shortened prompts (len_b - vis_len[b] + keep[b]
 *   tokens each); calls naming earlier layers keep the original values.  qc_seq_len keeps reporting
 *   the unpruned length; qc_stats, qc_layer_rows and qc_locate answer per layer.  qc_reset ends it. */
qc_status qc_prune_select(const float* scores, int64_t stride, int32_t batch, const int32_t* cu_seqlens,
                          const int32_t* vis_start, const int32_t* vis_len, const int32_t* keep,
                          int32_t* row_map, void* stream);
qc_status qc_gather_rows(const void* src, int64_t src_stride, const int32_t* row_map, int64_t n_rows,
                         int64_t row_bytes, void* dst, int64_t dst_stride, void* stream);
qc_status qc_prune(qc_kvcache* kv, qc_qcache* qc, const int32_t* keep);

/* ---- capacity planning (the maximum-batch comparison of the "Efficiency Evaluation" paragraph) ----
 * Largest max_batch for which the buffers named by `what` (a sum of the QC_PLAN_ values), sized for
 * cfg with that max_batch, fit together into budget_bytes; cfg->max_batch itself is ignored.  0 if
 * not even one sequence fits.  Host only.  QC_EINVAL for an invalid configuration or what == 0. */
enum { QC_PLAN_KV = 1, QC_PLAN_Q = 2, QC_PLAN_WORKSPACE = 4 };
qc_status qc_plan_max_batch(const qc_config* cfg, size_t budget_bytes, int32_t what, int32_t* max_batch);

/* ---- optional instrumentation ------------------------------------------------------------------
 * While enabled, qc_prefill and qc_decode record a pair of HIP events on the call's stream around
 * their dominant kernel (prefill: the attention kernel; decode: the kernel that streams the caches,
 * not the small merge pass).  qc_timing_read waits for the recorded events of one kind (which = 0
 * prefill, 1 decode, 2 decode calls of lazy layers under QC_GLA, which run the score-sharing
 * variant of the kernel and are not counted under 1), returns the sum of their durations and the
 * number of launches, and starts over.  At most 131072 launches are kept between reads; further ones are not timed.  Event
 * creation allocates: leave this off on paths that must not. */
qc_status qc_timing_enable(qc_kvcache* kv, int32_t enable);
qc_status qc_timing_read(qc_kvcache* kv, int32_t which, double* total_ms, int64_t* launches);

const char* qc_status_str(qc_status s);
const char* qc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QCACHE_H */
