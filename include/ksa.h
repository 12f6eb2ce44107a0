/*
 * ksa.h -- C ABI of the MI355X (gfx950) Kwai Summary Attention hot path.
 *
 * The library computes  O = softmax(Q K^T * scale + M_KSA) V  (the KSA attention formula of the
 * paper's distillation section) over the augmented sequence of section 2.2.1 / Eq. 1, in which
 * n_summary summary tokens follow every chunk of chunk_len text tokens, with the visibility M_KSA
 * of section 2.2.2 / Eq. 3:
 *   - a text token in chunk j sees the text of chunks max(0, j - window_chunks) .. j up to itself,
 *     and the summary tokens of chunks 0 .. j - window_chunks - 1 (summaries of chunks still inside
 *     the window are not visible);
 *   - a summary token sees the text of its own chunk, itself, and the earlier summary tokens of
 *     its own chunk (KSA_FLAG_SUMMARY_SELF_ONLY drops the earlier siblings).
 * The paper has one summary token per chunk (n_summary = 1, chunk_len = k); n_summary > 1 with
 * compress_ratio = chunk_len / n_summary is this library's generalisation of it.
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary.  Every function returns a ksa_status (0 = OK).
 *   - "host" / "device" is stated for every pointer.  The caller owns every tensor and the stream;
 *     the library owns the opaque ksa_layout until ksa_layout_destroy.
 *   - Argument validation happens before any HIP call, so bad arguments are reported even on a
 *     machine without a GPU.  Inputs are never written.
 *   - Kernels are enqueued on the caller's HIP stream and are asynchronous; nothing synchronises.
 *   - Tensor element type is bf16 (q, k, v, o, caches); log-sum-exp outputs are fp32.
 *     Scores and accumulators are fp32; P is rounded to bf16 before the P V product in prefill.
 */
#ifndef KSA_H_
#define KSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ksa_status {
    KSA_OK = 0,
    KSA_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, inconsistent parameters, ... */
    KSA_ERR_UNSUPPORTED = -2,        /* head_dim / group size the kernels were not built for        */
    KSA_ERR_WORKSPACE_TOO_SMALL = -3,
    KSA_ERR_HIP = -4,                /* a HIP runtime call failed (no device, launch error, OOM)    */
    KSA_ERR_OUT_OF_RANGE = -5,       /* an index argument lies outside the layout                   */
    KSA_ERR_SCRATCH_LIMIT = -6,      /* the problem needs more than the library's static scratch buffer holds */
    KSA_ERR_OUT_OF_MEMORY = -7       /* a host allocation failed while building a layout            */
} ksa_status;

#define KSA_FLAG_SUMMARY_SELF_ONLY 1u /* summary rows see, among summaries, only themselves */

/* Problem statement, in the paper's terms (Eq. 1-3; Table "model_config"). */
typedef struct ksa_params {
    int32_t batch;           /* B                                                               */
    int32_t n_text;          /* n: text tokens per sequence (prefill); context capacity (decode) */
    int32_t chunk_len;       /* c: text tokens per chunk (an incomplete last chunk has no summaries) */
    int32_t n_summary;       /* m: summary tokens after each chunk (paper: 1); 0 = no summaries  */
    int32_t compress_ratio;  /* k = c / m; validated (k * m == c) when m > 0, ignored when m == 0 */
    int32_t window_chunks;   /* C >= 0: previous chunks whose text stays visible (Eq. 2 / Eq. 3)  */
    int32_t n_q_heads;       /* Hq, a multiple of n_kv_heads (GQA: query head h reads KV head h / (Hq/Hkv)) */
    int32_t n_kv_heads;      /* Hkv                                                              */
    int32_t head_dim;        /* d: 64 or 128                                                     */
    float softmax_scale;     /* <= 0 selects 1/sqrt(head_dim)                                    */
    uint32_t flags;          /* KSA_FLAG_*                                                       */
} ksa_params;

typedef struct ksa_layout ksa_layout;

/* Key-tile kinds reported by ksa_layout_tile_pairs. */
#define KSA_TILE_FULL 0    /* every (query row, key) pair of the tile pair is visible: no mask applied */
#define KSA_TILE_MASKED 1  /* per-element bounds are applied                                          */
/* Index spaces of a tile: compact text index i (0..n-1) or compact summary ordinal u (0..J*m-1). */
#define KSA_SPACE_TEXT 0
#define KSA_SPACE_SUMMARY 1

/*
 * ksa_build_layout: the integer side of Eq. 1 and Eq. 3 -- index maps of the augmented sequence,
 * per-row visible ranges, and the block-sparse schedule that lists, for every query tile, only the
 * key tiles that hold at least one visible pair (section 2.3: only non-zero block pairs are loaded).
 * Pure host work; touches no GPU.  *out (host) receives a new layout owned by the library.
 * Errors: INVALID_ARG for bad params (see ksa_params), UNSUPPORTED for head_dim not in {64, 128},
 * OUT_OF_MEMORY if the host cannot hold the schedule.
 */
int ksa_build_layout(const ksa_params *params /*host*/, ksa_layout **out /*host*/);
void ksa_layout_destroy(ksa_layout *layout);

/*
 * Copies the schedule to the current HIP device (one hipMalloc + one hipMemcpy).  ksa_prefill_fwd
 * does this itself on first use; calling it ahead keeps the first timed call allocation-free.  After it,
 * ksa_prefill_fwd and ksa_prefill_bwd enqueue kernels only (no allocation, memset or synchronisation) and may be
 * captured into a HIP graph.
 */
int ksa_layout_upload(ksa_layout *layout);

/* Rows of the augmented sequence (Eq. 1) of n_text text tokens under params' chunk_len and n_summary:
 * (n_text / c)(c + m) + n_text mod c (params->n_text itself is not used).  For sizing the q / k / v tensors. */
int ksa_augmented_rows(const ksa_params *params /*host*/, int64_t n_text, int64_t *rows /*host*/);

/* ---- introspection (host arrays, caller-allocated) used by the bit-exact layout tests ---------- */

/* L = (n/c) * (c+m) + n mod c augmented rows (an incomplete last chunk has text rows only), J = n/c whole chunks,
 * the query / key tile heights of the schedule, and the number of query heads (of one KV head) a prefill
 * workgroup handles together: 1, 2 or 4, with q_tile_rows * heads_per_workgroup = 256.  Any pointer may be NULL. */
int ksa_layout_dims(const ksa_layout *layout, int64_t *aug_len, int32_t *n_chunks, int32_t *q_tile_rows,
                    int32_t *k_tile_rows, int32_t *heads_per_workgroup);
/* Eq. 1 index maps.  aug_chunk, aug_is_summary, position_ids: [L]; text_to_aug: [n]; summary_to_aug: [J*m].
 * position_ids gives a summary token the position of its chunk's last text token (section 2.2.1).
 * Any pointer may be NULL to skip that array. */
int ksa_layout_index_maps(const ksa_layout *layout, int32_t *aug_chunk, uint8_t *aug_is_summary,
                          int32_t *position_ids, int32_t *text_to_aug, int32_t *summary_to_aug);
/* Visible ranges of augmented row aq: out = {summary_lo, summary_hi, text_lo, text_hi}: summary ordinals
 * [summary_lo, summary_hi) and text indices [text_lo, text_hi) are visible, nothing else. */
int ksa_layout_row_ranges(const ksa_layout *layout, int64_t aq, int32_t out[4]);
/* Row aq of M_KSA expanded from the row ranges: row_out[ak] = 1 iff visible, ak in [0, L). */
int ksa_layout_mask_row(const ksa_layout *layout, int64_t aq, uint8_t *row_out);
/*
 * The (query tile, key tile) pairs the prefill kernel visits, for one (batch, head).  Pass NULL arrays to
 * get *n_pairs only.  Pair x: query rows [q_begin[x], q_begin[x]+q_count[x]) of space q_space[x], key rows
 * [k_begin[x], k_begin[x]+k_count[x]) of space k_space[x], kind[x] = KSA_TILE_FULL or KSA_TILE_MASKED.
 */
int ksa_layout_tile_pairs(const ksa_layout *layout, int64_t *n_pairs, uint8_t *q_space, int32_t *q_begin,
                          int32_t *q_count, uint8_t *k_space, int32_t *k_begin, int32_t *k_count, uint8_t *kind);

/*
 * The prefill launch order: entry x is what workgroup x does -- the query tile (q_space[x], q_begin[x]) for
 * batch[x] and the query heads q_head[x] .. q_head[x] + heads_per_workgroup - 1 (ksa_layout_dims);
 * q_begin[x] = -1 marks a padding workgroup that does nothing.  Consecutive workgroup
 * ids are dealt to the 8 XCDs round-robin, so entries congruent mod 8 share an L2.  NULL arrays: count only.
 */
int ksa_layout_launch_order(const ksa_layout *layout, int64_t *n_entries, uint8_t *q_space, int32_t *q_begin,
                            int32_t *batch, int32_t *q_head);

/* ---- prefill ------------------------------------------------------------------------------------ */

/*
 * Bytes of device scratch memory ksa_prefill_fwd needs for this layout (0 for a NULL layout): room for a
 * key-major copy of V, batch * n_kv_heads * head_dim * (n_text + n_summary_tokens, each rounded up to 64) bf16,
 * followed by the largest squared K row norm per (batch, KV head, 64-key tile) and per (batch, KV head), fp32.
 */
size_t ksa_prefill_workspace_bytes(const ksa_layout *layout);

/*
 * ksa_prefill_fwd: attention output of all L augmented rows (text and summary rows alike),
 *   O = softmax(Q K^T * scale + M_KSA) V with the visibility of Eq. 3 over the sequence of Eq. 1.
 *   q [B, L, Hq, d], k and v [B, L, Hkv, d], o [B, L, Hq, d]: device, bf16, last dim contiguous;
 *   *_strides = {batch, row, head} strides in elements; NULL = contiguous in the order above.
 *   lse: device fp32 [B, Hq, L] contiguous, natural-log sum-exp of the scaled visible scores; may be NULL.
 *   workspace: device memory, 16-byte aligned, at least ksa_prefill_workspace_bytes(layout) bytes, owned by the
 *   caller; the call overwrites it (a preparation pass re-lays V out key-major for the main kernel and takes the
 *   largest K row norm of every KV head, from which the main kernel derives a fixed softmax reference per row
 *   wherever |q| max |k| * scale is small enough to rule out overflow and underflow; other rows keep a running
 *   maximum) and needs it until the work enqueued on `stream` has finished.  Calls that share a workspace must be
 *   stream-ordered.
 *   stream: hipStream_t (NULL = default stream).
 * The main kernel walks the layout's schedule: bf16 MFMA for Q K^T and P V, fp32 online softmax.
 * Value range: the weights of a row are kept within [2^-88, 2^32] relative to its reference and summed in fp32, so
 * the output is finite as long as max |v| times the number of visible keys stays below 2^95.
 * Errors: INVALID_ARG (null tensors or workspace, misaligned pointers: 16-byte alignment required),
 * WORKSPACE_TOO_SMALL, HIP.
 */
int ksa_prefill_fwd(ksa_layout *layout, const void *q, const void *k, const void *v, void *o, float *lse,
                    const int64_t q_strides[3], const int64_t kv_strides[3], const int64_t o_strides[3],
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * ksa_prefill_relayout_v: only the preparation pass of ksa_prefill_fwd, run on v alone: the key-major copy of V
 * goes into the workspace (same v, kv_strides, workspace and error rules as there), and the row-norm part of the pass
 * reads v in place of k (same shape, same cost; its result is not used by anything).  ksa_prefill_fwd always runs the
 * pass itself; this entry point exists so that the pass and the main kernel can be timed apart.
 */
int ksa_prefill_relayout_v(ksa_layout *layout, const void *v, const int64_t kv_strides[3], void *workspace,
                           size_t workspace_bytes, void *stream);

/* Bytes of device scratch memory ksa_prefill_bwd needs for this layout (0 for a NULL layout): two fp32 per
 * (batch, query head, row), the rows of each index space (text, summary) rounded up to a multiple of 64. */
size_t ksa_prefill_bwd_workspace_bytes(const ksa_layout *layout);

/*
 * ksa_prefill_bwd: gradients of ksa_prefill_fwd's output with respect to q, k and v for an upstream gradient
 * d_o = dLoss/dO (the paper's block-sparse kernel is its training kernel too, section 2.3, Kernel Design; the formulas are
 * the derivative of the attention definition):
 *   P = exp(Q K^T * scale - lse) on visible pairs (Eq. 3), dV = P^T dO, dS = P o (dO V^T - rowsum(dO o O)),
 *   dQ = scale * dS K, dK = scale * dS^T Q; with grouped heads a KV head sums over its query heads.
 *   q, k, v, o, lse: what ksa_prefill_fwd read and wrote (same shapes, o_strides for o AND d_o; lse is required);
 *   d_o [B, L, Hq, d], dq [B, L, Hq, d], dk and dv [B, L, Hkv, d]: device, bf16, last dim contiguous;
 *   dq_strides for dq, dkv_strides for dk and dv ({batch, row, head}, NULL = contiguous).  Every row of dq, dk
 *   and dv is written.
 *   workspace: device memory, 16-byte aligned, at least ksa_prefill_bwd_workspace_bytes(layout) bytes, owned by
 *   the caller, overwritten, needed until the work enqueued on `stream` has finished.
 * No atomics: results do not depend on the launch order.  head_dim 64 or 128.  The row strides of q, k / v and d_o
 * must be positive, and the rows that 64 consecutive text (or summary) positions span in the augmented sequence must
 * lie within 4 GiB of each other in each of these tensors (a chunk_len of 4096 at a row stride of 8 KiB still does);
 * else UNSUPPORTED.
 * Errors: INVALID_ARG (null or misaligned pointers, bad strides), WORKSPACE_TOO_SMALL, UNSUPPORTED, HIP.
 */
int ksa_prefill_bwd(ksa_layout *layout, const void *q, const void *k, const void *v, const void *o, const float *lse,
                    const void *d_o, void *dq, void *dk, void *dv, const int64_t q_strides[3],
                    const int64_t kv_strides[3], const int64_t o_strides[3], const int64_t dq_strides[3],
                    const int64_t dkv_strides[3], void *workspace, size_t workspace_bytes, void *stream);

/* ---- decode over the summary KV cache (section 2.3.1) ------------------------------------------ */

/*
 * Cache geometry of this library (one K and one V tensor, device bf16, [B, Hkv, cache_rows, d]):
 *   rows [0, S_cap)                         Summary Token Buffer: summary ordinal u = j*m + slot at row u;
 *   rows [S_cap, S_cap + (C+1)*c)           text ring: text index i of chunk j = i / c at row
 *                                           S_cap + (j mod (C+1)) * c + i mod c.
 * S_cap = (n_text / c) * m.  The chunk being written overwrites, in place, the chunk that just left the
 * window, so no copy is needed when a chunk completes.  Summaries of in-window chunks are resident in the
 * buffer but are not read (Eq. 3).
 */
int ksa_cache_geometry(const ksa_params *params /*host*/, int32_t *summary_capacity, int32_t *cache_rows);
/* Cache row of text index i / of summary ordinal u (host helpers for packing a cache). */
int ksa_cache_text_row(const ksa_params *params, int64_t text_index, int32_t *row);
int ksa_cache_summary_row(const ksa_params *params, int64_t summary_ordinal, int32_t *row);
/*
 * Rows a new text token at text index pos reads: up to three (offset, length) row ranges, in the order
 * summaries, ring part 1, ring part 2; unused ranges have length 0.  out = {off0, len0, off1, len1, off2, len2}.
 */
int ksa_decode_ranges(const ksa_params *params /*host*/, int64_t pos, int32_t out[6]);

/* Bytes of device workspace ksa_decode_fwd needs for the given number of key splits (0 = library default). */
size_t ksa_decode_workspace_bytes(const ksa_params *params, int32_t n_splits);

/*
 * ksa_decode_fwd: one new text token per sequence.
 *   q [B, Hq, d] device bf16 contiguous; k_cache, v_cache device bf16 with cache_strides = {batch, head, row}
 *   in elements (NULL = contiguous [B, Hkv, cache_rows, d]); pos: device int32 [B], text index of the new
 *   token, whose K/V must already be in the cache; o [B, Hq, d] device bf16; lse device fp32 [B, Hq] or NULL.
 *   workspace: device, at least ksa_decode_workspace_bytes(params, n_splits); n_splits = 0 picks a default.
 * Split-K over the visible rows: each workgroup streams one span of K and V rows once for all Hq/Hkv query
 * heads of a KV head and writes a partial (max, sum, o); a second kernel merges the spans by log-sum-exp.
 * Sequences whose pos is outside [0, n_text) produce NaN rows (device-side positions cannot be validated
 * on the host without a synchronisation).
 */
int ksa_decode_fwd(const ksa_params *params /*host*/, const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *pos, void *o, float *lse, const int64_t cache_strides[3], void *workspace,
                   size_t workspace_bytes, int32_t n_splits, void *stream);

/*
 * ksa_decode_fwd_static: ksa_decode_fwd for callers that cannot allocate device memory or hand over a workspace --
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as ksa_decode_fwd (bit for bit, for the same n_splits), but the partial records of the spans live in a
 * static device array inside the library instead of a caller workspace; the call allocates and frees nothing.
 *   - Limit: ksa_decode_workspace_bytes(params, n_splits) must not exceed KSA_DECODE_STATIC_SCRATCH_BYTES (8 MiB;
 *     the 128K decode workload -- batch 64, 32 query heads, 3 spans -- needs 3.2 MB); otherwise the call returns
 *     KSA_ERR_SCRATCH_LIMIT and enqueues nothing.
 *   - Every GPU holds its own copy of the array for the life of the process; its address is looked up on the
 *     first call on that GPU (one hipGetSymbolAddress, no allocation).
 *   - All calls on one GPU share the array: calls on different streams that overlap in time race on it; calls must
 *     be stream-ordered or otherwise serialised by the caller.  The array keeps the previous call's records; every
 *     record the merge kernel reads is rewritten by the same call's first kernel, so nothing needs clearing.
 */
#define KSA_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
int ksa_decode_fwd_static(const ksa_params *params /*host*/, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *pos, void *o, float *lse, const int64_t cache_strides[3], int32_t n_splits,
                          void *stream);

/* ---- cache lifecycle of the decode loop (section 2.3.1, the step-by-step cache description) ----------- */

/* Kind of a row / of a query in the calls below. */
#define KSA_ROW_TEXT 0     /* a text token; its position argument is a text index i in [0, n_text)            */
#define KSA_ROW_SUMMARY 1  /* a summary token; its position argument is a summary ordinal u = j*m + slot      */

/*
 * ksa_cache_from_prefill: hand-off from a prefilled sequence to the decode loop.  k, v: device bf16
 * [B, L, Hkv, d], the augmented sequence of n_prefill text tokens (at most params->n_text;
 * L = (n_prefill / c)(c + m) + n_prefill mod c), kv_strides = {batch, row, head} in elements (NULL = contiguous).
 * Writes, per (batch, KV head), the summaries of all n_prefill / c whole chunks into the Summary Token Buffer and
 * the text of the window into the text ring of k_cache, v_cache: the incomplete last chunk, if any, and the C whole
 * chunks before it; without an incomplete chunk the last min(n_prefill / c, C + 1) whole chunks (geometry above,
 * cache_strides = {batch, head, row}, NULL = contiguous).  Other cache rows are left as they are.  The next
 * token of every sequence is then text index n_prefill.  params->n_text is the capacity of the cache.
 * n_prefill = 0 is a no-op (k and v may be NULL then).
 * Errors: INVALID_ARG (null or misaligned pointers, negative n_prefill, strides not multiples of 8),
 * OUT_OF_RANGE (n_prefill > n_text), HIP.
 */
int ksa_cache_from_prefill(const ksa_params *params /*host*/, int64_t n_prefill, const void *k, const void *v,
                           const int64_t kv_strides[3], void *k_cache, void *v_cache,
                           const int64_t cache_strides[3], void *stream);

/*
 * ksa_cache_append: one new row per sequence.  k_new, v_new: device bf16 [B, Hkv, d] contiguous.
 * kind = KSA_ROW_TEXT: pos[b] (device int32 [B]) is the text index of the token; its row goes into the slot of the
 * current chunk in the ring, over the row of the chunk that left the window C + 1 chunks ago (the paper's insert
 * and evict steps in one store).  kind = KSA_ROW_SUMMARY: pos[b] is the summary ordinal j*m + slot; the row is
 * committed to the Summary Token Buffer (the paper's commit step).  A sequence whose pos is outside the cache
 * is skipped.  Errors: INVALID_ARG (null or misaligned pointers, unknown kind, kind = SUMMARY with m = 0), HIP.
 */
int ksa_cache_append(const ksa_params *params /*host*/, int32_t kind, const void *k_new, const void *v_new,
                     const int32_t *pos, void *k_cache, void *v_cache, const int64_t cache_strides[3],
                     void *stream);

/*
 * Rows a summary token with ordinal u = j*m + slot reads (Eq. 3, summary rows): the text of its own chunk j
 * (c ring rows) and the summaries of the same chunk up to itself (only itself with params->flags bit 0).
 * out = {off0, len0, off1, len1}: summary buffer range, ring range.
 */
int ksa_decode_summary_ranges(const ksa_params *params /*host*/, int64_t ordinal, int32_t out[4]);

/*
 * ksa_decode_summary_fwd: the summary-token step of the decode loop: one summary query per sequence, run when
 * a chunk has been completed.  Arguments as ksa_decode_fwd, except that ordinal[b] (device int32 [B]) is the
 * summary ordinal j*m + slot of the query; the K/V rows of the chunk's text and of the summary itself must be in
 * the cache (ksa_cache_append).  Same kernels as ksa_decode_fwd over at most c + m rows.
 */
int ksa_decode_summary_fwd(const ksa_params *params /*host*/, const void *q, const void *k_cache,
                           const void *v_cache, const int32_t *ordinal, void *o, float *lse,
                           const int64_t cache_strides[3], void *workspace, size_t workspace_bytes,
                           int32_t n_splits, void *stream);

const char *ksa_status_string(int status);
/* Static description of the build: tile sizes and the gfx target, e.g. for logs. */
const char *ksa_build_info(void);

#ifdef __cplusplus
}
#endif
#endif /* KSA_H_ */
