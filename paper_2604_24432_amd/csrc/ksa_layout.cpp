// Host side of libksa: the integer work of Eq. 1 / Eq. 3 (index maps, per-row visible ranges), the
// block-sparse tile scheduler of section 2.3, and the geometry of the decode cache (section 2.3.1).
// No GPU call in this file.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

#include "ksa_internal.h"

namespace {

inline int32_t pos_part(int64_t x) { return x > 0 ? (int32_t)x : 0; }

// Visible ranges of a text row (chunk j, text index i): summaries of chunks 0..j-C-1 and text of chunks
// max(0,j-C)..j up to i (Eq. 3).
inline void text_row_ranges(const ksa_params &p, int64_t i, int32_t out[4]) {
    const int64_t j = i / p.chunk_len;
    out[0] = 0;
    out[1] = pos_part(j - p.window_chunks) * p.n_summary;
    out[2] = pos_part(j - p.window_chunks) * p.chunk_len;
    out[3] = (int32_t)i + 1;
}

// Visible ranges of a summary row (ordinal u = j*m + slot): its chunk's text, itself, and (unless the
// self-only flag is set) the earlier summaries of its chunk.
inline void summary_row_ranges(const ksa_params &p, int64_t u, int32_t out[4]) {
    const int64_t j = u / p.n_summary;
    out[0] = (p.flags & KSA_FLAG_SUMMARY_SELF_ONLY) ? (int32_t)u : (int32_t)(j * p.n_summary);
    out[1] = (int32_t)u + 1;
    out[2] = (int32_t)(j * p.chunk_len);
    out[3] = (int32_t)((j + 1) * p.chunk_len);
}

inline int32_t tiles_in(const KsaSegment &s) { return (s.end - s.begin + KSA_K_TILE - 1) / KSA_K_TILE; }

// The run starts at the multiple of 16 at or below its first visible key: the kernel's pipelined loop wants that
// alignment (see item_pipelined), and the up to 15 extra keys in front lie outside every row's visible range, so
// the first tile stays live and its mask clips them.
void push_segment(KsaWorkItem &it, int32_t space, int64_t begin, int64_t end, int64_t full_lo, int64_t full_hi) {
    if (end <= begin) return;
    begin -= begin % 16;
    KsaSegment &s = it.seg[it.n_seg++];
    s.space = space;
    s.begin = (int32_t)begin;
    s.end = (int32_t)end;
    s.full_lo = (int32_t)full_lo;
    s.full_hi = (int32_t)full_hi;
    s.pad = 0;
    it.n_tiles += tiles_in(s);
}

// Does tile t of the run need no mask?
inline bool tile_is_full(const KsaSegment &s, int32_t t) {
    const int64_t k0 = (int64_t)s.begin + (int64_t)t * KSA_K_TILE;
    return k0 >= s.full_lo && k0 + KSA_K_TILE <= s.full_hi;
}

// Query tile of text rows [t0, t0+cnt).
KsaWorkItem text_item(const ksa_params &p, int64_t t0, int32_t cnt) {
    KsaWorkItem it;
    std::memset(&it, 0, sizeof(it));
    it.q_space = KSA_SPACE_TEXT;
    it.q_begin = (int32_t)t0;
    it.q_count = cnt;
    const int64_t c = p.chunk_len, m = p.n_summary, C = p.window_chunks;
    const int64_t j0 = t0 / c, j1 = (t0 + cnt - 1) / c;
    // distant summaries: the first row's chunk sees the fewest (those every row sees), the last row's chunk the most
    if (m > 0) push_segment(it, KSA_SPACE_SUMMARY, 0, pos_part(j1 - C) * m, 0, pos_part(j0 - C) * m);
    // sliding-chunk text: [lo_first, ...) is seen by the first row's chunk, [lo_last, t0) by every row
    const int64_t lo_first = pos_part(j0 - C) * c, lo_last = pos_part(j1 - C) * c;
    push_segment(it, KSA_SPACE_TEXT, lo_first, t0 + cnt, lo_last, t0);
    return it;
}

// Query tile of summary rows [u0, u0+cnt): block-diagonal against their chunks' text and summaries.
KsaWorkItem summary_item(const ksa_params &p, int64_t u0, int32_t cnt) {
    KsaWorkItem it;
    std::memset(&it, 0, sizeof(it));
    it.q_space = KSA_SPACE_SUMMARY;
    it.q_begin = (int32_t)u0;
    it.q_count = cnt;
    const int64_t c = p.chunk_len, m = p.n_summary;
    const int64_t j0 = u0 / m, j1 = (u0 + cnt - 1) / m;
    push_segment(it, KSA_SPACE_TEXT, j0 * c, (j1 + 1) * c, 0, 0);
    push_segment(it, KSA_SPACE_SUMMARY, j0 * m, u0 + cnt, 0, 0);
    return it;
}

// Can the kernel walk every key run of the item with its pipelined loop?  That loop computes each lane's row
// offsets once per run and reads V from a key-major copy whose keys are permuted in groups of 16, so it needs
//   - tiles that all start at the same phase of the chunk pattern (64 % period == 0) or never cross a chunk
//     (period % 64 == 0 and an aligned start), period = c for text keys and m for summary keys,
//   - a run that starts at a multiple of 16,
//   - a last tile that ends inside the index space (all 64 rows of every tile exist), and
//   - a chunk length and a summary count that are powers of two.
bool item_pipelined(const ksa_params &p, const KsaWorkItem &it) {
    const int64_t n_sum = (int64_t)(p.n_text / p.chunk_len) * p.n_summary;
    // ... and chunk shapes that are powers of two: that loop maps compact indices to rows with shifts, in scalar code
    // it can afford inside an MFMA slot
    auto pow2 = [](int64_t x) { return x > 0 && (x & (x - 1)) == 0; };
    if (!pow2(p.chunk_len) || (p.n_summary > 0 && !pow2(p.n_summary))) return false;
    for (int s = 0; s < it.n_seg; ++s) {
        const KsaSegment &g = it.seg[s];
        const int64_t period = g.space == KSA_SPACE_TEXT ? p.chunk_len : p.n_summary;
        const int64_t n_space = g.space == KSA_SPACE_TEXT ? p.n_text : n_sum;
        const bool invariant = (KSA_K_TILE % period == 0) || (period % KSA_K_TILE == 0 && g.begin % KSA_K_TILE == 0);
        if (!invariant || g.begin % 16 != 0 || g.begin + (int64_t)tiles_in(g) * KSA_K_TILE > n_space) return false;
    }
    return true;
}

// Launch order.  Workgroups are dealt to the 8 XCDs round-robin by workgroup id, and each XCD has its
// own L2: queue q (workgroup ids congruent to q mod 8) is given whole (batch, KV head) groups so that the
// workgroups running together on one XCD stream the same K/V rows, and items go heaviest first so the
// long tiles start early (longest-processing-time order).  The entries of the items that the forward kernel's
// pipelined instantiation walks come first, those of the other items after them, each part a launch of its own.
// Appends the launch entries of items [item_lo, item_hi) to lay.entries (a whole number of rounds of 8).
void build_entries(ksa_layout &lay, int32_t item_lo, int32_t item_hi) {
    const ksa_params &p = lay.p;
    const int32_t n_groups = p.batch * p.n_kv_heads;
    const int32_t gsz = p.n_q_heads / p.n_kv_heads;
    std::vector<std::vector<KsaWgEntry>> queue(KSA_NUM_XCD);
    auto emit = [&](int q, int32_t item, int32_t grp) {
        for (int32_t x = 0; x < gsz; x += lay.head_stack) {
            KsaWgEntry e;
            e.item = item;
            e.batch = grp / p.n_kv_heads;
            e.q_head = (grp % p.n_kv_heads) * gsz + x;
            e.pad = 0;
            queue[q].push_back(e);
        }
    };
    if (n_groups >= KSA_NUM_XCD) {
        for (int q = 0; q < KSA_NUM_XCD; ++q)
            for (int32_t it = item_lo; it < item_hi; ++it)
                for (int32_t grp = q; grp < n_groups; grp += KSA_NUM_XCD) emit(q, it, grp);
    } else {
        // fewer groups than XCDs: the queues congruent to grp mod n_groups share the items of group grp
        for (int q = 0; q < KSA_NUM_XCD; ++q) {
            const int32_t grp = q % n_groups;
            const int32_t sharers = (KSA_NUM_XCD - grp + n_groups - 1) / n_groups;  // queues serving grp
            const int32_t rank = q / n_groups;
            for (int32_t it = item_lo + rank; it < item_hi; it += sharers) emit(q, it, grp);
        }
    }
    size_t longest = 0;
    for (auto &qv : queue) longest = std::max(longest, qv.size());
    const size_t base = lay.entries.size();
    lay.entries.resize(base + longest * KSA_NUM_XCD, KsaWgEntry{-1, 0, 0, 0});
    for (int q = 0; q < KSA_NUM_XCD; ++q)
        for (size_t x = 0; x < queue[q].size(); ++x) lay.entries[base + x * KSA_NUM_XCD + q] = queue[q][x];
}

}  // namespace

int ksa_validate_params(const ksa_params *p) {
    if (!p) return KSA_ERR_INVALID_ARG;
    if (p->batch <= 0 || p->n_text <= 0 || p->chunk_len <= 0 || p->n_summary < 0 || p->window_chunks < 0)
        return KSA_ERR_INVALID_ARG;
    if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->n_q_heads % p->n_kv_heads != 0) return KSA_ERR_INVALID_ARG;
    if (p->n_summary > 0 && (int64_t)p->compress_ratio * p->n_summary != p->chunk_len) return KSA_ERR_INVALID_ARG;
    if (p->flags & ~KSA_FLAG_SUMMARY_SELF_ONLY) return KSA_ERR_INVALID_ARG;
    if (!(p->softmax_scale == p->softmax_scale)) return KSA_ERR_INVALID_ARG;  // NaN
    // an incomplete last chunk has text positions only (its summaries do not exist yet)
    const int64_t L = (int64_t)(p->n_text / p->chunk_len) * (p->chunk_len + p->n_summary) + p->n_text % p->chunk_len;
    if (L >= (int64_t)1 << 30) return KSA_ERR_UNSUPPORTED;  // row indices are int32 on the device
    if (p->batch > 65535 || p->n_q_heads > 65535) return KSA_ERR_UNSUPPORTED;
    if (p->head_dim != 64 && p->head_dim != 128) return KSA_ERR_UNSUPPORTED;
    return KSA_OK;
}

extern "C" {

int ksa_build_layout(const ksa_params *params, ksa_layout **out) {
    if (!out) return KSA_ERR_INVALID_ARG;
    *out = nullptr;
    const int rc = ksa_validate_params(params);
    if (rc != KSA_OK) return rc;
    ksa_layout *lay = new (std::nothrow) ksa_layout();
    if (!lay) return KSA_ERR_OUT_OF_MEMORY;
    // the schedule grows std::vectors: no exception may leave through the C boundary
    try {
    lay->p = *params;
    if (lay->p.softmax_scale <= 0.f) lay->p.softmax_scale = 1.0f / std::sqrt((float)params->head_dim);
    if (lay->p.n_summary == 0) lay->p.compress_ratio = 0;
    const ksa_params &p = lay->p;
    lay->n_chunks = p.n_text / p.chunk_len;
    lay->aug_len = (int64_t)lay->n_chunks * (p.chunk_len + p.n_summary) + p.n_text % p.chunk_len;

    // query heads per workgroup: as many heads of one KV group as divide it, up to KSA_MAX_HEAD_STACK
    const int32_t gsz = p.n_q_heads / p.n_kv_heads;
    lay->head_stack = gsz % 4 == 0 ? 4 : gsz % 2 == 0 ? 2 : 1;
    static_assert(KSA_MAX_HEAD_STACK == 4, "head stacks are 1, 2 or 4");
    lay->q_tile_rows = KSA_Q_TILE / lay->head_stack;
    const int64_t qt = lay->q_tile_rows;
    for (int64_t t0 = 0; t0 < p.n_text; t0 += qt)
        lay->items.push_back(text_item(p, t0, (int32_t)std::min<int64_t>(qt, p.n_text - t0)));
    const int64_t n_sum = (int64_t)lay->n_chunks * p.n_summary;
    for (int64_t u0 = 0; u0 < n_sum; u0 += qt)
        lay->items.push_back(summary_item(p, u0, (int32_t)std::min<int64_t>(qt, n_sum - u0)));
    for (KsaWorkItem &it : lay->items) {
        it.pipelined = item_pipelined(p, it) ? 1 : 0;
        lay->n_pipelined_items += it.pipelined;
    }
    std::stable_sort(lay->items.begin(), lay->items.end(), [](const KsaWorkItem &a, const KsaWorkItem &b) {
        return a.pipelined != b.pipelined ? a.pipelined > b.pipelined : a.n_tiles > b.n_tiles;
    });
    build_entries(*lay, 0, lay->n_pipelined_items);
    lay->n_pipelined_entries = (int32_t)lay->entries.size();
    build_entries(*lay, lay->n_pipelined_items, (int32_t)lay->items.size());
    } catch (...) {
        delete lay;
        return KSA_ERR_OUT_OF_MEMORY;
    }
    *out = lay;
    return KSA_OK;
}

int ksa_augmented_rows(const ksa_params *p, int64_t n_text, int64_t *rows) {
    if (!p || !rows || n_text < 0 || p->chunk_len <= 0 || p->n_summary < 0) return KSA_ERR_INVALID_ARG;
    *rows = n_text / p->chunk_len * (int64_t)(p->chunk_len + p->n_summary) + n_text % p->chunk_len;
    return KSA_OK;
}

int ksa_layout_dims(const ksa_layout *lay, int64_t *aug_len, int32_t *n_chunks, int32_t *q_tile_rows,
                    int32_t *k_tile_rows, int32_t *heads_per_workgroup) {
    if (!lay) return KSA_ERR_INVALID_ARG;
    if (aug_len) *aug_len = lay->aug_len;
    if (n_chunks) *n_chunks = lay->n_chunks;
    if (q_tile_rows) *q_tile_rows = lay->q_tile_rows;
    if (k_tile_rows) *k_tile_rows = KSA_K_TILE;
    if (heads_per_workgroup) *heads_per_workgroup = lay->head_stack;
    return KSA_OK;
}

int ksa_layout_index_maps(const ksa_layout *lay, int32_t *aug_chunk, uint8_t *aug_is_summary,
                          int32_t *position_ids, int32_t *text_to_aug, int32_t *summary_to_aug) {
    if (!lay) return KSA_ERR_INVALID_ARG;
    const int64_t c = lay->p.chunk_len, m = lay->p.n_summary, w = c + m;
    for (int64_t a = 0; a < lay->aug_len; ++a) {
        const int64_t j = a / w, r = a % w;
        if (aug_chunk) aug_chunk[a] = (int32_t)j;
        if (aug_is_summary) aug_is_summary[a] = r >= c;
        // a summary token shares the position of its chunk's last text token (section 2.2.1)
        if (position_ids) position_ids[a] = (int32_t)(j * c + std::min<int64_t>(r, c - 1));
    }
    if (text_to_aug)
        for (int64_t i = 0; i < lay->p.n_text; ++i) text_to_aug[i] = (int32_t)(i / c * w + i % c);
    if (summary_to_aug)
        for (int64_t u = 0; u < (int64_t)lay->n_chunks * m; ++u) summary_to_aug[u] = (int32_t)(u / m * w + c + u % m);
    return KSA_OK;
}

int ksa_layout_row_ranges(const ksa_layout *lay, int64_t aq, int32_t out[4]) {
    if (!lay || !out) return KSA_ERR_INVALID_ARG;
    if (aq < 0 || aq >= lay->aug_len) return KSA_ERR_OUT_OF_RANGE;
    const int64_t c = lay->p.chunk_len, w = c + lay->p.n_summary;
    const int64_t j = aq / w, r = aq % w;
    if (r < c)
        text_row_ranges(lay->p, j * c + r, out);
    else
        summary_row_ranges(lay->p, j * lay->p.n_summary + (r - c), out);
    return KSA_OK;
}

int ksa_layout_mask_row(const ksa_layout *lay, int64_t aq, uint8_t *row_out) {
    if (!lay || !row_out) return KSA_ERR_INVALID_ARG;
    int32_t rg[4];
    const int rc = ksa_layout_row_ranges(lay, aq, rg);
    if (rc != KSA_OK) return rc;
    const int64_t c = lay->p.chunk_len, m = lay->p.n_summary, w = c + m;
    std::memset(row_out, 0, (size_t)lay->aug_len);
    for (int64_t u = rg[0]; u < rg[1]; ++u) row_out[u / m * w + c + u % m] = 1;
    for (int64_t i = rg[2]; i < rg[3]; ++i) row_out[i / c * w + i % c] = 1;
    return KSA_OK;
}

int ksa_layout_tile_pairs(const ksa_layout *lay, int64_t *n_pairs, uint8_t *q_space, int32_t *q_begin,
                          int32_t *q_count, uint8_t *k_space, int32_t *k_begin, int32_t *k_count, uint8_t *kind) {
    if (!lay || !n_pairs) return KSA_ERR_INVALID_ARG;
    int64_t x = 0;
    for (const KsaWorkItem &it : lay->items)
        for (int32_t s = 0; s < it.n_seg; ++s)
            for (int32_t kb = it.seg[s].begin; kb < it.seg[s].end; kb += KSA_K_TILE, ++x) {
                if (q_space) q_space[x] = (uint8_t)it.q_space;
                if (q_begin) q_begin[x] = it.q_begin;
                if (q_count) q_count[x] = it.q_count;
                if (k_space) k_space[x] = (uint8_t)it.seg[s].space;
                if (k_begin) k_begin[x] = kb;
                if (k_count) k_count[x] = std::min(KSA_K_TILE, it.seg[s].end - kb);
                if (kind) kind[x] = tile_is_full(it.seg[s], (kb - it.seg[s].begin) / KSA_K_TILE) ? KSA_TILE_FULL : KSA_TILE_MASKED;
            }
    *n_pairs = x;
    return KSA_OK;
}

int ksa_layout_launch_order(const ksa_layout *lay, int64_t *n_entries, uint8_t *q_space, int32_t *q_begin,
                            int32_t *batch, int32_t *q_head) {
    if (!lay || !n_entries) return KSA_ERR_INVALID_ARG;
    *n_entries = (int64_t)lay->entries.size();
    for (size_t x = 0; x < lay->entries.size(); ++x) {
        const KsaWgEntry &e = lay->entries[x];
        if (q_space) q_space[x] = e.item >= 0 ? (uint8_t)lay->items[e.item].q_space : 0;
        if (q_begin) q_begin[x] = e.item >= 0 ? lay->items[e.item].q_begin : -1;
        if (batch) batch[x] = e.batch;
        if (q_head) q_head[x] = e.q_head;
    }
    return KSA_OK;
}

// ---- decode cache geometry ---------------------------------------------------------------------

int ksa_cache_geometry(const ksa_params *p, int32_t *summary_capacity, int32_t *cache_rows) {
    const int rc = ksa_validate_params(p);
    if (rc != KSA_OK) return rc;
    const int64_t s_cap = (int64_t)(p->n_text / p->chunk_len) * p->n_summary;
    const int64_t rows = s_cap + (int64_t)(p->window_chunks + 1) * p->chunk_len;
    if (rows >= (int64_t)1 << 30) return KSA_ERR_UNSUPPORTED;
    if (summary_capacity) *summary_capacity = (int32_t)s_cap;
    if (cache_rows) *cache_rows = (int32_t)rows;
    return KSA_OK;
}

int ksa_cache_text_row(const ksa_params *p, int64_t i, int32_t *row) {
    int32_t s_cap;
    const int rc = ksa_cache_geometry(p, &s_cap, nullptr);
    if (rc != KSA_OK) return rc;
    if (!row) return KSA_ERR_INVALID_ARG;
    if (i < 0 || i >= p->n_text) return KSA_ERR_OUT_OF_RANGE;
    const int64_t j = i / p->chunk_len;
    *row = (int32_t)(s_cap + (j % (p->window_chunks + 1)) * p->chunk_len + i % p->chunk_len);
    return KSA_OK;
}

int ksa_cache_summary_row(const ksa_params *p, int64_t u, int32_t *row) {
    int32_t s_cap;
    const int rc = ksa_cache_geometry(p, &s_cap, nullptr);
    if (rc != KSA_OK) return rc;
    if (!row) return KSA_ERR_INVALID_ARG;
    if (u < 0 || u >= s_cap) return KSA_ERR_OUT_OF_RANGE;
    *row = (int32_t)u;
    return KSA_OK;
}

int ksa_decode_summary_ranges(const ksa_params *p, int64_t u, int32_t out[4]) {
    int32_t s_cap;
    const int rc = ksa_cache_geometry(p, &s_cap, nullptr);
    if (rc != KSA_OK) return rc;
    if (!out) return KSA_ERR_INVALID_ARG;
    if (p->n_summary == 0) return KSA_ERR_INVALID_ARG;
    if (u < 0 || u >= s_cap) return KSA_ERR_OUT_OF_RANGE;
    const int64_t c = p->chunk_len, C = p->window_chunks, m = p->n_summary;
    const int64_t j = u / m, slot = u % m;
    // summaries of the same chunk up to and including itself (Eq. 3, summary rows); only itself with flag bit 0
    const bool self_only = (p->flags & 1u) != 0;
    out[0] = (int32_t)(self_only ? u : j * m);
    out[1] = (int32_t)(self_only ? 1 : slot + 1);
    // the text of its own chunk: one whole ring slot
    out[2] = (int32_t)(s_cap + (j % (C + 1)) * c);
    out[3] = (int32_t)c;
    return KSA_OK;
}

int ksa_decode_ranges(const ksa_params *p, int64_t pos, int32_t out[6]) {
    int32_t s_cap;
    const int rc = ksa_cache_geometry(p, &s_cap, nullptr);
    if (rc != KSA_OK) return rc;
    if (!out) return KSA_ERR_INVALID_ARG;
    if (pos < 0 || pos >= p->n_text) return KSA_ERR_OUT_OF_RANGE;
    const int64_t c = p->chunk_len, C = p->window_chunks;
    const int64_t j = pos / c, r = pos % c;
    const int64_t slot = j % (C + 1);
    // summaries of chunks 0 .. j-C-1 (Eq. 3 left term): a prefix of the summary buffer
    out[0] = 0;
    out[1] = pos_part(j - C) * p->n_summary;
    // ring slots below the current chunk's slot are complete chunks; the current slot is filled up to r
    out[2] = s_cap;
    out[3] = (int32_t)(slot * c + r + 1);
    // slots above the current one hold older in-window chunks once the ring has wrapped (j >= C)
    out[4] = (int32_t)(s_cap + (slot + 1) * c);
    out[5] = j >= C ? (int32_t)((C - slot) * c) : 0;
    return KSA_OK;
}

const char *ksa_status_string(int status) {
    switch (status) {
        case KSA_OK: return "ok";
        case KSA_ERR_INVALID_ARG: return "invalid argument";
        case KSA_ERR_UNSUPPORTED: return "unsupported configuration";
        case KSA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case KSA_ERR_HIP: return "HIP runtime error";
        case KSA_ERR_OUT_OF_RANGE: return "index out of range";
        case KSA_ERR_SCRATCH_LIMIT: return "problem exceeds the static scratch buffer";
        case KSA_ERR_OUT_OF_MEMORY: return "out of host memory";
        default: return "unknown status";
    }
}

}  // extern "C"
