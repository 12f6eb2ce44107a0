// C-ABI entry points that touch the GPU: schedule upload, prefill and decode launches.
// Every argument check happens before the first HIP call.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstring>

#include "ksa_internal.h"

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void default_strides(int64_t out[3], const int64_t *given, int64_t d0, int64_t d1, int64_t d2) {
    // contiguous [x, d0-dim, d1-dim, d2] -> strides of the three leading dims
    if (given) {
        out[0] = given[0], out[1] = given[1], out[2] = given[2];
    } else {
        out[2] = d2;
        out[1] = d1 * d2;
        out[0] = d0 * d1 * d2;
    }
}

bool strides_ok(const int64_t s[3]) {
    // rows must keep 16-byte alignment of the head vectors (bf16: multiples of 8 elements)
    return s[0] >= 0 && s[1] > 0 && s[2] > 0 && s[0] % 8 == 0 && s[1] % 8 == 0 && s[2] % 8 == 0;
}

}  // namespace

extern "C" {

void ksa_layout_destroy(ksa_layout *lay) {
    if (!lay) return;
    if (lay->d_items) (void)hipFree(lay->d_items);
    if (lay->d_entries) (void)hipFree(lay->d_entries);
    delete lay;
}

int ksa_layout_upload(ksa_layout *lay) {
    if (!lay) return KSA_ERR_INVALID_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return KSA_ERR_HIP;
    if (lay->d_items && lay->device == dev) return KSA_OK;
    if (lay->d_items) {
        (void)hipFree(lay->d_items);
        (void)hipFree(lay->d_entries);
        lay->d_items = lay->d_entries = nullptr;
    }
    const size_t ib = lay->items.size() * sizeof(KsaWorkItem), eb = lay->entries.size() * sizeof(KsaWgEntry);
    if (hipMalloc(&lay->d_items, ib) != hipSuccess) return KSA_ERR_HIP;
    if (hipMalloc(&lay->d_entries, eb) != hipSuccess) {
        (void)hipFree(lay->d_items);
        lay->d_items = nullptr;
        return KSA_ERR_HIP;
    }
    if (hipMemcpy(lay->d_items, lay->items.data(), ib, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(lay->d_entries, lay->entries.data(), eb, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(lay->d_items);
        (void)hipFree(lay->d_entries);
        lay->d_items = lay->d_entries = nullptr;
        return KSA_ERR_HIP;
    }
    lay->device = dev;
    return KSA_OK;
}

size_t ksa_prefill_workspace_bytes(const ksa_layout *lay) { return lay ? ksa_prefill_workspace_size(lay->p) : 0; }

namespace {

int prefill_call(ksa_layout *lay, const void *q, const void *k, const void *v, void *o, float *lse,
                 const int64_t q_strides[3], const int64_t kv_strides[3], const int64_t o_strides[3], void *workspace,
                 size_t workspace_bytes, void *stream, int32_t phases) {
    if (!lay || !q || !k || !v || !o || !workspace) return KSA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return KSA_ERR_INVALID_ARG;
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return KSA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return KSA_ERR_INVALID_ARG;
    if (workspace_bytes < ksa_prefill_workspace_size(lay->p)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    const ksa_params &p = lay->p;
    KsaPrefillLaunch a;
    default_strides(a.q_strides, q_strides, lay->aug_len, p.n_q_heads, p.head_dim);
    default_strides(a.kv_strides, kv_strides, lay->aug_len, p.n_kv_heads, p.head_dim);
    default_strides(a.o_strides, o_strides, lay->aug_len, p.n_q_heads, p.head_dim);
    if (!strides_ok(a.q_strides) || !strides_ok(a.kv_strides) || !strides_ok(a.o_strides)) return KSA_ERR_INVALID_ARG;
    const int rc = ksa_layout_upload(lay);
    if (rc != KSA_OK) return rc;
    a.q = q, a.k = k, a.v = v, a.o = o, a.lse = lse;
    a.items = static_cast<const KsaWorkItem *>(lay->d_items);
    a.entries = static_cast<const KsaWgEntry *>(lay->d_entries);
    a.n_entries = (int32_t)lay->entries.size();
    a.n_pipelined_entries = lay->n_pipelined_entries;
    a.n_pipelined_items = lay->n_pipelined_items;
    a.n_generic_items = (int32_t)lay->items.size() - lay->n_pipelined_items;
    a.head_stack = lay->head_stack;
    a.p = p;
    a.aug_len = lay->aug_len;
    a.workspace = workspace;
    a.workspace_bytes = workspace_bytes;
    a.phases = phases;
    return ksa_launch_prefill(a, stream);
}

}  // namespace

int ksa_prefill_fwd(ksa_layout *lay, const void *q, const void *k, const void *v, void *o, float *lse,
                    const int64_t q_strides[3], const int64_t kv_strides[3], const int64_t o_strides[3],
                    void *workspace, size_t workspace_bytes, void *stream) {
    return prefill_call(lay, q, k, v, o, lse, q_strides, kv_strides, o_strides, workspace, workspace_bytes, stream, 3);
}

int ksa_prefill_relayout_v(ksa_layout *lay, const void *v, const int64_t kv_strides[3], void *workspace,
                           size_t workspace_bytes, void *stream) {
    // the attention tensors are not touched in this phase; v stands in for them in the shared argument checks
    return prefill_call(lay, v, v, v, workspace, nullptr, nullptr, kv_strides, nullptr, workspace, workspace_bytes, stream, 1);
}

size_t ksa_prefill_bwd_workspace_bytes(const ksa_layout *lay) {
    return lay ? ksa_prefill_bwd_workspace_size(lay->p, lay->aug_len) : 0;
}

int ksa_prefill_bwd(ksa_layout *lay, const void *q, const void *k, const void *v, const void *o, const float *lse,
                    const void *d_o, void *dq, void *dk, void *dv, const int64_t q_strides[3],
                    const int64_t kv_strides[3], const int64_t o_strides[3], const int64_t dq_strides[3],
                    const int64_t dkv_strides[3], void *workspace, size_t workspace_bytes, void *stream) {
    if (!lay || !q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace) return KSA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
        return KSA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(lse) & 3u) return KSA_ERR_INVALID_ARG;
    if (workspace_bytes < ksa_prefill_bwd_workspace_size(lay->p, lay->aug_len)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    const ksa_params &p = lay->p;
    KsaPrefillBwdLaunch a;
    default_strides(a.q_strides, q_strides, lay->aug_len, p.n_q_heads, p.head_dim);
    default_strides(a.kv_strides, kv_strides, lay->aug_len, p.n_kv_heads, p.head_dim);
    default_strides(a.o_strides, o_strides, lay->aug_len, p.n_q_heads, p.head_dim);
    default_strides(a.dq_strides, dq_strides, lay->aug_len, p.n_q_heads, p.head_dim);
    default_strides(a.dkv_strides, dkv_strides, lay->aug_len, p.n_kv_heads, p.head_dim);
    if (!strides_ok(a.q_strides) || !strides_ok(a.kv_strides) || !strides_ok(a.o_strides) ||
        !strides_ok(a.dq_strides) || !strides_ok(a.dkv_strides))
        return KSA_ERR_INVALID_ARG;
    const int rc = ksa_layout_upload(lay);
    if (rc != KSA_OK) return rc;
    a.q = q, a.k = k, a.v = v, a.o = o, a.d_o = d_o, a.lse = lse;
    a.dq = dq, a.dk = dk, a.dv = dv;
    a.items = static_cast<const KsaWorkItem *>(lay->d_items);
    a.entries = static_cast<const KsaWgEntry *>(lay->d_entries);
    a.n_entries = (int32_t)lay->entries.size();
    a.head_stack = lay->head_stack;
    a.p = p;
    a.aug_len = lay->aug_len;
    a.workspace = workspace;
    a.workspace_bytes = workspace_bytes;
    return ksa_launch_prefill_bwd(a, stream);
}

size_t ksa_decode_workspace_bytes(const ksa_params *p, int32_t n_splits) {
    if (ksa_validate_params(p) != KSA_OK || n_splits < 0) return 0;
    if (n_splits == 0) n_splits = ksa_decode_default_splits(p);
    // per (batch, query head, split): head_dim partial outputs + running max + running sum, fp32
    return (size_t)p->batch * p->n_q_heads * n_splits * (p->head_dim + 2) * sizeof(float);
}

namespace {

int decode_call(const ksa_params *p, int32_t kind, const void *q, const void *k_cache, const void *v_cache,
                const int32_t *pos, void *o, float *lse, const int64_t cache_strides[3], void *workspace,
                size_t workspace_bytes, int32_t n_splits, void *stream) {
    int32_t s_cap = 0, rows = 0;
    const int rc = ksa_cache_geometry(p, &s_cap, &rows);
    if (rc != KSA_OK) return rc;
    if (!q || !k_cache || !v_cache || !pos || !o || !workspace) return KSA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o) || !aligned16(workspace))
        return KSA_ERR_INVALID_ARG;
    if (n_splits < 0 || n_splits > 1024) return KSA_ERR_INVALID_ARG;
    if (kind == KSA_ROW_SUMMARY && p->n_summary == 0) return KSA_ERR_INVALID_ARG;
    if (p->n_q_heads / p->n_kv_heads > 8) return KSA_ERR_UNSUPPORTED;
    if (n_splits == 0) n_splits = ksa_decode_default_splits(p);
    if (workspace_bytes < ksa_decode_workspace_bytes(p, n_splits)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    KsaDecodeLaunch a;
    default_strides(a.cache_strides, cache_strides, p->n_kv_heads, rows, p->head_dim);
    if (!strides_ok(a.cache_strides)) return KSA_ERR_INVALID_ARG;
    a.q = q, a.k_cache = k_cache, a.v_cache = v_cache, a.pos = pos, a.o = o, a.lse = lse;
    a.workspace = static_cast<float *>(workspace);
    a.n_splits = n_splits;
    a.summary_capacity = s_cap;
    a.kind = kind;
    a.p = *p;
    if (a.p.softmax_scale <= 0.f) a.p.softmax_scale = 1.0f / __builtin_sqrtf((float)p->head_dim);
    return ksa_launch_decode(a, stream);
}

}  // namespace

int ksa_decode_fwd(const ksa_params *p, const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *pos, void *o, float *lse, const int64_t cache_strides[3], void *workspace,
                   size_t workspace_bytes, int32_t n_splits, void *stream) {
    return decode_call(p, KSA_ROW_TEXT, q, k_cache, v_cache, pos, o, lse, cache_strides, workspace, workspace_bytes,
                       n_splits, stream);
}

int ksa_decode_fwd_static(const ksa_params *p, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *pos, void *o, float *lse, const int64_t cache_strides[3], int32_t n_splits,
                          void *stream) {
    // size check first (host arithmetic only), so that an oversized problem is refused even without a GPU
    const int rc = ksa_validate_params(p);
    if (rc != KSA_OK) return rc;
    if (n_splits < 0 || n_splits > 1024) return KSA_ERR_INVALID_ARG;
    const int32_t splits = n_splits == 0 ? ksa_decode_default_splits(p) : n_splits;
    const size_t need = ksa_decode_workspace_bytes(p, splits);
    if (need > KSA_DECODE_STATIC_SCRATCH_BYTES) return KSA_ERR_SCRATCH_LIMIT;
    if (!q || !k_cache || !v_cache || !pos || !o) return KSA_ERR_INVALID_ARG;
    float *buf = nullptr;
    const int rs = ksa_decode_static_scratch(&buf);
    if (rs != KSA_OK) return rs;
    return decode_call(p, KSA_ROW_TEXT, q, k_cache, v_cache, pos, o, lse, cache_strides, buf, need, splits, stream);
}

int ksa_decode_summary_fwd(const ksa_params *p, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *ordinal, void *o, float *lse, const int64_t cache_strides[3],
                           void *workspace, size_t workspace_bytes, int32_t n_splits, void *stream) {
    return decode_call(p, KSA_ROW_SUMMARY, q, k_cache, v_cache, ordinal, o, lse, cache_strides, workspace,
                       workspace_bytes, n_splits, stream);
}

int ksa_cache_from_prefill(const ksa_params *p, int64_t n_prefill, const void *k, const void *v,
                           const int64_t kv_strides[3], void *k_cache, void *v_cache,
                           const int64_t cache_strides[3], void *stream) {
    int32_t s_cap = 0, rows = 0;
    const int rc = ksa_cache_geometry(p, &s_cap, &rows);
    if (rc != KSA_OK) return rc;
    if (n_prefill < 0) return KSA_ERR_INVALID_ARG;
    if (n_prefill > p->n_text) return KSA_ERR_OUT_OF_RANGE;
    if (!k_cache || !v_cache || !aligned16(k_cache) || !aligned16(v_cache)) return KSA_ERR_INVALID_ARG;
    if (n_prefill == 0) return KSA_OK;   // nothing to hand over (k and v may be NULL then)
    if (!k || !v || !aligned16(k) || !aligned16(v)) return KSA_ERR_INVALID_ARG;
    KsaCacheFillLaunch a;
    const int64_t L = n_prefill / p->chunk_len * (int64_t)(p->chunk_len + p->n_summary) + n_prefill % p->chunk_len;
    if (kv_strides) {
        for (int x = 0; x < 3; ++x) a.kv_strides[x] = kv_strides[x];
    } else {   // contiguous [B, L, Hkv, d]: {batch, row, head}
        a.kv_strides[2] = p->head_dim;
        a.kv_strides[1] = (int64_t)p->n_kv_heads * p->head_dim;
        a.kv_strides[0] = L * a.kv_strides[1];
    }
    default_strides(a.cache_strides, cache_strides, p->n_kv_heads, rows, p->head_dim);
    if (!strides_ok(a.kv_strides) || !strides_ok(a.cache_strides)) return KSA_ERR_INVALID_ARG;
    a.k = k, a.v = v, a.k_cache = k_cache, a.v_cache = v_cache;
    a.n_prefill = n_prefill;
    a.summary_capacity = s_cap;
    a.p = *p;
    return ksa_launch_cache_fill(a, stream);
}

int ksa_cache_append(const ksa_params *p, int32_t kind, const void *k_new, const void *v_new, const int32_t *pos,
                     void *k_cache, void *v_cache, const int64_t cache_strides[3], void *stream) {
    int32_t s_cap = 0, rows = 0;
    const int rc = ksa_cache_geometry(p, &s_cap, &rows);
    if (rc != KSA_OK) return rc;
    if (kind != KSA_ROW_TEXT && kind != KSA_ROW_SUMMARY) return KSA_ERR_INVALID_ARG;
    if (kind == KSA_ROW_SUMMARY && p->n_summary == 0) return KSA_ERR_INVALID_ARG;
    if (!k_new || !v_new || !pos || !k_cache || !v_cache) return KSA_ERR_INVALID_ARG;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return KSA_ERR_INVALID_ARG;
    KsaCacheAppendLaunch a;
    default_strides(a.cache_strides, cache_strides, p->n_kv_heads, rows, p->head_dim);
    if (!strides_ok(a.cache_strides)) return KSA_ERR_INVALID_ARG;
    a.k_new = k_new, a.v_new = v_new, a.pos = pos, a.k_cache = k_cache, a.v_cache = v_cache;
    a.kind = kind;
    a.summary_capacity = s_cap;
    a.p = *p;
    return ksa_launch_cache_append(a, stream);
}

const char *ksa_build_info(void) {
    static char info[320];
    // the compiler is part of the description: the kernels place MFMA wait states by hand in inline assembly, and
    // those were validated with this one
#ifdef __clang_version__
    const char *compiler = "clang " __clang_version__;
#else
    const char *compiler = "not hipcc (host-only test build)";
#endif
    std::snprintf(info, sizeof(info), "libksa gfx950 q_tile=%d k_tile=%d max_segments=%d compiler=%s", KSA_Q_TILE,
                  KSA_K_TILE, KSA_MAX_SEGMENTS, compiler);
    return info;
}

}  // extern "C"
