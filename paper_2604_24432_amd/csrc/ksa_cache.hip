// Cache lifecycle of the decode loop (section 2.3.1): hand-off from a prefilled sequence into the decode cache,
// and the per-step inserts (a new text token into the current chunk; a finished summary into the Summary Token
// Buffer).  Pure data movement, bound by HBM.  The ring layout of the text part makes the paper's eviction step
// disappear: a chunk is written over the chunk that has just left the window.
#include <hip/hip_runtime.h>

#include "ksa_internal.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct FillArgs {
    const __bf16 *k, *v;       // [B, L, Hkv, d] augmented sequence, strides ks
    __bf16 *kc, *vc;           // caches, strides cs
    int64_t ks[3], cs[3];      // {batch, row, head} / {batch, head, row}
    int32_t c, m, C, s_cap;
    int32_t n_chunks;          // J: whole chunks in the prefilled sequence
    int32_t n_sum_rows;        // J * m
    int32_t first_text_chunk;  // first chunk copied into the ring
    int32_t first_text_index;  // = first_text_chunk * c
    int32_t n_rows;            // rows copied per (batch, head): n_sum_rows + text rows
    int32_t chunks16;          // 16-byte pieces per row (d / 8)
};

// One thread moves one 16-byte piece of one row of K and of V.  Row x of the copy list: x < J m is summary ordinal x
// (augmented row (x / m)(c + m) + c + x % m, cache row x); the others are the text of the window in order, up to the
// last prefilled token (text index i: augmented row (i / c)(c + m) + i % c, cache row
// s_cap + ((i / c) mod (C + 1)) c + i % c).
__global__ __launch_bounds__(256) void ksa_cache_fill_kernel(const FillArgs a) {
    const int per_block = 256 / a.chunks16;
    const int x = blockIdx.x * per_block + threadIdx.x / a.chunks16;
    const int piece = threadIdx.x % a.chunks16;
    if (x >= a.n_rows) return;
    const int h = blockIdx.y, b = blockIdx.z;
    int64_t src_row, dst_row;
    if (x < a.n_sum_rows) {
        const int j = x / a.m, u = x - j * a.m;
        src_row = (int64_t)j * (a.c + a.m) + a.c + u;
        dst_row = x;
    } else {
        const int i = a.first_text_index + (x - a.n_sum_rows);
        const int j = i / a.c, r = i - j * a.c;
        src_row = (int64_t)j * (a.c + a.m) + r;
        dst_row = a.s_cap + (j % (a.C + 1)) * a.c + r;
    }
    const int64_t so = b * a.ks[0] + src_row * a.ks[1] + h * a.ks[2] + piece * 8;
    const int64_t dof = b * a.cs[0] + h * a.cs[1] + dst_row * a.cs[2] + piece * 8;
    *reinterpret_cast<u32x4 *>(a.kc + dof) = *reinterpret_cast<const u32x4 *>(a.k + so);
    *reinterpret_cast<u32x4 *>(a.vc + dof) = *reinterpret_cast<const u32x4 *>(a.v + so);
}

struct AppendArgs {
    const __bf16 *k_new, *v_new;   // [B, Hkv, d] contiguous
    const int32_t *pos;            // device [B]
    __bf16 *kc, *vc;
    int64_t cs[3];
    int32_t kind, c, m, C, s_cap, n_text, n_kv_heads, d;
};

// grid (Hkv, B), d / 8 threads: one row of K and V per (batch, KV head).  A position outside the cache is skipped.
__global__ void ksa_cache_append_kernel(const AppendArgs a) {
    const int h = blockIdx.x, b = blockIdx.y, piece = threadIdx.x;
    const int p = a.pos[b];
    int64_t row;
    if (a.kind == KSA_ROW_TEXT) {
        if (p < 0 || p >= a.n_text) return;
        const int j = p / a.c;
        row = a.s_cap + (j % (a.C + 1)) * a.c + (p - j * a.c);
    } else {
        if (p < 0 || p >= a.s_cap) return;
        row = p;
    }
    const int64_t so = ((int64_t)b * a.n_kv_heads + h) * a.d + piece * 8;
    const int64_t dof = b * a.cs[0] + h * a.cs[1] + row * a.cs[2] + piece * 8;
    *reinterpret_cast<u32x4 *>(a.kc + dof) = *reinterpret_cast<const u32x4 *>(a.k_new + so);
    *reinterpret_cast<u32x4 *>(a.vc + dof) = *reinterpret_cast<const u32x4 *>(a.v_new + so);
}

}  // namespace

int ksa_launch_cache_fill(const KsaCacheFillLaunch &L, void *stream) {
    FillArgs a;
    a.k = static_cast<const __bf16 *>(L.k);
    a.v = static_cast<const __bf16 *>(L.v);
    a.kc = static_cast<__bf16 *>(L.k_cache);
    a.vc = static_cast<__bf16 *>(L.v_cache);
    for (int x = 0; x < 3; ++x) a.ks[x] = L.kv_strides[x], a.cs[x] = L.cache_strides[x];
    a.c = L.p.chunk_len, a.m = L.p.n_summary, a.C = L.p.window_chunks, a.s_cap = L.summary_capacity;
    a.n_chunks = (int32_t)(L.n_prefill / L.p.chunk_len);
    a.n_sum_rows = a.n_chunks * a.m;
    // the ring holds C + 1 chunks: an incomplete last chunk takes one slot, so only the C whole chunks before it fit
    const int tail = (int)(L.n_prefill % L.p.chunk_len);
    const int whole_in_ring = tail > 0 ? a.C : a.C + 1;
    a.first_text_chunk = a.n_chunks > whole_in_ring ? a.n_chunks - whole_in_ring : 0;
    a.first_text_index = a.first_text_chunk * a.c;
    a.n_rows = a.n_sum_rows + (int32_t)(L.n_prefill - a.first_text_index);
    a.chunks16 = L.p.head_dim / 8;
    if (a.n_rows == 0) return KSA_OK;
    const int per_block = 256 / a.chunks16;
    const dim3 grid((a.n_rows + per_block - 1) / per_block, L.p.n_kv_heads, L.p.batch);
    hipLaunchKernelGGL(ksa_cache_fill_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}

int ksa_launch_cache_append(const KsaCacheAppendLaunch &L, void *stream) {
    AppendArgs a;
    a.k_new = static_cast<const __bf16 *>(L.k_new);
    a.v_new = static_cast<const __bf16 *>(L.v_new);
    a.pos = L.pos;
    a.kc = static_cast<__bf16 *>(L.k_cache);
    a.vc = static_cast<__bf16 *>(L.v_cache);
    for (int x = 0; x < 3; ++x) a.cs[x] = L.cache_strides[x];
    a.kind = L.kind;
    a.c = L.p.chunk_len, a.m = L.p.n_summary, a.C = L.p.window_chunks, a.s_cap = L.summary_capacity;
    a.n_text = L.p.n_text, a.n_kv_heads = L.p.n_kv_heads, a.d = L.p.head_dim;
    hipLaunchKernelGGL(ksa_cache_append_kernel, dim3(L.p.n_kv_heads, L.p.batch), dim3(L.p.head_dim / 8), 0,
                       static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}
