// KSA decode for gfx950: one new text token per sequence attends over the summary KV cache
// (section 2.3.1).  The work is bandwidth bound: every visible K and V row is read from HBM exactly once
// per KV head and serves all Hq/Hkv query heads of that head.
//
// Split-K: workgroup (split, kv head, batch) streams one span of the visible rows.  A cache row of
// head_dim bf16 is read by head_dim/8 adjacent lanes with one 16-byte load each, so a wavefront load covers
// 1 KiB of consecutive memory; U such loads of K and of V are in flight per lane.  Each lane keeps the
// partial dot products of its 8 columns for all query heads of the group, a 4-step DPP all-reduce over the
// row's lanes finishes the scores, and every lane group runs its own online softmax on the rows it saw.
// The lane groups of a workgroup are merged through LDS into one partial (max, sum, o) per query head;
// a second kernel merges the spans of a sequence by log-sum-exp.
#include <hip/hip_runtime.h>

#include <mutex>

#include "ksa_internal.h"

// Scratch memory of ksa_decode_fwd_static: the partial (o, max, sum) records of the spans, which ksa_decode_fwd
// keeps in the caller's workspace.  Every GPU the library runs on holds its own copy of the array, at its own
// address, until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address it returns (ksa_decode_static_scratch below) is what kernels and HIP calls are given.
static __device__ __align__(256) unsigned char scratch[KSA_DECODE_STATIC_SCRATCH_BYTES];

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;      // threads per workgroup
constexpr int U = 4;         // row loads in flight per lane, K and V each

struct DecodeArgs {
    const __bf16 *q, *k, *v;
    const int32_t *pos;
    __bf16 *o;
    float *lse;
    float *ws;
    int64_t cs[3];   // {batch, head, row} strides of the caches in elements
    int32_t n_splits, s_cap;
    int32_t kind, self_only;   // KSA_ROW_TEXT / KSA_ROW_SUMMARY query; flag bit 0 of the parameters
    int32_t c, m, C, n_text;
    int32_t n_q_heads, n_kv_heads;
    float scale_log2e;
};

struct Ranges {
    int off0, n0, off1, n1, off2, n2;   // summaries [off0, off0+n0), ring [off1, off1+n1), ring [off2, off2+n2)
};

// Is p a position the query kind can have?  (text index / summary ordinal)
__device__ __forceinline__ bool valid_pos(const DecodeArgs &a, int p) {
    return p >= 0 && p < (a.kind == KSA_ROW_TEXT ? a.n_text : a.s_cap);
}

// Rows the query reads (Eq. 3 mapped onto the cache geometry); all zero if p is invalid.
// Text token at text index p: the summaries of the chunks that have left the window and the text of the window up to
// itself.  Summary token with ordinal p = j m + slot: the summaries of its chunk up to itself (only itself with
// self_only) and the text of its chunk, one whole ring slot.
__device__ __forceinline__ Ranges visible_rows(const DecodeArgs &a, int p) {
    Ranges R = {0, 0, 0, 0, 0, 0};
    if (!valid_pos(a, p)) return R;
    if (a.kind == KSA_ROW_SUMMARY) {
        const int j = p / a.m, slot = p - j * a.m;
        R.off0 = a.self_only ? p : j * a.m;
        R.n0 = a.self_only ? 1 : slot + 1;
        R.off1 = a.s_cap + (j % (a.C + 1)) * a.c;
        R.n1 = a.c;
        return R;
    }
    const int j = p / a.c, r = p - j * a.c;
    const int slot = j % (a.C + 1);
    R.n0 = (j - a.C > 0 ? j - a.C : 0) * a.m;
    R.off1 = a.s_cap;
    R.n1 = slot * a.c + r + 1;
    R.off2 = a.s_cap + (slot + 1) * a.c;
    R.n2 = j >= a.C ? (a.C - slot) * a.c : 0;
    return R;
}

__device__ __forceinline__ int phys_row(const Ranges &R, int v) {
    if (v < R.n0) return R.off0 + v;
    v -= R.n0;
    if (v < R.n1) return R.off1 + v;
    return R.off2 + (v - R.n1);
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false);
    return x + __builtin_bit_cast(float, y);
}
// sum over the LPR adjacent lanes that share a row; every one of them ends with the total
template <int LPR>
__device__ __forceinline__ float row_allreduce(float x) {
    x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);   // row_half_mirror: the other quad of the 8
    if (LPR == 16) x = dpp_add<0x140>(x);   // row_mirror: the other 8 of the 16
    return x;
}

// eight bf16 -> eight fp32 (a bf16 is the high half of an fp32)
__device__ __forceinline__ void unpack8(const u32x4 &x, float f[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __builtin_bit_cast(float, x[e] << 16);
        f[2 * e + 1] = __builtin_bit_cast(float, x[e] & 0xffff0000u);
    }
}

// partial record in the workspace: [D] unnormalised o, then running max (log2 domain), then running sum
template <int D, int G>
__global__ __launch_bounds__(NT) void ksa_decode_split_kernel(const DecodeArgs a) {
    constexpr int LPR = D / 8;          // lanes per cache row
    constexpr int RPW = 64 / LPR;       // rows per wavefront load
    constexpr int NG = NT / LPR;        // lane groups per workgroup
    constexpr int R_IT = (NT / 64) * RPW * U;   // rows per workgroup iteration

    const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int chunk = lane % LPR, gi = lane / LPR;

    const Ranges R = visible_rows(a, a.pos[b]);
    const int N = R.n0 + R.n1 + R.n2;
    const int per = (N + a.n_splits - 1) / a.n_splits;
    const int v0 = split * per, v1 = min(N, v0 + per);

    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const u32x4 raw = *reinterpret_cast<const u32x4 *>(a.q + ((int64_t)b * a.n_q_heads + hkv * G + g) * D + chunk * 8);
        unpack8(raw, qf[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[g][e] *= a.scale_log2e;
    }
    float m_run[G], l_run[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m_run[g] = -1e30f;
        l_run[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
    }

    const __bf16 *kb = a.k + b * a.cs[0] + hkv * a.cs[1] + chunk * 8;
    const __bf16 *vb = a.v + b * a.cs[0] + hkv * a.cs[1] + chunk * 8;

    for (int base = v0 + wave * (RPW * U); base < v1; base += R_IT) {
        u32x4 kk[U], vv[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int vr = base + u * RPW + gi;
            ok[u] = vr < v1;
            const int64_t off = (int64_t)phys_row(R, ok[u] ? vr : v1 - 1) * a.cs[2];
            kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kb + off));
            vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vb + off));
        }
        float s[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[8];
            unpack8(kk[u], kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = fmaf(qf[g][e], kf[e], acc);
                acc = row_allreduce<LPR>(acc);
                s[u][g] = ok[u] ? acc : -INFINITY;
            }
        }
        float p[U][G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mx = s[0][g];
#pragma unroll
            for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][g]);
            const float m_new = fmaxf(m_run[g], mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run[g] - m_new);
            m_run[g] = m_new;
            float sum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[u][g] = __builtin_amdgcn_exp2f(s[u][g] - m_new);
                sum += p[u][g];
            }
            l_run[g] = l_run[g] * alpha + sum;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[g][e] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[8];
            unpack8(vv[u], vf);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[g][e] = fmaf(p[u][g], vf[e], o[g][e]);
        }
    }

    // ---- merge the NG lane groups of the workgroup ------------------------------------------------
    __shared__ float sh_o[NG][G][D];
    __shared__ float sh_m[NG][G], sh_l[NG][G];
    const int grp = tid / LPR;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sh_o[grp][g][chunk * 8 + e] = o[g][e];
        if (chunk == 0) {
            sh_m[grp][g] = m_run[g];
            sh_l[grp][g] = l_run[g];
        }
    }
    __syncthreads();
    for (int x = tid; x < G * (D + 2); x += NT) {
        const int g = x / (D + 2), col = x % (D + 2);
        float M = sh_m[0][g];
        for (int y = 1; y < NG; ++y) M = fmaxf(M, sh_m[y][g]);
        float acc = 0.f;
        if (col < D) {
            for (int y = 0; y < NG; ++y) acc += sh_o[y][g][col] * __builtin_amdgcn_exp2f(sh_m[y][g] - M);
        } else if (col == D) {
            acc = M;
        } else {
            for (int y = 0; y < NG; ++y) acc += sh_l[y][g] * __builtin_amdgcn_exp2f(sh_m[y][g] - M);
        }
        a.ws[(((int64_t)b * a.n_q_heads + hkv * G + g) * a.n_splits + split) * (D + 2) + col] = acc;
    }
}

// one workgroup of D threads per (batch, query head): log-sum-exp merge of the spans
template <int D>
__global__ __launch_bounds__(D) void ksa_decode_merge_kernel(const DecodeArgs a) {
    const int hq = blockIdx.x, b = blockIdx.y, col = threadIdx.x;
    const float *rec = a.ws + ((int64_t)b * a.n_q_heads + hq) * a.n_splits * (D + 2);
    const bool valid = valid_pos(a, a.pos[b]);
    float M = -1e30f;
    for (int s = 0; s < a.n_splits; ++s) M = fmaxf(M, rec[s * (D + 2) + D]);
    float acc = 0.f, den = 0.f;
    for (int s = 0; s < a.n_splits; ++s) {
        const float wgt = __builtin_amdgcn_exp2f(rec[s * (D + 2) + D] - M);
        acc += rec[s * (D + 2) + col] * wgt;
        den += rec[s * (D + 2) + D + 1] * wgt;
    }
    const float out = valid ? acc / den : __builtin_nanf("");
    a.o[((int64_t)b * a.n_q_heads + hq) * D + col] = (__bf16)out;
    if (a.lse && col == 0)
        a.lse[(int64_t)b * a.n_q_heads + hq] = valid ? M * 0.6931471805599453f + __logf(den) : __builtin_nanf("");
}

template <int D, int G>
void launch_split(const DecodeArgs &a, int batch, hipStream_t st) {
    hipLaunchKernelGGL((ksa_decode_split_kernel<D, G>), dim3(a.n_splits, a.n_kv_heads, batch), dim3(NT), 0, st, a);
}

template <int D>
int launch_all(const DecodeArgs &a, int batch, hipStream_t st) {
    switch (a.n_q_heads / a.n_kv_heads) {
        case 1: launch_split<D, 1>(a, batch, st); break;
        case 2: launch_split<D, 2>(a, batch, st); break;
        case 4: launch_split<D, 4>(a, batch, st); break;
        case 8: launch_split<D, 8>(a, batch, st); break;
        default: return KSA_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL(ksa_decode_merge_kernel<D>, dim3(a.n_q_heads, batch), dim3(D), 0, st, a);
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}

}  // namespace

// Enough spans that the launch has about six workgroups per compute unit (1536 in all: measured best at batch 16 to
// 128 on the 128K cache, where 2048 workgroups run 4 to 12 % longer), but no span shorter than 768 rows (shorter
// spans are dominated by the workgroup's fixed costs: measured at batch 1 and 4).
int ksa_decode_default_splits(const ksa_params *p) {
    const int64_t groups = (int64_t)p->batch * p->n_kv_heads;
    const int64_t rows = (int64_t)(p->n_text / p->chunk_len) * p->n_summary + (int64_t)(p->window_chunks + 1) * p->chunk_len;
    int64_t want = (1536 + groups - 1) / groups;
    const int64_t most = rows / 768 > 1 ? rows / 768 : 1;
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    return (int)want;
}

// Device address of `scratch` on the current device, resolved once per device (with that device current).
int ksa_decode_static_scratch(float **ptr) {
    constexpr int MAX_DEVICES = 64;
    static void *addr[MAX_DEVICES] = {};
    static std::mutex lock;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return KSA_ERR_HIP;
    std::lock_guard<std::mutex> guard(lock);
    if (!addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KSA_ERR_HIP;
        addr[dev] = p;
    }
    *ptr = static_cast<float *>(addr[dev]);
    return KSA_OK;
}

int ksa_launch_decode(const KsaDecodeLaunch &L, void *stream) {
    DecodeArgs a;
    a.q = static_cast<const __bf16 *>(L.q);
    a.k = static_cast<const __bf16 *>(L.k_cache);
    a.v = static_cast<const __bf16 *>(L.v_cache);
    a.pos = L.pos;
    a.o = static_cast<__bf16 *>(L.o);
    a.lse = L.lse;
    a.ws = L.workspace;
    for (int x = 0; x < 3; ++x) a.cs[x] = L.cache_strides[x];
    a.n_splits = L.n_splits;
    a.s_cap = L.summary_capacity;
    a.kind = L.kind;
    a.self_only = (L.p.flags & 1u) ? 1 : 0;
    a.c = L.p.chunk_len;
    a.m = L.p.n_summary;
    a.C = L.p.window_chunks;
    a.n_text = L.p.n_text;
    a.n_q_heads = L.p.n_q_heads;
    a.n_kv_heads = L.p.n_kv_heads;
    a.scale_log2e = L.p.softmax_scale * 1.4426950408889634f;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (L.p.head_dim == 128) return launch_all<128>(a, L.p.batch, st);
    if (L.p.head_dim == 64) return launch_all<64>(a, L.p.batch, st);
    return KSA_ERR_UNSUPPORTED;
}
