// KSA prefill forward for gfx950: flash-style online softmax over the live key tiles of the schedule.
//
// One workgroup (4 wavefronts of 64 lanes) owns one query tile of one (batch, query head).  Each wave
// owns 32*QB query rows.  Scores are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the 32x32 result block gives lane l the query column l%32 and the key rows 8*(g/4) + 4*(l/32) + g%4
// for its 16 registers g, so
//   - the softmax statistics of a query row live in one lane pair (l, l^32): the row max / sum are
//     in-lane reductions plus one v_permlane32_swap, no LDS, no shuffle tree;
//   - the same registers, rounded to bf16, are already the B operand of O^T += V^T P^T (eight registers
//     of one lane = eight k slots), so P never leaves the register file;
//   - the rescale factor of the output accumulator is a per-lane scalar.
// K and V tiles (64 keys) are staged in LDS with an XOR swizzle of the 16-byte chunks; the K operand is
// read with ds_read_b128, the V^T operand with the gfx950 transposing read ds_read_b64_tr_b16, which hands
// each lane four consecutive keys of one head-dim column out of a row-major [key][d] tile.
//
// Rows are addressed in two compact index spaces, text index i and summary ordinal u (Eq. 1):
//   augmented row of text i    = (i / c) * (c + m) + i % c
//   augmented row of summary u = (u / m) * (c + m) + c + u % m
// and every query row's visible set is one range of each space (Eq. 3), so a masked tile costs two
// integer compares per score.
#include <hip/hip_runtime.h>

#include "ksa_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NW = 4;                         // waves per workgroup
constexpr int BN = KSA_K_TILE;                // keys per tile
constexpr int QB = KSA_Q_TILE / (NW * 32);    // 32-row query blocks per wave
static_assert(KSA_Q_TILE == NW * QB * 32, "query tile must be a whole number of 32-row blocks per wave");
static_assert(BN == 64, "key tile is two 32-key MFMA blocks");

struct PrefillArgs {
    const __bf16 *q, *k, *v;
    __bf16 *o;
    float *lse;
    int64_t qs[3], ks[3], os[3];   // {batch, row, head} strides in elements
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t c, m, C, w;            // chunk_len, n_summary, window_chunks, c + m
    int32_t c_shift, m_shift;      // log2 when a power of two, else -1
    int32_t group;                 // Hq / Hkv
    int32_t n_q_heads;
    int32_t self_only;
    int64_t aug_len;
    float scale, scale_log2e;
};

__device__ __forceinline__ int div_by(int x, int d, int shift) { return shift >= 0 ? (x >> shift) : (x / d); }

__device__ __forceinline__ int aug_row(const PrefillArgs &a, int space, int idx) {
    if (space == KSA_SPACE_TEXT) {
        const int j = div_by(idx, a.c, a.c_shift);
        return j * a.w + (idx - j * a.c);
    }
    const int j = div_by(idx, a.m, a.m_shift);
    return j * a.w + a.c + (idx - j * a.m);
}

__device__ __forceinline__ float other_half(float x) {
    // value held by lane l^32
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned mine_is_low = threadIdx.x & 32 ? r[0] : r[1];
    return __builtin_bit_cast(float, mine_is_low);
}

template <int D>
__device__ __forceinline__ int k_tile_off(int row, int chunk) {
    return row * (D * 2) + ((chunk ^ (row & (D / 8 - 1))) << 4);
}
template <int D>
__device__ __forceinline__ int v_tile_off(int row, int chunk) {
    return row * (D * 2) + ((chunk ^ (((row & 3) << 2) & (D / 8 - 1))) << 4);
}

template <int D>
__global__ __launch_bounds__(NW * 64) void ksa_prefill_kernel(const PrefillArgs a) {
    constexpr int CH = D / 8;            // 16-byte chunks per row
    constexpr int RPP = NW * 64 / CH;    // tile rows loaded per pass of the workgroup
    constexpr int NP = BN / RPP;         // passes per tile
    constexpr int KS = D / 16;           // k steps of the score MFMA
    constexpr int DB = D / 32;           // 32-column blocks of the output

    __shared__ __attribute__((aligned(16))) unsigned char lds_k[BN * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char lds_v[BN * D * 2];

    const KsaWgEntry ent = a.entries[blockIdx.x];
    if (ent.item < 0) return;
    const KsaWorkItem &item = a.items[ent.item];
    const int b = ent.batch, hq = ent.q_head, hkv = hq / a.group;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, h = lane >> 5;

    const int q_space = item.q_space, q_begin = item.q_begin, q_end = item.q_begin + item.q_count;
    const int n_seg = item.n_seg;

    // ---- per-lane query rows: visible ranges (Eq. 3) and the Q operand -------------------------
    int lo[QB][2], hi[QB][2];   // [.][space]
    int q_aug[QB];
    bool q_valid[QB];
    bf16x8 qreg[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int idx = q_begin + (wave * QB + qb) * 32 + r;
        q_valid[qb] = idx < q_end;
        const int idc = q_valid[qb] ? idx : q_end - 1;
        q_aug[qb] = aug_row(a, q_space, idc);
        if (q_space == KSA_SPACE_TEXT) {
            const int j = div_by(idc, a.c, a.c_shift);
            const int first = j - a.C > 0 ? j - a.C : 0;
            lo[qb][KSA_SPACE_SUMMARY] = 0;
            hi[qb][KSA_SPACE_SUMMARY] = first * a.m;
            lo[qb][KSA_SPACE_TEXT] = first * a.c;
            hi[qb][KSA_SPACE_TEXT] = idc + 1;
        } else {
            const int j = div_by(idc, a.m, a.m_shift);
            lo[qb][KSA_SPACE_SUMMARY] = a.self_only ? idc : j * a.m;
            hi[qb][KSA_SPACE_SUMMARY] = idc + 1;
            lo[qb][KSA_SPACE_TEXT] = j * a.c;
            hi[qb][KSA_SPACE_TEXT] = (j + 1) * a.c;
        }
        if (!q_valid[qb]) {
            lo[qb][0] = lo[qb][1] = 0x7fffffff;
            hi[qb][0] = hi[qb][1] = 0;
        }
        const __bf16 *qp = a.q + b * a.qs[0] + (int64_t)q_aug[qb] * a.qs[1] + hq * a.qs[2] + h * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (q_valid[qb])
                qreg[qb][s] = *reinterpret_cast<const bf16x8 *>(qp + s * 16);
            else
                qreg[qb][s] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    // union of the wave's rows' ranges per space: a tile outside it is skipped by the whole wave
    int wlo[2], whi[2];
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
        int mn = lo[0][sp], mx = hi[0][sp];
#pragma unroll
        for (int qb = 1; qb < QB; ++qb) {
            mn = min(mn, lo[qb][sp]);
            mx = max(mx, hi[qb][sp]);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn = min(mn, __shfl_xor(mn, off));
            mx = max(mx, __shfl_xor(mx, off));
        }
        wlo[sp] = mn;
        whi[sp] = mx;
    }

    // ---- accumulators -------------------------------------------------------------------------
    f32x16 oacc[QB][DB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -1e30f;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 16; ++g) oacc[qb][db][g] = 0.f;
    }

    const __bf16 *kbase = a.k + b * a.ks[0] + hkv * a.ks[2];
    const __bf16 *vbase = a.v + b * a.ks[0] + hkv * a.ks[2];
    const int ld_chunk = tid % CH, ld_row = tid / CH;

    uint4 kreg[NP], vreg[NP];
    auto fetch = [&](int seg, int kt) {
        const int space = item.seg[seg].space, last = item.seg[seg].end - 1;
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
            int kc = kt + ps * RPP + ld_row;
            kc = kc < last ? kc : last;   // rows past the run are clamped (and masked out below)
            const int64_t off = (int64_t)aug_row(a, space, kc) * a.ks[1] + ld_chunk * 8;
            kreg[ps] = *reinterpret_cast<const uint4 *>(kbase + off);
            vreg[ps] = *reinterpret_cast<const uint4 *>(vbase + off);
        }
    };

    int seg = 0, kt = item.seg[0].begin;
    fetch(seg, kt);

    while (seg < n_seg) {
        const int cur_seg = seg, cur_kt = kt;
        kt += BN;
        if (kt >= item.seg[seg].end) {
            ++seg;
            if (seg < n_seg) kt = item.seg[seg].begin;
        }
        __syncthreads();   // everyone is done reading the previous tile
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
            const int row = ps * RPP + ld_row;
            *reinterpret_cast<uint4 *>(lds_k + k_tile_off<D>(row, ld_chunk)) = kreg[ps];
            *reinterpret_cast<uint4 *>(lds_v + v_tile_off<D>(row, ld_chunk)) = vreg[ps];
        }
        __syncthreads();
        if (seg < n_seg) fetch(seg, kt);   // next tile's global loads fly during this tile's math

        const int space = item.seg[cur_seg].space;
        const bool masked = item.seg[cur_seg].masked != 0;
        const int seg_begin = item.seg[cur_seg].begin, seg_end = item.seg[cur_seg].end;
        if (masked) {
            const int t_lo = max(cur_kt, seg_begin), t_hi = min(cur_kt + BN, seg_end);
            if (t_lo >= whi[space] || t_hi <= wlo[space]) continue;   // wave-uniform: nothing visible here
        }

        // ---- S^T = K Q^T ----------------------------------------------------------------------
        f32x16 sacc[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 16; ++g) sacc[qb][kb][g] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(lds_k + k_tile_off<D>(kb * 32 + r, 2 * s + h));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    sacc[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[qb][s], sacc[qb][kb], 0, 0, 0);
            }
        }

        // ---- mask + online softmax ------------------------------------------------------------
        bf16x8 pb[QB][2][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (masked) {
                const int elo = max(lo[qb][space], seg_begin), ehi = min(hi[qb][space], seg_end);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 16; ++g) {
                        const int key = cur_kt + kb * 32 + 8 * (g / 4) + 4 * h + (g % 4);
                        if (key < elo || key >= ehi) sacc[qb][kb][g] = -INFINITY;
                    }
            }
            float tmax = sacc[qb][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 16; ++g) tmax = fmaxf(tmax, sacc[qb][kb][g]);
            tmax = fmaxf(tmax, other_half(tmax));
            const float m_new = fmaxf(m_run[qb], tmax);
            const float msl = m_new * a.scale_log2e;
            // (m_old - m_new) first: equal maxima (also the -1e30 start value) must give exactly 2^0
            const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * a.scale_log2e);
            m_run[qb] = m_new;
            float rsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 16; ++g) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][g], a.scale_log2e, -msl));
                    rsum += pv;
                    pb[qb][kb][g / 8][g % 8] = (__bf16)pv;
                }
            rsum += other_half(rsum);
            l_run[qb] = l_run[qb] * alpha + rsum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 16; ++g) oacc[qb][db][g] *= alpha;
        }

        // ---- O^T += V^T P^T -------------------------------------------------------------------
        {
            const int grp = lane >> 4, li = lane & 15;
            // lane (grp, li) supplies the address of key 4*(grp/2) + li/4, columns 16*(grp%2) + 4*(li%4) .. +3
            const int t_row = 4 * (grp >> 1) + (li >> 2);
            const int t_col = 16 * (grp & 1) + 4 * (li & 3);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int base = kb * 32 + hf * 16;
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const int col = db * 32 + t_col;
                        const int o0 = v_tile_off<D>(base + t_row, col >> 3) + ((col & 7) << 1);
                        const int o1 = v_tile_off<D>(base + 8 + t_row, col >> 3) + ((col & 7) << 1);
                        const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(lds_v + o0));
                        const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(lds_v + o1));
                        const s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                        const bf16x8 va = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            oacc[qb][db] =
                                __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[qb][kb][hf], oacc[qb][db], 0, 0, 0);
                    }
                }
        }
    }

    // ---- epilogue: O = O^T / l, LSE ---------------------------------------------------------------
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        if (!q_valid[qb]) continue;
        const float inv = 1.0f / l_run[qb];
        __bf16 *op = a.o + b * a.os[0] + (int64_t)q_aug[qb] * a.os[1] + hq * a.os[2];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(oacc[qb][db][g4 * 4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + db * 32 + g4 * 8 + h * 4) = pk;
            }
        if (a.lse && h == 0)
            a.lse[((int64_t)b * a.n_q_heads + hq) * a.aug_len + q_aug[qb]] = m_run[qb] * a.scale + __logf(l_run[qb]);
    }
}

int log2_exact(int x) {
    if (x <= 0 || (x & (x - 1))) return -1;
    int s = 0;
    while ((1 << s) < x) ++s;
    return s;
}

}  // namespace

int ksa_launch_prefill(const KsaPrefillLaunch &L, void *stream) {
    PrefillArgs a;
    a.q = static_cast<const __bf16 *>(L.q);
    a.k = static_cast<const __bf16 *>(L.k);
    a.v = static_cast<const __bf16 *>(L.v);
    a.o = static_cast<__bf16 *>(L.o);
    a.lse = L.lse;
    for (int x = 0; x < 3; ++x) a.qs[x] = L.q_strides[x], a.ks[x] = L.kv_strides[x], a.os[x] = L.o_strides[x];
    a.items = L.items;
    a.entries = L.entries;
    a.c = L.p.chunk_len;
    a.m = L.p.n_summary;
    a.C = L.p.window_chunks;
    a.w = a.c + a.m;
    a.c_shift = log2_exact(a.c);
    a.m_shift = log2_exact(a.m);
    a.group = L.p.n_q_heads / L.p.n_kv_heads;
    a.n_q_heads = L.p.n_q_heads;
    a.self_only = (L.p.flags & KSA_FLAG_SUMMARY_SELF_ONLY) ? 1 : 0;
    a.aug_len = L.aug_len;
    a.scale = L.p.softmax_scale;
    a.scale_log2e = L.p.softmax_scale * 1.4426950408889634f;
    if (L.n_entries <= 0) return KSA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (L.p.head_dim == 128)
        hipLaunchKernelGGL(ksa_prefill_kernel<128>, dim3(L.n_entries), dim3(NW * 64), 0, st, a);
    else if (L.p.head_dim == 64)
        hipLaunchKernelGGL(ksa_prefill_kernel<64>, dim3(L.n_entries), dim3(NW * 64), 0, st, a);
    else
        return KSA_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}
