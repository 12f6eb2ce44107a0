// KSA prefill backward for gfx950: dQ, dK, dV of O = softmax(Q K^T scale + M_KSA) V for an upstream gradient
// G = dLoss/dO, from the saved log-sum-exp of the forward pass (the paper's block-sparse kernel serves training
// as well as prefill; it prints no backward formula, this is the derivative of the attention definition):
//   P_ij  = exp(scale q_i.k_j - lse_i) for visible pairs, else 0
//   dV_j  = sum_i P_ij G_i
//   dS_ij = P_ij (G_i.v_j - delta_i),  delta_i = G_i.O_i  (= sum_l P_il G_i.v_l)
//   dQ_i  = scale sum_j dS_ij k_j,     dK_j = scale sum_i dS_ij q_i
// Three kernels, no atomics, results independent of the launch order:
//   ksa_bwd_delta_kernel  delta_i per (batch, head, row);
//   ksa_bwd_dq_kernel     one workgroup per query tile of the forward schedule walks that tile's key runs;
//   ksa_bwd_dkv_kernel    one workgroup per 128-key tile of an index space walks the query rows that can see it
//                         (two runs, closed form from Eq. 3), for every query head of the KV head's group.
// Both main kernels recompute the scores with v_mfma_f32_32x32x16_bf16 and keep the result block in the layout
// whose registers are the B operand of the next product: dQ works on S^T (keys x queries, the forward kernel's
// layout, per-lane query statistics), dK/dV on S (queries x keys, per-lane key, per-register query statistics
// read from LDS).  The operand that has to be contracted over the tile's rows (K^T, Q^T, G^T) is read out of the
// same row-major LDS tile with the gfx950 transposing read (ds_read_b64_tr_b16).  Every score is masked with its
// row's visible range (Eq. 3); there is no unmasked fast path yet.
#include <hip/hip_runtime.h>

#include "ksa_device.h"
#include "ksa_internal.h"

namespace {

constexpr int NW = 4;                         // waves per workgroup
constexpr int BN = KSA_K_TILE;                // rows of an LDS tile
constexpr int RW = BN / NW;                   // rows of a tile each wave fetches
constexpr int QB = KSA_Q_TILE / (NW * 32);    // 32-row query blocks per wave (dQ kernel)
constexpr int KEYS_PER_WG = NW * 32;          // dK/dV kernel: 32 keys per wave
static_assert(BN == 64, "an LDS tile is two 32-row MFMA blocks");

struct BwdArgs {
    const __bf16 *q, *k, *v, *o, *g;          // g: upstream gradient dLoss/dO, laid out like o
    const float *lse;                         // [B, Hq, L] natural-log sum-exp of the forward pass
    float *delta;                             // [B, Hq, L] workspace
    __bf16 *dq, *dk, *dv;
    int64_t qs[3], ks[3], os[3], dqs[3], dks[3];   // {batch, row, head} strides in elements (os: o and g)
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t c, m, C, w;                       // chunk_len, n_summary, window_chunks, c + m
    int32_t c_shift, m_shift;
    int32_t group, n_q_heads, n_kv_heads, self_only;
    int32_t n_text, n_sum;                    // rows per index space
    int32_t sum_tiles;                        // dK/dV grid: summary-space key tiles come first (the long ones)
    int64_t aug_len;
    float scale, scale_log2e;
};

// LDS tile: row-major [64][D] bf16; the 16-byte chunk index is XORed with a function of the row that spreads both
// the 16 rows of a plain 16-byte operand read and the 4 rows of a transposing read over different banks.
template <int D>
__device__ __forceinline__ int swz(int row) { return (((row & 3) << 2) | ((row >> 2) & 3)) & (D / 8 - 1); }

// Rows first .. first + 63 (clamped to `last`) of one index space -> LDS tile.  base points at (batch, head).
template <int D>
__device__ __forceinline__ void load_tile(const BwdArgs &a, const __bf16 *base, int64_t row_stride, int space, int first,
                                          int last, unsigned char *tile, int wave, int lane) {
    constexpr int CH = D / 8, RPI = 64 / CH, NI = RW / RPI;
    static_assert(RW % RPI == 0 && NI >= 1, "a wave's share of a tile is a whole number of load instructions");
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = RW * wave + RPI * i + lane / CH;
        const int pch = lane % CH;
        int idx = first + row;
        idx = idx < last ? idx : last;
        const __bf16 *src = base + (int64_t)aug_row(a, space, idx) * row_stride + ((pch ^ swz<D>(row)) << 3);
        lds_direct_load_16(src, tile + (RW * wave + RPI * i) * (D * 2));
    }
}

struct LaneLds {
    int rows;           // plain operand read: row r, chunk (h ^ swizzle(r)); XOR (s << 5) selects k step s
    int t_row, t_col;   // transposing read: this lane addresses tile row t_row (+ base), columns t_col .. t_col + 3
};

template <int D>
__device__ __forceinline__ LaneLds lane_lds(int lane) {
    const int r = lane & 31, h = lane >> 5, grp = lane >> 4, li = lane & 15;
    LaneLds L;
    L.rows = r * (D * 2) + ((h ^ swz<D>(r)) << 4);
    L.t_row = 4 * (grp >> 1) + (li >> 2);
    L.t_col = 16 * (grp & 1) + 4 * (li & 3);
    return L;
}

// A operand [32 tile rows of block rb] x [16 head-dim columns of k step s]
template <int D>
__device__ __forceinline__ bf16x8 read_rows(const unsigned char *tile, const LaneLds &ll, int rb, int s) {
    return *reinterpret_cast<const bf16x8 *>(tile + ((ll.rows ^ (s << 5)) + rb * 32 * (D * 2)));
}

// A operand [32 head-dim columns of block db] x [16 tile rows from R0]: lane l gets column 32 db + l % 32 and the
// rows R0 + 4 h + (0..3), R0 + 8 + 4 h + (0..3), h = l / 32 -- the order in which a lane's registers of a 32x32
// result block hold its rows, so that eight result registers are the matching B operand.
template <int D>
__device__ __forceinline__ bf16x8 read_cols(const unsigned char *tile, const LaneLds &ll, int R0, int db) {
    auto at = [&](int R) {
        const int row = R + ll.t_row;
        return row * (D * 2) + (((db * 4 + (ll.t_col >> 3)) ^ swz<D>(row)) << 4) + ((ll.t_col & 7) << 1);
    };
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(tile + at(R0)));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(tile + at(R0 + 8)));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ void zero(f32x16 &x) {
#pragma unroll
    for (int g = 0; g < 16; ++g) x[g] = 0.f;
}

// Visible key range [lo, hi) of query idx (index space q_space) among the keys of index space k_space (Eq. 3).
__device__ __forceinline__ void visible_range(const BwdArgs &a, int q_space, int idx, int k_space, int &lo, int &hi) {
    if (q_space == KSA_SPACE_TEXT) {
        const int j = div_by(idx, a.c, a.c_shift);
        const int first = j - a.C > 0 ? j - a.C : 0;
        if (k_space == KSA_SPACE_TEXT)
            lo = first * a.c, hi = idx + 1;
        else
            lo = 0, hi = first * a.m;
    } else {
        const int j = div_by(idx, a.m, a.m_shift);
        if (k_space == KSA_SPACE_TEXT)
            lo = j * a.c, hi = (j + 1) * a.c;
        else
            lo = a.self_only ? idx : j * a.m, hi = idx + 1;
    }
}

// ---- delta_i = G_i . O_i ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void ksa_bwd_delta_kernel(const BwdArgs a, int64_t n_rows /* B * L * Hq */) {
    constexpr int CH = D / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t rh = idx / CH;
    const int piece = (int)(idx % CH);
    const bool live = rh < n_rows;
    if (!live) rh = n_rows - 1;
    const int hq = (int)(rh % a.n_q_heads);
    const int64_t br = rh / a.n_q_heads;
    const int64_t aq = br % a.aug_len, b = br / a.aug_len;
    const int64_t off = b * a.os[0] + aq * a.os[1] + hq * a.os[2] + piece * 8;
    const bf16x8 o8 = *reinterpret_cast<const bf16x8 *>(a.o + off);
    const bf16x8 g8 = *reinterpret_cast<const bf16x8 *>(a.g + off);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += (float)o8[e] * (float)g8[e];
#pragma unroll
    for (int d = CH / 2; d > 0; d >>= 1) s += __shfl_xor(s, d);
    if (live && piece == 0) a.delta[(b * a.n_q_heads + hq) * a.aug_len + aq] = s;
}

// ---- dQ -----------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(NW * 64) void ksa_bwd_dq_kernel(const BwdArgs a) {
    constexpr int KS = D / 16, DB = D / 32, BYTES = BN * D * 2;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * BYTES];
    unsigned char *k_tile = lds, *v_tile = lds + BYTES;

    const KsaWgEntry ent = a.entries[blockIdx.x];
    if (ent.item < 0) return;
    const KsaWorkItem &item = a.items[ent.item];
    const int b = ent.batch, hq = ent.q_head, hkv = hq / a.group;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, h = lane >> 5;
    const LaneLds ll = lane_lds<D>(lane);
    const int q_space = item.q_space, q_begin = item.q_begin, q_end = item.q_begin + item.q_count;

    int q_aug[QB];
    bool q_valid[QB];
    int idc[QB];
    float lse2[QB], dl[QB];
    bf16x8 qreg[QB][KS], greg[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int idx = q_begin + (wave * QB + qb) * 32 + r;
        q_valid[qb] = idx < q_end;
        idc[qb] = q_valid[qb] ? idx : q_end - 1;
        q_aug[qb] = aug_row(a, q_space, idc[qb]);
        const __bf16 *qp = a.q + b * a.qs[0] + (int64_t)q_aug[qb] * a.qs[1] + hq * a.qs[2] + h * 8;
        const __bf16 *gp = a.g + b * a.os[0] + (int64_t)q_aug[qb] * a.os[1] + hq * a.os[2] + h * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            qreg[qb][s] = *reinterpret_cast<const bf16x8 *>(qp + s * 16);
            greg[qb][s] = *reinterpret_cast<const bf16x8 *>(gp + s * 16);
        }
        const int64_t stat = ((int64_t)b * a.n_q_heads + hq) * a.aug_len + q_aug[qb];
        lse2[qb] = a.lse[stat] * 1.4426950408889634f;
        dl[qb] = a.delta[stat];
    }
    f32x16 dqacc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) zero(dqacc[qb][db]);

    const __bf16 *kbase = a.k + b * a.ks[0] + hkv * a.ks[2];
    const __bf16 *vbase = a.v + b * a.ks[0] + hkv * a.ks[2];
    const float sl = a.scale_log2e;

    for (int seg = 0; seg < item.n_seg; ++seg) {
        const int space = item.seg[seg].space, seg_begin = item.seg[seg].begin, seg_end = item.seg[seg].end;
        int elo[QB], ehi[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            int lo, hi;
            visible_range(a, q_space, idc[qb], space, lo, hi);
            elo[qb] = lo > seg_begin ? lo : seg_begin;
            ehi[qb] = hi < seg_end ? hi : seg_end;
            if (!q_valid[qb]) elo[qb] = 0x7fffffff, ehi[qb] = 0;
        }
        for (int kt = seg_begin; kt < seg_end; kt += BN) {
            __syncthreads();   // everybody is done with the previous tile
            load_tile<D>(a, kbase, a.ks[1], space, kt, seg_end - 1, k_tile, wave, lane);
            load_tile<D>(a, vbase, a.ks[1], space, kt, seg_end - 1, v_tile, wave, lane);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                // nothing of this tile is visible to any row of the block: skip the math (wave-uniform)
                const bool some = elo[qb] < kt + BN && ehi[qb] > kt;
                if (__builtin_amdgcn_ballot_w64(some) == 0) continue;
                f32x16 sacc[2], gacc[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) zero(sacc[kb]), zero(gacc[kb]);
#pragma unroll
                for (int s = 0; s < KS; ++s)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        const bf16x8 ka = read_rows<D>(k_tile, ll, kb, s);
                        const bf16x8 va = read_rows<D>(v_tile, ll, kb, s);
                        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[qb][s], sacc[kb], 0, 0, 0);
                        gacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, greg[qb][s], gacc[kb], 0, 0, 0);
                    }
                // dS^T in the B-operand layout: lane = query, eight registers = eight keys
                bf16x8 pb[2][2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 16; ++g) {
                        const int key = kt + kb * 32 + 8 * (g / 4) + 4 * h + (g % 4);
                        const bool vis = key >= elo[qb] && key < ehi[qb];
                        const float p = vis ? __builtin_amdgcn_exp2f(fmaf(sacc[kb][g], sl, -lse2[qb])) : 0.f;
                        pb[kb][g / 8][g % 8] = (__bf16)(p * (gacc[kb][g] - dl[qb]));
                    }
                // dQ^T += K^T dS^T
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const bf16x8 kt_op = read_cols<D>(k_tile, ll, kb * 32 + hf * 16, db);
                            dqacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_op, pb[kb][hf], dqacc[qb][db], 0, 0, 0);
                        }
            }
        }
    }

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        if (!q_valid[qb]) continue;
        __bf16 *op = a.dq + b * a.dqs[0] + (int64_t)q_aug[qb] * a.dqs[1] + hq * a.dqs[2];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(dqacc[qb][db][g4 * 4 + e] * a.scale);
                *reinterpret_cast<bf16x4 *>(op + db * 32 + g4 * 8 + h * 4) = pk;
            }
    }
}

// ---- dK, dV -------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(NW * 64) void ksa_bwd_dkv_kernel(const BwdArgs a) {
    constexpr int KS = D / 16, DB = D / 32, BYTES = BN * D * 2;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * BYTES];
    __shared__ __attribute__((aligned(16))) float st_lse[BN], st_dl[BN];
    __shared__ __attribute__((aligned(16))) int st_lo[BN], st_hi[BN];
    unsigned char *q_tile = lds, *g_tile = lds + BYTES;

    int t = blockIdx.x, space = KSA_SPACE_SUMMARY;
    if (t >= a.sum_tiles) t -= a.sum_tiles, space = KSA_SPACE_TEXT;
    const int hkv = blockIdx.y, b = blockIdx.z;
    const int n_space = space == KSA_SPACE_TEXT ? a.n_text : a.n_sum;
    const int k0 = t * KEYS_PER_WG;
    const int k1 = k0 + KEYS_PER_WG < n_space ? k0 + KEYS_PER_WG : n_space;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, h = lane >> 5;
    const LaneLds ll = lane_lds<D>(lane);

    // this lane's key: B operands of S = Q K^T and of G V^T
    const int key = k0 + wave * 32 + r;
    const bool key_valid = key < n_space;
    const int key_aug = aug_row(a, space, key_valid ? key : n_space - 1);
    bf16x8 kreg[KS], vreg[KS];
    {
        const __bf16 *kp = a.k + b * a.ks[0] + (int64_t)key_aug * a.ks[1] + hkv * a.ks[2] + h * 8;
        const __bf16 *vp = a.v + b * a.ks[0] + (int64_t)key_aug * a.ks[1] + hkv * a.ks[2] + h * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kreg[s] = *reinterpret_cast<const bf16x8 *>(kp + s * 16);
            vreg[s] = *reinterpret_cast<const bf16x8 *>(vp + s * 16);
        }
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) zero(dkacc[db]), zero(dvacc[db]);

    // The query rows that can see a key of [k0, k1): one run of text rows, one of summary rows (supersets: every
    // score is masked below).  Text keys of chunks jl..jh are seen by the text rows from k0 to the end of chunk
    // jh + C and by the summary rows of chunks jl..jh; summary keys of chunks jl..jh by the text rows from chunk
    // jl + C + 1 on and by the summary rows of their own chunks from k0 on.
    int run_space[2], run_begin[2], run_end[2];
    run_space[0] = KSA_SPACE_TEXT, run_space[1] = KSA_SPACE_SUMMARY;
    if (space == KSA_SPACE_TEXT) {
        const int jl = div_by(k0, a.c, a.c_shift), jh = div_by(k1 - 1, a.c, a.c_shift);
        const int64_t te = ((int64_t)jh + a.C + 1) * a.c;
        run_begin[0] = k0, run_end[0] = te < a.n_text ? (int)te : a.n_text;
        const int64_t se = ((int64_t)jh + 1) * a.m;
        run_begin[1] = jl * a.m, run_end[1] = se < a.n_sum ? (int)se : a.n_sum;
    } else {
        const int jl = div_by(k0, a.m, a.m_shift), jh = div_by(k1 - 1, a.m, a.m_shift);
        const int64_t tb = ((int64_t)jl + a.C + 1) * a.c;
        run_begin[0] = tb < a.n_text ? (int)tb : a.n_text, run_end[0] = a.n_text;
        const int64_t se = ((int64_t)jh + 1) * a.m;
        run_begin[1] = k0, run_end[1] = se < a.n_sum ? (int)se : a.n_sum;
    }
    const float sl = a.scale_log2e;

    for (int hq = hkv * a.group; hq < (hkv + 1) * a.group; ++hq) {
        const __bf16 *qbase = a.q + b * a.qs[0] + hq * a.qs[2];
        const __bf16 *gbase = a.g + b * a.os[0] + hq * a.os[2];
        const int64_t stat = ((int64_t)b * a.n_q_heads + hq) * a.aug_len;
        for (int run = 0; run < 2; ++run) {
            const int q_space = run_space[run], q_end = run_end[run];
            for (int qt = run_begin[run]; qt < q_end; qt += BN) {
                __syncthreads();   // everybody is done with the previous tile and its row statistics
                load_tile<D>(a, qbase, a.qs[1], q_space, qt, q_end - 1, q_tile, wave, lane);
                load_tile<D>(a, gbase, a.os[1], q_space, qt, q_end - 1, g_tile, wave, lane);
                if (tid < BN) {
                    const int qi = qt + tid;
                    int lo = 0x7fffffff, hi = 0;
                    float l2 = 0.f, dd = 0.f;
                    if (qi < q_end) {
                        visible_range(a, q_space, qi, space, lo, hi);
                        const int aq = aug_row(a, q_space, qi);
                        l2 = a.lse[stat + aq] * 1.4426950408889634f;
                        dd = a.delta[stat + aq];
                    }
                    st_lo[tid] = lo, st_hi[tid] = hi, st_lse[tid] = l2, st_dl[tid] = dd;
                }
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    f32x16 sacc, gacc;
                    zero(sacc), zero(gacc);
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        const bf16x8 qa = read_rows<D>(q_tile, ll, qb, s);
                        const bf16x8 ga = read_rows<D>(g_tile, ll, qb, s);
                        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kreg[s], sacc, 0, 0, 0);
                        gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vreg[s], gacc, 0, 0, 0);
                    }
                    // P and dS in the B-operand layout: lane = key, eight registers = eight query rows
                    bf16x8 pp[2], pd[2];
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        const int row0 = qb * 32 + 8 * gg + 4 * h;
                        const f32x4 l4 = *reinterpret_cast<const f32x4 *>(&st_lse[row0]);
                        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(&st_dl[row0]);
                        const int4 lo4 = *reinterpret_cast<const int4 *>(&st_lo[row0]);
                        const int4 hi4 = *reinterpret_cast<const int4 *>(&st_hi[row0]);
                        const int lo_e[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi_e[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int g = gg * 4 + e;
                            const bool vis = key >= lo_e[e] && key < hi_e[e];
                            const float p = vis ? __builtin_amdgcn_exp2f(fmaf(sacc[g], sl, -l4[e])) : 0.f;
                            pp[g / 8][g % 8] = (__bf16)p;
                            pd[g / 8][g % 8] = (__bf16)(p * (gacc[g] - d4[e]));
                        }
                    }
                    // dV^T += G^T P,  dK^T += Q^T dS
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const bf16x8 gt_op = read_cols<D>(g_tile, ll, qb * 32 + hf * 16, db);
                            const bf16x8 qt_op = read_cols<D>(q_tile, ll, qb * 32 + hf * 16, db);
                            dvacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt_op, pp[hf], dvacc[db], 0, 0, 0);
                            dkacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt_op, pd[hf], dkacc[db], 0, 0, 0);
                        }
                }
            }
        }
    }

    if (!key_valid) return;
    __bf16 *kp = a.dk + b * a.dks[0] + (int64_t)key_aug * a.dks[1] + hkv * a.dks[2];
    __bf16 *vp = a.dv + b * a.dks[0] + (int64_t)key_aug * a.dks[1] + hkv * a.dks[2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            bf16x4 pk, pv;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pk[e] = (__bf16)(dkacc[db][g4 * 4 + e] * a.scale);
                pv[e] = (__bf16)dvacc[db][g4 * 4 + e];
            }
            *reinterpret_cast<bf16x4 *>(kp + db * 32 + g4 * 8 + h * 4) = pk;
            *reinterpret_cast<bf16x4 *>(vp + db * 32 + g4 * 8 + h * 4) = pv;
        }
}

}  // namespace

size_t ksa_prefill_bwd_workspace_size(const ksa_params &p, int64_t aug_len) {
    return (size_t)((int64_t)p.batch * p.n_q_heads * aug_len * (int64_t)sizeof(float));
}

int ksa_launch_prefill_bwd(const KsaPrefillBwdLaunch &L, void *stream) {
    BwdArgs a;
    a.q = static_cast<const __bf16 *>(L.q);
    a.k = static_cast<const __bf16 *>(L.k);
    a.v = static_cast<const __bf16 *>(L.v);
    a.o = static_cast<const __bf16 *>(L.o);
    a.g = static_cast<const __bf16 *>(L.d_o);
    a.lse = L.lse;
    a.delta = static_cast<float *>(L.workspace);
    a.dq = static_cast<__bf16 *>(L.dq);
    a.dk = static_cast<__bf16 *>(L.dk);
    a.dv = static_cast<__bf16 *>(L.dv);
    for (int x = 0; x < 3; ++x) {
        a.qs[x] = L.q_strides[x], a.ks[x] = L.kv_strides[x], a.os[x] = L.o_strides[x];
        a.dqs[x] = L.dq_strides[x], a.dks[x] = L.dkv_strides[x];
    }
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
    a.n_kv_heads = L.p.n_kv_heads;
    a.self_only = (L.p.flags & KSA_FLAG_SUMMARY_SELF_ONLY) ? 1 : 0;
    a.n_text = L.p.n_text;
    a.n_sum = (L.p.n_text / L.p.chunk_len) * L.p.n_summary;
    a.sum_tiles = (a.n_sum + KEYS_PER_WG - 1) / KEYS_PER_WG;
    a.aug_len = L.aug_len;
    a.scale = L.p.softmax_scale;
    a.scale_log2e = L.p.softmax_scale * 1.4426950408889634f;
    if (!L.workspace || L.workspace_bytes < ksa_prefill_bwd_workspace_size(L.p, L.aug_len)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    if (L.n_entries <= 0 || L.aug_len <= 0) return KSA_OK;
    if (L.p.head_dim != 128 && L.p.head_dim != 64) return KSA_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);

    const int64_t n_rows = (int64_t)L.p.batch * L.aug_len * L.p.n_q_heads;
    const int64_t delta_blocks = (n_rows * (L.p.head_dim / 8) + 255) / 256;
    const int text_tiles = (a.n_text + KEYS_PER_WG - 1) / KEYS_PER_WG;
    if (delta_blocks >= ((int64_t)1 << 31) || L.p.n_kv_heads > 65535 || L.p.batch > 65535) return KSA_ERR_UNSUPPORTED;
    const dim3 block(NW * 64), grid_dq(L.n_entries), grid_dkv(a.sum_tiles + text_tiles, L.p.n_kv_heads, L.p.batch);
    if (L.p.head_dim == 128) {
        hipLaunchKernelGGL(ksa_bwd_delta_kernel<128>, dim3((unsigned)delta_blocks), dim3(256), 0, st, a, n_rows);
        hipLaunchKernelGGL(ksa_bwd_dq_kernel<128>, grid_dq, block, 0, st, a);
        hipLaunchKernelGGL(ksa_bwd_dkv_kernel<128>, grid_dkv, block, 0, st, a);
    } else {
        hipLaunchKernelGGL(ksa_bwd_delta_kernel<64>, dim3((unsigned)delta_blocks), dim3(256), 0, st, a, n_rows);
        hipLaunchKernelGGL(ksa_bwd_dq_kernel<64>, grid_dq, block, 0, st, a);
        hipLaunchKernelGGL(ksa_bwd_dkv_kernel<64>, grid_dkv, block, 0, st, a);
    }
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}
