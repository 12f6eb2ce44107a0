// KSA prefill backward for gfx950: dQ, dK, dV of O = softmax(Q K^T scale + M_KSA) V for an upstream gradient
// G = dLoss/dO, from the saved log-sum-exp of the forward pass (the paper's block-sparse kernel serves training
// as well as prefill; it prints no backward formula, this is the derivative of the attention definition):
//   P_ij  = exp(scale q_i.k_j - lse_i) for visible pairs, else 0
//   dV_j  = sum_i P_ij G_i
//   dS_ij = P_ij (G_i.v_j - delta_i),  delta_i = G_i.O_i  (= sum_l P_il G_i.v_l)
//   dQ_i  = scale sum_j dS_ij k_j,     dK_j = scale sum_i dS_ij q_i
// Three kernels, no atomics, results independent of the launch order:
//   ksa_bwd_delta_kernel  delta_i and lse_i log2(e) per (batch, head, row), in compact row order, into the workspace;
//   ksa_bwd_dq_kernel     one workgroup per query tile of the forward schedule walks that tile's key runs;
//   ksa_bwd_dkv_kernel    one workgroup per 128-key tile of an index space walks the query rows that can see it
//                         (two runs, closed form from Eq. 3), for every query head of the KV head's group.
// Both main kernels recompute the scores with v_mfma_f32_32x32x16_bf16 and keep the result block in the layout
// whose registers are the B operand of the next product: dQ works on S^T (keys x queries, the forward kernel's
// layout, per-lane query statistics), dK/dV on S (queries x keys, per-lane key, per-register query statistics
// read from LDS).  The operand that has to be contracted over the tile's rows (K^T, Q^T, G^T) is read out of the
// same row-major LDS tile with the gfx950 transposing read (ds_read_b64_tr_b16).  The rows a wave owns for the
// whole kernel (Q and dO, or K and V) and its gradient accumulators live in accumulation registers and feed the
// MFMAs from there (inline assembly), which leaves the vector registers to the operands streamed through LDS.
// Tiles that every row sees whole skip the visibility test (Eq. 3); the others clip each score to its row's range.
#include <hip/hip_runtime.h>

#include <type_traits>

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
    // workspace: per-row statistics in COMPACT order, [B, Hq, nt_pad + ns_pad] fp32 each: position p < nt_pad is
    // text index p, position nt_pad + u is summary ordinal u; rows past the end of an index space hold zeros
    float *lse2c;                             // log-sum-exp times log2(e)
    float *dlc;                               // MINUS delta_i = -(dO_i . O_i): added to dP, or the start value of its MFMAs
    int32_t nt_pad, ns_pad;                   // rows per index space rounded up to 64
    __bf16 *dq, *dk, *dv;
    int64_t qs[3], ks[3], os[3], dqs[3], dks[3];   // {batch, row, head} strides in elements (os: o and g)
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t c, m, C, w;                       // chunk_len, n_summary, window_chunks, c + m
    int32_t c_shift, m_shift;
    int32_t group, n_q_heads, n_kv_heads, self_only, batch;
    int32_t stack, stack_shift;    // dQ kernel: query heads per workgroup of the forward schedule (1, 2 or 4), its log2
    int32_t n_text, n_sum;                    // rows per index space
    int32_t sum_tiles;                        // dK/dV grid: summary-space key tiles come first (the long ones)
    int64_t aug_len;
    float scale, scale_log2e;
};

// LDS tile: row-major [64][D] bf16; the 16-byte chunk index is XORed with a function of the row that spreads both
// the 16 rows of a plain 16-byte operand read and the 4 rows of a transposing read over different banks.
template <int D>
__device__ __forceinline__ int swz(int row) { return (((row & 3) << 2) | ((row >> 2) & 3)) & (D / 8 - 1); }

// Rows first .. first + 63 (clamped to `last`) of one index space, of two tensors that share the row map (K and V, or
// Q and G) -> two LDS tiles.  The bases point at (batch, head).
template <int D>
__device__ __forceinline__ void load_tile_pair(const BwdArgs &a, const __bf16 *base0, int64_t row_stride0,
                                               const __bf16 *base1, int64_t row_stride1, int space, int first, int last,
                                               unsigned char *tile0, unsigned char *tile1, int wave, int lane) {
    constexpr int CH = D / 8, RPI = 64 / CH, NI = RW / RPI;
    static_assert(RW % RPI == 0 && NI >= 1, "a wave's share of a tile is a whole number of load instructions");
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = RW * wave + RPI * i + lane / CH;
        const int pch = lane % CH;
        int idx = first + row;
        idx = idx < last ? idx : last;
        const int64_t arow = aug_row(a, space, idx);
        const int col = (pch ^ swz<D>(row)) << 3;
        lds_direct_load_16(base0 + arow * row_stride0 + col, tile0 + (RW * wave + RPI * i) * (D * 2));
        lds_direct_load_16(base1 + arow * row_stride1 + col, tile1 + (RW * wave + RPI * i) * (D * 2));
    }
}

// global -> LDS, 4 bytes per lane: the wave's 64 pieces land back to back (lane order) from the wave-uniform LDS
// address dst.  Inline assembly for the same reason as lds_direct_load_16().
__device__ __forceinline__ void lds_direct_load_4(const float *src, const unsigned char *dst) {
    const unsigned lds_addr = __builtin_amdgcn_readfirstlane((unsigned)(size_t)dst);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(src), "s"(lds_addr) : "memory");
}

// Byte addresses inside an LDS tile are written as (per-lane constant XOR small constant) + constant, so that one
// register per tile plus the instructions' immediate offsets cover every operand read.
struct LaneLds {
    int rows;   // plain operand read: row r, chunk (h ^ swizzle(r)); XOR (s << 5) selects k step s
    int cols;   // transposing read: row t_row, the 8 bytes at column t_col of chunk (t_col / 8 ^ swizzle(t_row))
};

template <int D>
__device__ __forceinline__ LaneLds lane_lds(int lane) {
    const int r = lane & 31, h = lane >> 5, grp = lane >> 4, li = lane & 15;
    // transposing read: lane (grp, li) supplies the address of tile row 4 (grp / 2) + li / 4, columns
    // 16 (grp % 2) + 4 (li % 4) .. + 3, and receives rows 4 (grp / 2) .. + 3 of column 16 (grp % 2) + li
    const int t_row = 4 * (grp >> 1) + (li >> 2), t_col = 16 * (grp & 1) + 4 * (li & 3);
    LaneLds L;
    L.rows = r * (D * 2) + ((h ^ swz<D>(r)) << 4);
    L.cols = t_row * (D * 2) + (((t_col >> 3) ^ swz<D>(t_row)) << 4) + ((t_col & 7) << 1);
    return L;
}

// A operand [32 tile rows of block rb] x [16 head-dim columns of k step s].  tile_rows = tile offset + LaneLds::rows
// (tile offsets are multiples of the tile size, so the XOR below only touches the lane part).
template <int D>
__device__ __forceinline__ bf16x8 read_rows(const unsigned char *lds, int tile_rows, int rb, int s) {
    return *reinterpret_cast<const bf16x8 *>(lds + ((tile_rows ^ (s << 5)) + rb * 32 * (D * 2)));
}

// A operand [32 head-dim columns of block db] x [16 tile rows from R0, a multiple of 16]: lane l gets column
// 32 db + l % 32 and the rows R0 + 4 h + (0..3), R0 + 8 + 4 h + (0..3), h = l / 32 -- the order in which a lane's
// registers of a 32x32 result block hold its rows, so that eight result registers are the matching B operand.
// tile_cols = tile offset + LaneLds::cols.  For a row R + t_row with R a multiple of 8 and t_row < 8 the swizzle is
// swizzle(t_row) ^ ((R >> 2) & 2), and the chunk of column block db is 4 db higher: both are XORs of bits 4..7.
template <int D>
__device__ __forceinline__ bf16x8 read_cols(const unsigned char *lds, int tile_cols, int R0, int db) {
    const int x0 = (((db * 4) ^ ((R0 >> 2) & 2)) & (D / 8 - 1)) << 4;
    const int x1 = (((db * 4) ^ (((R0 + 8) >> 2) & 2)) & (D / 8 - 1)) << 4;
    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lds + ((tile_cols ^ x0) + R0 * (D * 2))));
    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lds + ((tile_cols ^ x1) + (R0 + 8) * (D * 2))));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
}

// acc += A B for an accumulator that lives across the whole tile loop.  Inline assembly pins it to accumulation
// registers: left to the compiler, the 128 registers of such accumulators are copied to VGPRs and back around every
// tile.  The compiler does not know this is an MFMA and inserts none of the wait states an MFMA needs after a VALU
// write of its operands (the s_nop: the compiler packs the bf16 weights right in front of the statement, and without
// it the results are wrong) or before a VALU read of its result (see accumulators_settle()).
__device__ __forceinline__ void mfma_acc(f32x16 &acc, const bf16x8 &a_op, const bf16x8 &b_op) {
    asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a_op), "v"(b_op));
}

// acc (+)= A B for a short-lived score block whose B operand is held in accumulation registers for the whole kernel
// (the wave's own Q / dO or K / V rows): MFMA reads them there directly, and the vector registers stay free for the
// operands streamed through LDS.  FIRST starts the block from zero.  Before VALU code reads acc the results have to
// reach the register file: scores_settle().
template <bool FIRST>
__device__ __forceinline__ void mfma_score(f32x16 &acc, const bf16x8 &a_op, const bf16x8 &b_resident) {
    if constexpr (FIRST)
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(acc) : "v"(a_op), "a"(b_resident));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a_op), "a"(b_resident));
}

// The last mfma_acc() results reach the register file (16 passes of 4 cycles) before anything reads them.
__device__ __forceinline__ void accumulators_settle() {
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
}

#define KSA_FENCE() __builtin_amdgcn_sched_barrier(0)

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

// ---- per-row statistics: delta_i = G_i . O_i and lse_i log2(e), in compact order ------------------------------------
template <int D>
__global__ __launch_bounds__(256) void ksa_bwd_delta_kernel(const BwdArgs a, int64_t n_slots /* B * Hq * (nt_pad + ns_pad) */) {
    constexpr int CH = D / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t slot = idx / CH;
    const int piece = (int)(idx % CH);
    const bool in_grid = slot < n_slots;
    if (!in_grid) slot = n_slots - 1;
    const int sp = a.nt_pad + a.ns_pad;
    const int pos = (int)(slot % sp);
    const int64_t bh = slot / sp;
    const int hq = (int)(bh % a.n_q_heads);
    const int64_t b = bh / a.n_q_heads;
    const int space = pos < a.nt_pad ? KSA_SPACE_TEXT : KSA_SPACE_SUMMARY;
    const int ci = space == KSA_SPACE_TEXT ? pos : pos - a.nt_pad;
    const bool live = ci < (space == KSA_SPACE_TEXT ? a.n_text : a.n_sum);   // wave-uniform per group of CH lanes
    float s = 0.f, l2 = 0.f;
    if (live) {
        const int64_t aq = aug_row(a, space, ci);
        const int64_t off = b * a.os[0] + aq * a.os[1] + hq * a.os[2] + piece * 8;
        const bf16x8 o8 = *reinterpret_cast<const bf16x8 *>(a.o + off);
        const bf16x8 g8 = *reinterpret_cast<const bf16x8 *>(a.g + off);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += (float)o8[e] * (float)g8[e];
        l2 = a.lse[(b * a.n_q_heads + hq) * a.aug_len + aq] * 1.4426950408889634f;
    }
#pragma unroll
    for (int d = CH / 2; d > 0; d >>= 1) s += __shfl_xor(s, d);
    if (in_grid && piece == 0) {
        a.dlc[slot] = -s;
        a.lse2c[slot] = l2;
    }
}

// ---- dQ -----------------------------------------------------------------------------------------------------
// POW2: chunk_len and n_summary are powers of two, so that the row maps are shifts and the bookkeeping of the next
// tile request is short straight-line code that can sit between the MFMAs of the tile in work.  Otherwise the same
// statements run in one block after the barrier.
template <int D, bool POW2>
__global__ __launch_bounds__(NW * 64) void ksa_bwd_dq_kernel(const BwdArgs a) {
    constexpr int KS = D / 16, DB = D / 32, BYTES = BN * D * 2;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[4 * BYTES];   // two buffers of a K and a V tile

    const KsaWgEntry ent = a.entries[blockIdx.x];
    if (ent.item < 0) return;
    // The item's few words are copied into scalar registers here: read through a reference inside the tile loop they
    // would be fetched from memory again after every tile request (the requests are opaque memory operations to the
    // compiler), each fetch followed by a wait for ALL outstanding loads, the tile in flight included.
    const KsaWorkItem *item_p = a.items + ent.item;
    const int n_seg = item_p->n_seg;
    int seg_space[KSA_MAX_SEGMENTS], seg_begin[KSA_MAX_SEGMENTS], seg_end[KSA_MAX_SEGMENTS];
    int seg_full_lo[KSA_MAX_SEGMENTS], seg_full_hi[KSA_MAX_SEGMENTS];
    static_assert(KSA_MAX_SEGMENTS == 2, "segment fields are selected with one compare");
#pragma unroll
    for (int x = 0; x < KSA_MAX_SEGMENTS; ++x) {
        seg_space[x] = item_p->seg[x].space, seg_begin[x] = item_p->seg[x].begin, seg_end[x] = item_p->seg[x].end;
        seg_full_lo[x] = item_p->seg[x].full_lo, seg_full_hi[x] = item_p->seg[x].full_hi;
    }
#define KSA_SEG(field, sg) ((sg) == 0 ? field[0] : field[1])
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // as in the forward kernel: wave w takes query head w % stack and row block w / stack of the query tile
    const int b = ent.batch, hq = ent.q_head + (wave & (a.stack - 1)), hkv = ent.q_head / a.group;
    const int wrow = wave >> a.stack_shift;
    const int r = lane & 31, h = lane >> 5;
    const LaneLds ll = lane_lds<D>(lane);
    const int q_space = item_p->q_space, q_begin = item_p->q_begin, q_end = item_p->q_begin + item_p->q_count;

    int q_aug[QB];
    bool q_valid[QB];
    int idc[QB];
    float lse2[QB], dl[QB];
    bf16x8 qreg[QB][KS], greg[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int idx = q_begin + (wrow * QB + qb) * 32 + r;
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
        const int64_t stat = ((int64_t)b * a.n_q_heads + hq) * (a.nt_pad + a.ns_pad) +
                             (q_space == KSA_SPACE_TEXT ? idc[qb] : a.nt_pad + idc[qb]);
        lse2[qb] = a.lse2c[stat];
        dl[qb] = a.dlc[stat];
    }
    f32x16 dqacc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) zero(dqacc[qb][db]);

    const __bf16 *kbase = a.k + b * a.ks[0] + hkv * a.ks[2];
    const __bf16 *vbase = a.v + b * a.ks[0] + hkv * a.ks[2];
    const float sl = a.scale_log2e;

    // The key tiles of all runs form one sequence; tile t sits in LDS buffer t % 2, and the loads of tile t + 1 go out
    // during the step of tile t, after the barrier that publishes tile t.
    int n_tiles = 0;
#pragma unroll
    for (int x = 0; x < KSA_MAX_SEGMENTS; ++x)
        if (x < n_seg && seg_end[x] > seg_begin[x]) n_tiles += (seg_end[x] - seg_begin[x] + BN - 1) / BN;

    // ---- the request of a tile, in two parts (as in the dK/dV kernel) ------------------------------------------
    // prepare: advances the sequence and works out where the tile's rows are; issue: the wave's 2 NI loads.  Once
    // the sequence is exhausted prepare stays on the last tile, which is then fetched again into the buffer nobody
    // reads: every step issues the same loads, and the tile loop carries no branch.
    constexpr int CH = D / 8, RPI = 64 / CH, NI = RW / RPI;
    static_assert(RW % RPI == 0 && NI >= 1, "a wave's share of a tile is a whole number of load instructions");
    const unsigned kv_row_bytes = (unsigned)a.ks[1] * 2u;
    // the next tile of the sequence (an empty first run is skipped; the host schedule has no item without tiles)
    const int second_run = (n_seg > 1 && seg_end[1] > seg_begin[1]) ? 1 : 0;
    int sq_seg = (n_seg > 1 && seg_end[0] <= seg_begin[0]) ? 1 : 0;
    int sq_kt = KSA_SEG(seg_begin, sq_seg);
    struct Request {
        const __bf16 *k_base, *v_base;   // row `first` of the tile (scalar)
        unsigned off[NI];                // per lane: byte offset of the 16 bytes it fetches, per load instruction
        int seg, first;
        bool full;                       // every row of the query tile sees every key of the tile
    } rq;
    rq.k_base = kbase, rq.v_base = vbase, rq.seg = 0, rq.first = 0, rq.full = false;
#pragma unroll
    for (int i = 0; i < NI; ++i) rq.off[i] = 0;
    // Both shift counts in one scalar register, byte `sp` that of index space sp (a shift takes its count modulo 32).
    // Opaque to the compiler: a select between two kernel arguments is otherwise compiled into a scalar load of the
    // selected argument inside the tile loop, and the wait for it drains every LDS operand read in flight.
    unsigned shifts = ((unsigned)a.c_shift & 31u) | (((unsigned)a.m_shift & 31u) << 8);
    asm volatile("" : "+s"(shifts));
    auto chunk_of = [&](int sp, int idx) {
        if constexpr (POW2) return idx >> (shifts >> (sp * 8));
        return idx / (sp == KSA_SPACE_TEXT ? a.c : a.m);
    };
    auto prepare_tile = [&]() {   // scalar part
        const int sg = sq_seg, first = sq_kt;
        const int space = KSA_SEG(seg_space, sg);
        {   // advance, unless this is the last tile
            const int nk = first + BN;
            const int run_done = nk >= KSA_SEG(seg_end, sg) ? 1 : 0;
            const int more = (run_done ^ 1) | ((sg == 0 ? 1 : 0) & second_run);   // bitwise: no short-circuit branches
            const int ns = sg + run_done, nkt = run_done ? seg_begin[1] : nk;
            sq_seg = more ? ns : sq_seg, sq_kt = more ? nkt : sq_kt;
        }
        const int per = space == KSA_SPACE_TEXT ? a.m : a.c;   // rows of the other kind per chunk
        const int add = space == KSA_SPACE_TEXT ? 0 : a.c;
        const int64_t arow = (int64_t)first + (int64_t)chunk_of(space, first) * per + add;
        rq.k_base = kbase + arow * a.ks[1], rq.v_base = vbase + arow * a.ks[1];
        rq.seg = sg, rq.first = first;
        rq.full = first >= KSA_SEG(seg_full_lo, sg) && first + BN <= KSA_SEG(seg_full_hi, sg);
    };
    auto prepare_row = [&](int i) {   // per-lane part of load instruction i
        const int sg = rq.seg, first = rq.first;
        const int space = KSA_SEG(seg_space, sg);
        const int row = RW * wave + RPI * i + lane / CH;
        int idx = first + row;
        const int last = KSA_SEG(seg_end, sg) - 1;
        idx = idx < last ? idx : last;
        const int per = space == KSA_SPACE_TEXT ? a.m : a.c;
        // augmented row of idx minus that of `first`: the index distance plus the other kind's rows in between
        const int d_rows = (idx - first) + (chunk_of(space, idx) - chunk_of(space, first)) * per;
        rq.off[i] = (unsigned)d_rows * kv_row_bytes + (unsigned)(((lane % CH) ^ swz<D>(row)) << 4);
    };
    auto prepare_all = [&]() {
        prepare_tile();
#pragma unroll
        for (int i = 0; i < NI; ++i) prepare_row(i);
    };
    const unsigned lds_tiles = (unsigned)(size_t)lds;
    auto issue_load = [&](int buffer, int x) {   // load instruction x of the prepared tile: K rows, V rows alternating
        const int i = x / 2;
        const unsigned dst = lds_tiles + (unsigned)buffer * 2 * BYTES + (x % 2) * BYTES + (RW * wave + RPI * i) * (D * 2);
        lds_direct_load_16_s(x % 2 == 0 ? rq.k_base : rq.v_base, rq.off[i], __builtin_amdgcn_readfirstlane(dst));
    };

    // the wave's own rows and statistics have arrived before the first tile request: from here on only tile requests
    // are outstanding, and the waits in the loop count those alone
    __builtin_amdgcn_s_waitcnt(0x0F70);
    int fly_seg = 0, fly_kt = 0;   // the tile whose loads went out last: the next one to work on
    bool fly_full = false;
    if (n_tiles > 0) {   // (the host schedule has no item without tiles; nothing is requested for one)
        prepare_all();
        fly_seg = rq.seg, fly_kt = rq.first, fly_full = rq.full;
#pragma unroll
        for (int x = 0; x < 2 * NI; ++x) issue_load(0, x);
        prepare_all();
    }
    int buf = 0;
    int elo[QB], espan[QB], range_seg = -1;

    // One tile: publish it, request the next one, compute.  The tile's work is a stream of MFMAs -- scores of key
    // block 0 (S and dO V^T of both query blocks of the wave, k step by k step: every operand read from LDS feeds
    // QB MFMAs), scores of key block 1, dQ products of block 0, of block 1 -- and one wave per SIMD has nobody else
    // to fill the matrix pipe while its other instructions issue, so everything else is dealt into that stream by
    // hand, one small piece behind each MFMA: the loads of the next request behind the first scores, the weights
    // of block 0 behind the scores of block 1, the weights of block 1 behind the dQ products (of block 0, and of
    // the first half of block 1, which only needs the first half of the weights), the arithmetic of the request after
    // next behind the last dQ products.  Source order is the intended issue order, pinned with scheduling fences; LDS
    // operands are read AHEAD operand steps before the MFMAs that consume them.  MASKED tiles clip every score to
    // its row's visible range; tiles the schedule marks as seen whole by every row of the query tile do not: the two
    // variants are separate instantiations walked in stretches.
    auto step = [&](auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();   // the tile in work is complete in buffer buf; everybody is done with the other buffer
        const int cur_seg = fly_seg, cur_kt = fly_kt;
        fly_seg = rq.seg, fly_kt = rq.first, fly_full = rq.full;   // the tile whose loads go out during this step
        const int k_rows = buf * 2 * BYTES + ll.rows, v_rows = k_rows + BYTES, k_cols = buf * 2 * BYTES + ll.cols;
        const int req_buf = buf ^ 1;
        constexpr int NU = 2 * KS + 4 * DB;   // operand steps: K and V rows per k step, then K columns per dQ product
        constexpr int AHEAD = 3;
        bf16x8 op_k[NU], op_v[2 * KS];
        auto read_ops = [&](int u) {
            if (u < 2 * KS) {
                op_k[u] = read_rows<D>(lds, k_rows, u / KS, u % KS), op_v[u] = read_rows<D>(lds, v_rows, u / KS, u % KS);
            } else {
                const int kb = (u - 2 * KS) / (2 * DB), j = (u - 2 * KS) % (2 * DB);
                op_k[u] = read_cols<D>(lds, k_cols, kb * 32 + (j / DB) * 16, j % DB);
            }
        };
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) read_ops(u);
        if (range_seg != cur_seg) {
            range_seg = cur_seg;
            const int space = KSA_SEG(seg_space, cur_seg), run_begin = KSA_SEG(seg_begin, cur_seg), run_end = KSA_SEG(seg_end, cur_seg);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                int lo, hi;
                visible_range(a, q_space, idc[qb], space, lo, hi);
                elo[qb] = lo > run_begin ? lo : run_begin;
                const int ehi = hi < run_end ? hi : run_end;
                espan[qb] = ehi > elo[qb] ? ehi - elo[qb] : 0;
                if (!q_valid[qb]) elo[qb] = 0x7fffffff, espan[qb] = 0;
            }
        }
        if constexpr (!POW2) {
#pragma unroll
            for (int x = 0; x < 2 * NI; ++x) issue_load(req_buf, x);
            prepare_all();
        }
        KSA_FENCE();

        f32x16 sacc[2][QB], gacc[2][QB];
        bf16x8 pb[2][QB][2];    // dS^T in the B-operand layout: lane = query, eight registers = eight keys
        float df[2][QB][16];
        // weight of score register g (one key of the lane's query) of key block kb, query block qb; the bf16 pair
        // is packed when its second member is done
        auto weight = [&](int kb, int qb, int g) {
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][g], sl, -lse2[qb]));
            // one subtraction and one unsigned compare per score: elo <= key < elo + espan
            if constexpr (MASKED) p = (unsigned)(cur_kt + kb * 32 + 4 * h - elo[qb] + 8 * (g / 4) + (g % 4)) < (unsigned)espan[qb] ? p : 0.f;
            df[kb][qb][g] = p * (gacc[kb][qb][g] + dl[qb]);   // dl holds minus delta
            if (g % 2 == 1)
                pb[kb][qb][g / 8][g % 8 - 1] = (__bf16)df[kb][qb][g - 1], pb[kb][qb][g / 8][g % 8] = (__bf16)df[kb][qb][g];
        };
        // element number e (0 .. 8 QB - 1) of a half (registers 8 hf .. 8 hf + 7) of block kb's weights: pairs of
        // registers, the query blocks alternating
        auto weight_of_half = [&](int kb, int hf, int e) {
            const int pair = e / (2 * QB), qb = (e / 2) % QB;
            weight(kb, qb, 8 * hf + 2 * pair + e % 2);
        };

        // scores of key block kb: slot = MFMA number within the phase
        auto score_phase = [&](auto kb_tag) {
            constexpr int kb = decltype(kb_tag)::value;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int u = kb * KS + s;
                if (u + AHEAD < NU) read_ops(u + AHEAD);
#pragma unroll
                for (int y = 0; y < 2 * QB; ++y) {
                    const int slot = s * 2 * QB + y, qb = y / 2;
                    f32x16 &acc = y % 2 == 0 ? sacc[kb][qb] : gacc[kb][qb];
                    const bf16x8 &a_op = y % 2 == 0 ? op_k[u] : op_v[u];
                    const bf16x8 &b_op = y % 2 == 0 ? qreg[qb][s] : greg[qb][s];
                    if (s == 0)
                        mfma_score<true>(acc, a_op, b_op);
                    else
                        mfma_score<false>(acc, a_op, b_op);
                    if constexpr (POW2 && kb == 0) {
                        if (slot < 2 * NI) issue_load(req_buf, slot);
                    }
                    if constexpr (kb == 1) {
                        // The scores of block 0 were completed by the MFMAs before this phase.  The compiler does not
                        // know that the statements above are MFMAs: the empty statement keeps the code that reads
                        // those scores behind the first two MFMAs of this phase, which take longer to issue than the
                        // last results need to land.
                        constexpr int PER = 16 * QB / (KS * 2 * QB) > 0 ? 16 * QB / (KS * 2 * QB) : 1;   // weights per slot
                        if (slot == 1) {
#pragma unroll
                            for (int qq = 0; qq < QB; ++qq) asm volatile("" : "+v"(sacc[0][qq]), "+v"(gacc[0][qq]));
#pragma unroll
                            for (int z = 0; z < PER; ++z) {
                                const int e = z;
                                weight_of_half(0, e / (8 * QB), e % (8 * QB));
                            }
                        }
                        if (slot >= 1) {
#pragma unroll
                            for (int z = 0; z < PER; ++z) {
                                const int e = slot * PER + z;
                                if (e < 16 * QB) weight_of_half(0, e / (8 * QB), e % (8 * QB));
                            }
                        }
                    }
                    KSA_FENCE();
                }
            }
        };
        // dQ^T += K^T dS^T of key block kb: operand step j = (16-key group j / DB, 32-column block j % DB)
        auto dq_phase = [&](auto kb_tag) {
            constexpr int kb = decltype(kb_tag)::value;
#pragma unroll
            for (int j = 0; j < 2 * DB; ++j) {
                const int u = 2 * KS + kb * 2 * DB + j;
                if (u + AHEAD < NU) read_ops(u + AHEAD);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int slot = j * QB + qb;
                    mfma_acc(dqacc[qb][j % DB], op_k[u], pb[kb][qb][j / DB]);
                    if constexpr (kb == 0) {
                        // first half of block 1's weights, one per MFMA (see above for the empty statement)
                        if (slot == 1) {
#pragma unroll
                            for (int qq = 0; qq < QB; ++qq) asm volatile("" : "+v"(sacc[1][qq]), "+v"(gacc[1][qq]));
                            weight_of_half(1, 0, 0);
                        }
                        if (slot >= 1 && slot < 8 * QB) weight_of_half(1, 0, slot);
                        if (slot == 2 * DB * QB - 1) {   // fewer MFMAs than weights: the rest behind the last one
#pragma unroll
                            for (int e = 2 * DB * QB; e < 8 * QB; ++e) weight_of_half(1, 0, e);
                        }
                    } else {
                        // second half of block 1's weights behind the products of the first half, two per MFMA; then
                        // the arithmetic of the request after next
                        constexpr int HALF = DB * QB;   // MFMAs of the first 16-key group
                        if (slot < HALF) {
#pragma unroll
                            for (int e = slot * (8 * QB / HALF); e < (slot + 1) * (8 * QB / HALF); ++e) weight_of_half(1, 1, e);
                        }
                        if constexpr (POW2) {
                            if (slot == HALF) prepare_tile();
                            if (slot > HALF && slot - HALF - 1 < NI) prepare_row(slot - HALF - 1);
                        }
                    }
                    KSA_FENCE();
                }
            }
        };
        score_phase(std::integral_constant<int, 0>{});
        score_phase(std::integral_constant<int, 1>{});
        dq_phase(std::integral_constant<int, 0>{});
        dq_phase(std::integral_constant<int, 1>{});
        buf ^= 1;
    };
    int left = n_tiles;
    while (left > 0) {
        if (fly_full) {
            do step(std::false_type{}), --left;
            while (left > 0 && fly_full);
        } else {
            do step(std::true_type{}), --left;
            while (left > 0 && !fly_full);
        }
    }
#undef KSA_SEG

    // nothing of this workgroup is in flight any more when it leaves (the last request fetched a tile nobody reads)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    accumulators_settle();
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
// POW2: chunk_len and n_summary are powers of two, so that the row maps are shifts and the bookkeeping of the next
// tile request is short straight-line code that can sit between the MFMAs of the tile in work.  Otherwise the same
// statements run in one block after the barrier.
template <int D, bool POW2>
__global__ __launch_bounds__(NW * 64) void ksa_bwd_dkv_kernel(const BwdArgs a) {
    constexpr int KS = D / 16, DB = D / 32, BYTES = BN * D * 2;
    // tiles in flight + 1: the query tiles of a long run stream from HBM (their total is far beyond the caches), and
    // the key tiles of a head advance in step, so every step sees the full memory latency unless the request runs
    // several steps ahead
    constexpr int STAGES = 4;
    // STAGES buffers of a Q and a G tile with the tiles' row statistics
    __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * 2 * BYTES];
    __shared__ __attribute__((aligned(256))) float st_lse[STAGES][BN], st_dl[STAGES][BN];
    __shared__ __attribute__((aligned(16))) int st_lo[STAGES][BN], st_span[STAGES][BN];   // visible keys: [lo, lo + span)

    // Workgroup index -> (key tile, batch, KV head), the head running fastest: consecutive workgroup ids go to the
    // XCDs round-robin, so with 8 (batch, KV head) pairs all key tiles of a head share one L2, and they walk the same
    // query rows at about the same time (see the loop order below).  Summary-space tiles come first, oldest chunks
    // first: their runs of query rows are the long ones.
    const int n_bh = a.n_kv_heads * a.batch;
    const int bh = blockIdx.x % n_bh;
    const int hkv = bh % a.n_kv_heads, b = bh / a.n_kv_heads;
    int t = blockIdx.x / n_bh, space = KSA_SPACE_SUMMARY;
    if (t >= a.sum_tiles) t -= a.sum_tiles, space = KSA_SPACE_TEXT;
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
    // jl + C + 1 on and by the summary rows of their own chunks from k0 on.  Run x is in index space x.
    static_assert(KSA_SPACE_TEXT == 0 && KSA_SPACE_SUMMARY == 1, "a run's number is its index space");
    int run_begin[2], run_end[2];
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

    // The query tiles of both runs and of all query heads of the group form one sequence: per run the aligned 64-row
    // blocks of the index space that overlap it, from the LAST one downwards (every key tile of a head then meets the
    // same query tiles in the same order, whatever its own first row is), the heads of the group innermost.  Rows
    // of a block outside the run are masked through their visible range.  Tile t of the sequence sits in LDS stage
    // t % STAGES with its row statistics.
    int run_first_blk[2], run_tiles[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        run_first_blk[x] = run_begin[x] / BN;
        run_tiles[x] = run_end[x] > run_begin[x] ? (run_end[x] - 1) / BN - run_first_blk[x] + 1 : 0;
    }
    const int n_tiles = (run_tiles[0] + run_tiles[1]) * a.group;   // > 0: a key is seen by its own row at least
    // Blocks [full_lo_blk, full_hi_blk) of a run (counted from the run's first block) are seen whole: no row of such
    // a block lies outside the run, and every row sees every key of the workgroup.  Visible ranges are monotone in
    // the row index (Eq. 3: both ends of a row's range never move backwards from one row to the next), so these
    // blocks are consecutive: the first block whose first row's range ends at or behind the last key, up to the last
    // block whose last row's range starts at or before the first key.  Two bisections per run, once per workgroup;
    // the tile loop then only compares block numbers.
    int full_lo_blk[2], full_hi_blk[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int w_lo = run_begin[x] % BN == 0 ? 0 : 1;                       // blocks without rows outside the run
        const int w_hi = run_tiles[x] - (run_end[x] % BN == 0 ? 0 : 1);
        int lo_b = w_lo, hi_b = w_hi > w_lo ? w_hi : w_lo;   // first block in [w_lo, w_hi) whose first row sees key k1 - 1
        while (lo_b < hi_b) {
            const int mid = (lo_b + hi_b) >> 1;
            int rlo, rhi;
            visible_range(a, x, (run_first_blk[x] + mid) * BN, space, rlo, rhi);
            if (rhi >= k1) hi_b = mid; else lo_b = mid + 1;
        }
        full_lo_blk[x] = lo_b;
        lo_b = w_lo, hi_b = w_hi > w_lo ? w_hi : w_lo;        // first block in [w_lo, w_hi) whose last row no longer sees key k0
        while (lo_b < hi_b) {
            const int mid = (lo_b + hi_b) >> 1;
            int rlo, rhi;
            visible_range(a, x, (run_first_blk[x] + mid) * BN + BN - 1, space, rlo, rhi);
            if (rlo > k0) hi_b = mid; else lo_b = mid + 1;
        }
        full_hi_blk[x] = lo_b;
    }
#define KSA_RUN(field, x) ((x) == 0 ? field[0] : field[1])

    // ---- the request of a tile, in two parts ----------------------------------------------------------------
    // prepare: advances the sequence and works out where the tile's rows are (scalar tile data, one offset per lane
    //          and load instruction); issue: the LOADS_PER_TILE global -> LDS loads of a wave.  The two are separate
    //          so that each can be dealt into the MFMA stream of the tile in work: the loads go out one behind each
    //          of the first MFMAs of a step (a load instruction occupies the issue port for tens of cycles), the
    //          arithmetic of the following request runs behind the last ones.  When the sequence is exhausted,
    //          prepare leaves the last tile in place and the loads fetch it again into a stage nobody reads: every
    //          step then issues the same number of loads, which is what the counted waits rely on.
    constexpr int CH = D / 8, RPI = 64 / CH, NI = RW / RPI;
    constexpr int LOADS_PER_TILE = 2 * NI + 2;
    static_assert(RW % RPI == 0 && NI >= 1, "a wave's share of a tile is a whole number of load instructions");
    static_assert(LOADS_PER_TILE <= 2 * KS, "one load behind each MFMA of the first score block");
    const int stats_stride = a.nt_pad + a.ns_pad;
    const unsigned q_row_bytes = (unsigned)a.qs[1] * 2u, g_row_bytes = (unsigned)a.os[1] * 2u;
    // bases of the KV head's first query head, and strides as unsigned 32-bit element counts
    const __bf16 *q_wg = a.q + b * a.qs[0] + (int64_t)hkv * a.group * a.qs[2];
    const __bf16 *g_wg = a.g + b * a.os[0] + (int64_t)hkv * a.group * a.os[2];
    const float *lse_wg = a.lse2c + ((int64_t)b * a.n_q_heads + hkv * a.group) * stats_stride;
    const float *dl_wg = a.dlc + ((int64_t)b * a.n_q_heads + hkv * a.group) * stats_stride;
    const unsigned q_row_elems = (unsigned)a.qs[1], g_row_elems = (unsigned)a.os[1];
    const unsigned q_head_elems = (unsigned)a.qs[2], g_head_elems = (unsigned)a.os[2];
    // the next tile of the sequence; stays on the last tile once the sequence is exhausted
    int sq_run = run_tiles[0] > 0 ? 0 : 1, sq_ti = 0, sq_hj = 0;
    struct Request {
        const __bf16 *q_base, *g_base;   // row `first` of the tile (scalar)
        const float *lse_p, *dl_p;       // statistics of row `first` (scalar)
        unsigned q_off[NI], g_off[NI];   // per lane: byte offset of the 16 bytes it fetches, per load instruction
        int q_space, first;
        bool full;                       // every row of the tile sees every key of the workgroup
    } rq;
    rq.q_base = a.q, rq.g_base = a.g, rq.lse_p = a.lse2c, rq.dl_p = a.dlc, rq.q_space = 0, rq.first = 0, rq.full = false;
#pragma unroll
    for (int i = 0; i < NI; ++i) rq.q_off[i] = rq.g_off[i] = 0;
    // compact index -> chunk number and augmented row, in index space sp (scalar sp)
    // Both shift counts in one scalar register, byte `sp` that of index space sp (a shift takes its count modulo 32).
    // Opaque to the compiler: a select between two kernel arguments is otherwise compiled into a scalar load of the
    // selected argument inside the tile loop, and the wait for it drains every LDS operand read in flight.
    unsigned shifts = ((unsigned)a.c_shift & 31u) | (((unsigned)a.m_shift & 31u) << 8);
    asm volatile("" : "+s"(shifts));
    auto chunk_of = [&](int sp, int idx) {
        if constexpr (POW2) return idx >> (shifts >> (sp * 8));
        return idx / (sp == KSA_SPACE_TEXT ? a.c : a.m);
    };
    auto prepare_tile = [&]() {   // scalar part
        const int run = sq_run, cur_ti = sq_ti, cur_hj = sq_hj;
        const int first = (KSA_RUN(run_first_blk, run) + KSA_RUN(run_tiles, run) - 1 - sq_ti) * BN;
        {   // advance, unless this is the last tile
            int hj = sq_hj + 1, ti = sq_ti, rn = sq_run;
            const bool wrap = hj == a.group;
            hj = wrap ? 0 : hj, ti = wrap ? ti + 1 : ti;
            const bool run_done = ti >= KSA_RUN(run_tiles, rn);
            rn = run_done ? rn + 1 : rn, ti = run_done ? 0 : ti;
            const bool more = rn < 2 && (rn == 0 || run_tiles[1] > 0);
            sq_hj = more ? hj : sq_hj, sq_ti = more ? ti : sq_ti, sq_run = more ? rn : sq_run;
        }
        const int per = run == KSA_SPACE_TEXT ? a.m : a.c;   // rows of the other kind per chunk
        const int add = run == KSA_SPACE_TEXT ? 0 : a.c;
        // (unsigned 32 x 32 -> 64 bit products from per-workgroup bases: a handful of scalar instructions; the launch
        // checks that the strides fit)
        const unsigned arow = (unsigned)(first + chunk_of(run, first) * per + add);
        rq.q_base = q_wg + ((uint64_t)arow * q_row_elems + (uint64_t)(unsigned)cur_hj * q_head_elems);
        rq.g_base = g_wg + ((uint64_t)arow * g_row_elems + (uint64_t)(unsigned)cur_hj * g_head_elems);
        const uint64_t at = (uint64_t)(unsigned)cur_hj * (unsigned)stats_stride + (unsigned)((run == KSA_SPACE_TEXT ? 0 : a.nt_pad) + first);
        rq.lse_p = lse_wg + at, rq.dl_p = dl_wg + at;
        rq.q_space = run, rq.first = first;
        const int bi = KSA_RUN(run_tiles, run) - 1 - cur_ti;
        rq.full = bi >= KSA_RUN(full_lo_blk, run) && bi < KSA_RUN(full_hi_blk, run);
    };
    auto prepare_row = [&](int i) {   // per-lane part of load instruction i
        const int run = rq.q_space, first = rq.first;
        const int row = RW * wave + RPI * i + lane / CH;
        int idx = first + row;
        const int last = KSA_RUN(run_end, run) - 1;
        idx = idx < last ? idx : last;
        const int per = run == KSA_SPACE_TEXT ? a.m : a.c;
        // augmented row of idx minus that of `first`: the index distance plus the other kind's rows in between
        const int d_rows = (idx - first) + (chunk_of(run, idx) - chunk_of(run, first)) * per;
        const unsigned col = (unsigned)(((lane % CH) ^ swz<D>(row)) << 4);
        rq.q_off[i] = (unsigned)d_rows * q_row_bytes + col;
        rq.g_off[i] = (unsigned)d_rows * g_row_bytes + col;
    };
    auto prepare_all = [&]() {
        prepare_tile();
#pragma unroll
        for (int i = 0; i < NI; ++i) prepare_row(i);
    };
    const unsigned lds_tiles = (unsigned)(size_t)lds, lds_lse = (unsigned)(size_t)&st_lse[0][0], lds_dl = (unsigned)(size_t)&st_dl[0][0];
    // load instruction x of the prepared tile into `stage`: x < 2 NI the tile rows, then the two statistics rows
    // (lse and delta of the 64 rows, one 4-byte piece per lane; all waves fetch the same 256 bytes, which keeps the
    // per-wave load count uniform and costs nothing)
    auto issue_load = [&](int stage, int x) {
        if (x < 2 * NI) {
            const int i = x / 2;
            const unsigned dst = lds_tiles + (unsigned)stage * 2 * BYTES + (x % 2) * BYTES + (RW * wave + RPI * i) * (D * 2);
            if (x % 2 == 0)
                lds_direct_load_16_s(rq.q_base, rq.q_off[i], __builtin_amdgcn_readfirstlane(dst));
            else
                lds_direct_load_16_s(rq.g_base, rq.g_off[i], __builtin_amdgcn_readfirstlane(dst));
        } else {
            const float *src = (x == 2 * NI ? rq.lse_p : rq.dl_p) + lane;
            lds_direct_load_4(src, reinterpret_cast<const unsigned char *>((size_t)((x == 2 * NI ? lds_lse : lds_dl) + (unsigned)stage * BN * 4)));
        }
    };
    unsigned full_mask = 0;   // bit `stage`: every row of the tile in that stage sees every key of the workgroup
    // what goes with the loads of a tile: the full flag of its stage and, unless the tile is seen whole, the visible
    // key range of each row (empty for rows of the block outside the run)
    auto issue_flags = [&](int stage) {
        full_mask = (full_mask & ~(1u << stage)) | ((rq.full ? 1u : 0u) << stage);
        if (!rq.full && tid < BN) {
            const int qi = rq.first + tid, run = rq.q_space;
            int lo = 0x7fffffff, hi = 0;
            if (qi >= KSA_RUN(run_begin, run) && qi < KSA_RUN(run_end, run)) visible_range(a, run, qi, space, lo, hi);
            st_lo[stage][tid] = lo, st_span[stage][tid] = hi > lo ? hi - lo : 0;
        }
    };

    // The wave's own K and V rows have arrived before the first tile request: from here on only tile requests are
    // outstanding, which is what the counted waits of the loop assume.  (Left to the compiler, the wait for these rows
    // sits in front of their first use inside the loop, where it also waits for every tile in flight.)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // tiles 0 .. STAGES - 2 are requested up front; the request of tile STAGES - 1 is prepared for step 0
    if (n_tiles > 0) {   // (a valid key is seen by its own row at least; nothing is requested otherwise)
#pragma unroll
        for (int st = 0; st < STAGES - 1; ++st) {
            prepare_all();
            issue_flags(st);
#pragma unroll
            for (int x = 0; x < LOADS_PER_TILE; ++x) issue_load(st, x);
        }
        prepare_all();
    }
    int buf = 0;   // stage of the tile in work

    // One tile: publish it, request the tile STAGES - 1 ahead, compute.  The tile's work is a stream of 4 KS pairs of
    // MFMAs -- scores of row block 0, scores of row block 1, gradient products of block 0, of block 1 -- and one wave
    // per SIMD has nobody else to fill the matrix pipe while its other instructions issue, so everything else is
    // dealt into that stream by hand: the loads of the next request behind the MFMAs of the first block's scores, the
    // weights of block 0 (one pair of query rows per MFMA) behind the scores of block 1, those of block 1 behind the
    // gradient products of block 0, the arithmetic of the request after next behind the gradient products of block 1.
    // An MFMA executes for 8 passes while the wave goes on issuing, so the pieces between two MFMAs have to stay
    // short.  Source order is the intended issue order, pinned with scheduling fences; LDS operands are read AHEAD
    // pairs before the MFMAs that consume them.  A tile all of whose rows see all of the workgroup's keys (nearly
    // every tile of a summary key) skips the visibility test: the two variants are separate instantiations walked in
    // stretches.
    auto step = [&](auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        // the tile in work is complete when at most the loads of the STAGES - 2 younger ones are outstanding
        constexpr int YOUNGER = (STAGES - 2) * LOADS_PER_TILE;
        static_assert(YOUNGER < 64, "vmcnt is a six-bit count");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (YOUNGER & 15) | ((YOUNGER >> 4) << 14));
        __syncthreads();   // that tile is published; everybody is done with the stage the next request overwrites
        const int q_rows = buf * 2 * BYTES + ll.rows, g_rows = q_rows + BYTES;
        const int q_cols = buf * 2 * BYTES + ll.cols, g_cols = q_cols + BYTES;
        const int req_stage = (buf + STAGES - 1) % STAGES;
        static_assert(2 * DB == KS, "a block's gradient products are as many MFMA pairs as its score steps");
        constexpr int NP = 4 * KS;      // MFMA pairs of a tile
        constexpr int AHEAD = 3;        // operand reads run this many pairs ahead
        constexpr int WPP = 8 / KS;     // weights (of a lane's 16 query rows per block) dealt behind one MFMA
        constexpr int STATS_AHEAD = 2;  // row statistics are read this many pairs before their first use
        f32x16 sacc[2], gacc[2];
        bf16x8 pp[2][2], pd[2][2];      // P and dS in the B-operand layout: lane = key, eight registers = eight query rows
        bf16x8 op_q[NP], op_g[NP];      // pair i: rows of Q / G (scores) or columns of Q / G (gradient products)
        auto read_ops = [&](int i) {
            const int ph = i / KS, x = i % KS;
            if (ph < 2) {
                op_q[i] = read_rows<D>(lds, q_rows, ph, x), op_g[i] = read_rows<D>(lds, g_rows, ph, x);
            } else {
                op_g[i] = read_cols<D>(lds, g_cols, (ph - 2) * 32 + (x / DB) * 16, x % DB);
                op_q[i] = read_cols<D>(lds, q_cols, (ph - 2) * 32 + (x / DB) * 16, x % DB);
            }
        };
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) read_ops(i);
        issue_flags(req_stage);
        if constexpr (!POW2) {
#pragma unroll
            for (int x = 0; x < LOADS_PER_TILE; ++x) issue_load(req_stage, x);
            prepare_all();
        }
        KSA_FENCE();

        // statistics of rows 8 gg + 4 h .. + 3 of block qb: the rows of a lane's score registers 4 gg .. 4 gg + 3
        struct Stats { f32x4 l4; int4 lo4, span4; };
        Stats stats[2][4];
        auto read_stats = [&](int qb, int gg) {
            const int row0 = qb * 32 + 8 * gg + 4 * h;
            stats[qb][gg].l4 = *reinterpret_cast<const f32x4 *>(&st_lse[buf][row0]);
            if constexpr (MASKED) {
                stats[qb][gg].lo4 = *reinterpret_cast<const int4 *>(&st_lo[buf][row0]);
                stats[qb][gg].span4 = *reinterpret_cast<const int4 *>(&st_span[buf][row0]);
            }
        };
        // dP of block qb starts from minus delta of its rows (the workspace holds it with that sign), read straight into
        // the accumulator of the dO V^T MFMAs: the subtraction dP - delta costs no instruction
        auto start_dp = [&](int qb) {
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                const f32x4 nd = *reinterpret_cast<const f32x4 *>(&st_dl[buf][qb * 32 + 8 * gg + 4 * h]);
#pragma unroll
                for (int e = 0; e < 4; ++e) gacc[qb][4 * gg + e] = nd[e];
            }
        };
        start_dp(0);
        // weights of score register g of block qb (one query row of the lane's key); the bf16 pair is packed when
        // its second member is done
        float pf[2][16], df[2][16];
        auto weight = [&](int qb, int g) {
            const Stats &cur = stats[qb][g / 4];
            const int lo_e[4] = {cur.lo4.x, cur.lo4.y, cur.lo4.z, cur.lo4.w};
            const int span_e[4] = {cur.span4.x, cur.span4.y, cur.span4.z, cur.span4.w};
            const int e = g % 4;
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[qb][g], sl, -cur.l4[e]));
            // one subtraction and one unsigned compare: lo <= key < lo + span
            if constexpr (MASKED) p = (unsigned)(key - lo_e[e]) < (unsigned)span_e[e] ? p : 0.f;
            pf[qb][g] = p;
            df[qb][g] = p * gacc[qb][g];   // gacc = dO . v - delta: its MFMAs started from minus delta
            if (g % 2 == 1) {
                pp[qb][g / 8][g % 8 - 1] = (__bf16)pf[qb][g - 1], pp[qb][g / 8][g % 8] = (__bf16)pf[qb][g];
                pd[qb][g / 8][g % 8 - 1] = (__bf16)df[qb][g - 1], pd[qb][g / 8][g % 8] = (__bf16)df[qb][g];
            }
        };
        // first pair whose weights use the statistics group gg of block qb
        auto first_use = [](int qb, int gg) { return (1 + qb) * KS + 4 * gg / (2 * WPP); };

        // one phase of the stream (a loop of its own per phase, so that each unrolls completely)
        auto phase = [&](auto ph_tag) {
            constexpr int ph = decltype(ph_tag)::value;
#pragma unroll
            for (int x = 0; x < KS; ++x) {
                const int i = ph * KS + x;
                if (i + AHEAD < NP) read_ops(i + AHEAD);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg)
                        if (i == (first_use(qb, gg) - STATS_AHEAD > 0 ? first_use(qb, gg) - STATS_AHEAD : 0)) read_stats(qb, gg);
                // the pair's two MFMAs, each followed by its share of the other work
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int slot = 2 * x + half;   // MFMA number within the phase
                    if constexpr (ph < 2) {
                        if (half == 0) {
                            if (x == 0)
                                mfma_score<true>(sacc[ph], op_q[i], kreg[x]);
                            else
                                mfma_score<false>(sacc[ph], op_q[i], kreg[x]);
                        } else {
                            mfma_score<false>(gacc[ph], op_g[i], vreg[x]);   // started from minus delta
                        }
                        if (ph == 0 && x == KS - 3 && half == 1) start_dp(1);
                    } else if (half == 0) {
                        // dV^T += G^T P, dK^T += Q^T dS for (16-row group x / DB, 32-column block x % DB) of block ph - 2
                        mfma_acc(dvacc[x % DB], op_g[i], pp[ph - 2][x / DB]);
                    } else {
                        mfma_acc(dkacc[x % DB], op_q[i], pd[ph - 2][x / DB]);
                    }
                    if constexpr (POW2 && ph == 0) {
                        if (slot < LOADS_PER_TILE) issue_load(req_stage, slot);
                    }
                    if constexpr (POW2 && ph == 3) {
                        if (slot == 0) prepare_tile();
                        if (slot >= 1 && slot - 1 < NI) prepare_row(slot - 1);
                    }
                    if constexpr (ph == 1 || ph == 2) {
                        // The scores of block ph - 1 were completed by the pair before this one.  The compiler does
                        // not know that the statements above are MFMAs: the empty statement keeps the code that reads
                        // those scores behind this pair's two MFMAs, which take longer to issue than the last results
                        // need to land.  (The first MFMA's share of the weights moves behind the second one.)
                        if (slot == 1) {
                            asm volatile("" : "+v"(sacc[ph - 1]), "+v"(gacc[ph - 1]));
#pragma unroll
                            for (int y = 0; y < WPP; ++y) weight(ph - 1, y);
                        }
                        if (slot >= 1) {
#pragma unroll
                            for (int y = 0; y < WPP; ++y) weight(ph - 1, slot * WPP + y);
                        }
                    }
                    KSA_FENCE();
                }
            }
        };
        phase(std::integral_constant<int, 0>{});
        phase(std::integral_constant<int, 1>{});
        phase(std::integral_constant<int, 2>{});
        phase(std::integral_constant<int, 3>{});
        buf = (buf + 1) % STAGES;
    };
#undef KSA_RUN
    auto next_is_full = [&]() { return ((full_mask >> buf) & 1u) != 0; };
    int left = n_tiles;
    while (left > 0) {
        if (next_is_full()) {
            do step(std::false_type{}), --left;
            while (left > 0 && next_is_full());
        } else {
            do step(std::true_type{}), --left;
            while (left > 0 && !next_is_full());
        }
    }

    // nothing of this workgroup is in flight any more when it leaves (the last requests fetched tiles nobody reads)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    accumulators_settle();
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

namespace {
int64_t pad64(int64_t x) { return (x + 63) / 64 * 64; }
// fp32 slots of one statistics array: B Hq (text rows + summary rows, each rounded up to 64)
int64_t stat_slots(const ksa_params &p) {
    const int64_t n_sum = (int64_t)(p.n_text / p.chunk_len) * p.n_summary;
    return (int64_t)p.batch * p.n_q_heads * (pad64(p.n_text) + pad64(n_sum));
}
}  // namespace

size_t ksa_prefill_bwd_workspace_size(const ksa_params &p, int64_t) {
    return (size_t)(2 * stat_slots(p) * (int64_t)sizeof(float));
}

int ksa_launch_prefill_bwd(const KsaPrefillBwdLaunch &L, void *stream) {
    BwdArgs a;
    a.q = static_cast<const __bf16 *>(L.q);
    a.k = static_cast<const __bf16 *>(L.k);
    a.v = static_cast<const __bf16 *>(L.v);
    a.o = static_cast<const __bf16 *>(L.o);
    a.g = static_cast<const __bf16 *>(L.d_o);
    a.lse = L.lse;
    a.lse2c = static_cast<float *>(L.workspace);
    a.dlc = a.lse2c + stat_slots(L.p);
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
    a.stack = L.head_stack;
    a.stack_shift = log2_exact(L.head_stack);
    if (a.stack_shift < 0 || L.head_stack > KSA_MAX_HEAD_STACK || a.group % L.head_stack != 0) return KSA_ERR_INVALID_ARG;
    a.n_q_heads = L.p.n_q_heads;
    a.n_kv_heads = L.p.n_kv_heads;
    a.batch = L.p.batch;
    a.self_only = (L.p.flags & KSA_FLAG_SUMMARY_SELF_ONLY) ? 1 : 0;
    a.n_text = L.p.n_text;
    a.n_sum = (L.p.n_text / L.p.chunk_len) * L.p.n_summary;
    a.sum_tiles = (a.n_sum + KEYS_PER_WG - 1) / KEYS_PER_WG;
    a.nt_pad = (int32_t)pad64(a.n_text);
    a.ns_pad = (int32_t)pad64(a.n_sum);
    a.aug_len = L.aug_len;
    a.scale = L.p.softmax_scale;
    a.scale_log2e = L.p.softmax_scale * 1.4426950408889634f;
    if (!L.workspace || L.workspace_bytes < ksa_prefill_bwd_workspace_size(L.p, L.aug_len)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    if (L.n_entries <= 0 || L.aug_len <= 0) return KSA_OK;
    if (L.p.head_dim != 128 && L.p.head_dim != 64) return KSA_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);

    const int64_t n_rows = stat_slots(L.p);
    const int64_t delta_blocks = (n_rows * (L.p.head_dim / 8) + 255) / 256;
    const int text_tiles = (a.n_text + KEYS_PER_WG - 1) / KEYS_PER_WG;
    if (delta_blocks >= ((int64_t)1 << 31) || L.p.batch > 65535 ||
        ((int64_t)a.sum_tiles + text_tiles) * L.p.n_kv_heads * L.p.batch >= ((int64_t)1 << 31))
        return KSA_ERR_UNSUPPORTED;
    const bool pow2 = a.c_shift >= 0 && (a.m == 0 || a.m_shift >= 0);
    {   // both kernels address the rows of a streamed tile (Q and dO in the dK/dV kernel, K and V in the dQ kernel) by
        // unsigned 32-bit byte offsets from the tile's first row
        const int64_t span_text = 63 + (63 / a.c + 1) * (int64_t)a.m;
        const int64_t span_sum = a.m > 0 ? 63 + (63 / a.m + 1) * (int64_t)a.c : 0;
        const int64_t span = span_text > span_sum ? span_text : span_sum;
        int64_t row_elems = a.qs[1] > a.os[1] ? a.qs[1] : a.os[1];
        row_elems = row_elems > a.ks[1] ? row_elems : a.ks[1];
        if (a.qs[1] <= 0 || a.os[1] <= 0 || a.ks[1] <= 0 || span * row_elems * 2 + 2 * L.p.head_dim >= ((int64_t)1 << 32))
            return KSA_ERR_UNSUPPORTED;
        // ... and the dK/dV kernel multiplies the head strides of q and d_o as unsigned 32-bit numbers
        if (a.qs[2] >= ((int64_t)1 << 32) || a.os[2] >= ((int64_t)1 << 32) || L.aug_len >= ((int64_t)1 << 31)) return KSA_ERR_UNSUPPORTED;
    }
    const dim3 block(NW * 64), grid_dq(L.n_entries), grid_dkv((unsigned)((a.sum_tiles + text_tiles) * L.p.n_kv_heads * L.p.batch));
    if (L.p.head_dim == 128) {
        hipLaunchKernelGGL(ksa_bwd_delta_kernel<128>, dim3((unsigned)delta_blocks), dim3(256), 0, st, a, n_rows);
        if (pow2)
            hipLaunchKernelGGL((ksa_bwd_dq_kernel<128, true>), grid_dq, block, 0, st, a);
        else
            hipLaunchKernelGGL((ksa_bwd_dq_kernel<128, false>), grid_dq, block, 0, st, a);
        if (pow2)
            hipLaunchKernelGGL((ksa_bwd_dkv_kernel<128, true>), grid_dkv, block, 0, st, a);
        else
            hipLaunchKernelGGL((ksa_bwd_dkv_kernel<128, false>), grid_dkv, block, 0, st, a);
    } else {
        hipLaunchKernelGGL(ksa_bwd_delta_kernel<64>, dim3((unsigned)delta_blocks), dim3(256), 0, st, a, n_rows);
        if (pow2)
            hipLaunchKernelGGL((ksa_bwd_dq_kernel<64, true>), grid_dq, block, 0, st, a);
        else
            hipLaunchKernelGGL((ksa_bwd_dq_kernel<64, false>), grid_dq, block, 0, st, a);
        if (pow2)
            hipLaunchKernelGGL((ksa_bwd_dkv_kernel<64, true>), grid_dkv, block, 0, st, a);
        else
            hipLaunchKernelGGL((ksa_bwd_dkv_kernel<64, false>), grid_dkv, block, 0, st, a);
    }
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}
