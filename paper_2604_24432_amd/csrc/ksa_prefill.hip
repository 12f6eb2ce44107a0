// KSA prefill forward for gfx950: flash-style online softmax over the live key tiles of the schedule.
//
// One workgroup (4 wavefronts of 64 lanes, one per SIMD) owns one query tile of one batch entry for S query
// heads of one KV head (S = 1, 2 or 4: the schedule's head stack); each wave owns 32*QB query rows of one head:
// wave w takes head w % S and row block w / S of the tile, so all waves of a workgroup share their K / V tiles.  Scores are produced TRANSPOSED, S^T = K Q^T, with
// v_mfma_f32_32x32x16_bf16: the 32x32 result block gives lane l the query column l%32 and the key rows
// 8*(g/4) + 4*(l/32) + g%4 for its 16 registers g, so
//   - the softmax statistics of a query row live in one lane pair (l, l^32): the row maximum is an in-lane
//     reduction plus one v_permlane32_swap, no LDS, no shuffle tree;
//   - the same registers, rounded to bf16, are already the B operand of O^T += V^T P^T (eight registers
//     of one lane = eight k slots), so P never leaves the register file;
//   - the rescale factor of the output accumulator is a per-lane scalar.
// K tiles (64 keys) go from global memory straight into LDS (global_load_lds_dwordx4, no VGPR staging) with
// an XOR swizzle of the 16-byte chunks applied on the global side and are read with ds_read_b128.
//
// Two kernels come out of one template.  PIPELINED = true (work items all of whose key runs meet the
// conditions the scheduler checks; every item of the paper's shapes): a software-pipelined loop over 32-key
// sub-tiles, three LDS buffers per operand, V read from a key-major copy made by ksa_vt_kernel so that the
// V^T operand is one ds_read_b128 as well; masked runs (window edges, the causal diagonal, summary rows) go
// through the same loop and clip every score to its row's visible key range.  PIPELINED = false: the
// remaining items, with a plain load -> compute loop per tile and the gfx950 transposing LDS read
// (ds_read_b64_tr_b16) for V^T out of the row-major tile.
// The running maximum is only raised when a tile exceeds it by more than 2^8 in the exponent domain, so the
// accumulator rescale almost never runs; results are unchanged because the final 1/l normalisation uses
// the same reference.
//
// Rows are addressed in two compact index spaces, text index i and summary ordinal u (Eq. 1):
//   augmented row of text i    = (i / c) * (c + m) + i % c
//   augmented row of summary u = (u / m) * (c + m) + c + u % m
// and every query row's visible set is one range of each space (Eq. 3), so a masked score costs one add,
// one unsigned compare and one select.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "ksa_device.h"
#include "ksa_internal.h"

namespace {

constexpr int NW = 4;                         // waves per workgroup: one per SIMD
constexpr int RW = KSA_K_TILE / NW;           // rows of a key tile each wave fetches
constexpr int BN = KSA_K_TILE;                // keys per tile
constexpr int QB = KSA_Q_TILE / (NW * 32);    // 32-row query blocks per wave
static_assert(KSA_Q_TILE == NW * QB * 32, "query tile must be a whole number of 32-row blocks per wave");
static_assert(BN == 64, "key tile is two 32-key MFMA blocks");
constexpr float RESCALE_THRESHOLD_LOG2 = 8.0f;   // raise the running max only for a jump above 2^8


struct PrefillArgs {
    const __bf16 *q, *k, *v;
    __bf16 *o;
    float *lse;
    int64_t qs[3], ks[3], os[3];   // {batch, row, head} strides in elements
    const __bf16 *vt;              // key-major copy of V per index space (see ksa_vt_kernel)
    float *knorm_tiles;            // workspace: largest squared K row norm per (batch, KV head, 64-key tile)
    float *knorm;                  // workspace: largest squared K row norm per (batch, KV head)
    int64_t vt_sum_off;            // element offset of the summary-space part of vt
    int32_t nt_pad, ns_pad;        // row lengths (keys) of the text / summary parts
    int32_t n_text, n_sum;         // keys per index space
    int32_t n_kv_heads;
    const KsaWorkItem *items;
    const KsaWgEntry *entries;
    int32_t c, m, C, w;            // chunk_len, n_summary, window_chunks, c + m
    int32_t c_shift, m_shift;      // log2 when a power of two, else -1
    int32_t group;                 // Hq / Hkv
    int32_t stack, stack_shift;    // query heads per workgroup (1, 2 or 4) and its log2
    int32_t n_q_heads;
    int32_t self_only;
    int64_t aug_len;
    float scale, scale_log2e;
};

__device__ __forceinline__ float other_half(float x) {
    // value held by lane l^32
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

// LDS tile: row-major [64][D] bf16, the 16-byte chunk index XORed with a function of the row
template <int D>
__device__ __forceinline__ int k_swz(int row) { return row & (D / 8 - 1); }
template <int D>
__device__ __forceinline__ int v_swz(int row) { return ((row & 3) << 2) & (D / 8 - 1); }

template <int D>
struct Tile {
    static constexpr int CH = D / 8;           // 16-byte chunks per row
    static constexpr int RPI = 64 / CH;        // rows covered by one wavefront load instruction
    static constexpr int NI = RW / RPI;        // load instructions per wave per tile (RW rows per wave)
    static_assert(RW % RPI == 0 && NI >= 1, "a wave's share of a tile is a whole number of load instructions");
    static constexpr int VROWS = D / NW;       // head-dim rows of a key-major V tile each wave fetches (128 bytes each)
    static constexpr int NIV = VROWS / 8;      // load instructions per wave for it
    static_assert(VROWS % 8 == 0 && NIV >= 1, "a wave's share of a key-major V tile is a whole number of load instructions");
    static constexpr int KS = D / 16;          // k steps of the score MFMA
    static constexpr int DB = D / 32;          // 32-column blocks of the output
    static constexpr int BYTES = BN * D * 2;
    static constexpr int STAGE_ROW = D * 2 + 16;   // bytes per row of the epilogue's staging area (32 rows per wave)
    // pipelined loop: LDS operand reads are issued this many k steps (two MFMAs each) ahead of their use (measured:
    // four steps are 1 % faster than two; more would not fit into the 256 VGPRs next to the scores and the Q operand)
    static constexpr int RING = KS / 2 > 2 ? KS / 2 : 2;
};

// Per-lane element offsets (relative to the tile's first row) of the 16-byte pieces this lane fetches.
template <int D>
struct LaneOffsets {
    int k[Tile<D>::NI], v[Tile<D>::NI];
    int vt[Tile<D>::NIV];   // key-major V: offsets relative to (row 0 of the head, first key of the tile)
};

// Offsets for the tile whose first key is kt; rows beyond `last` (inclusive bound) are clamped to it.
template <int D>
__device__ __forceinline__ void lane_offsets(const PrefillArgs &a, int space, int kt, int last, int wave, int lane,
                                             int base_aug, LaneOffsets<D> &off) {
    using T = Tile<D>;
#pragma unroll
    for (int i = 0; i < T::NI; ++i) {
        const int row = RW * wave + T::RPI * i + lane / T::CH;
        const int pch = lane % T::CH;
        int kc = kt + row;
        kc = kc < last ? kc : last;
        const int rel = (aug_row(a, space, kc) - base_aug) * (int)a.ks[1];
        off.k[i] = rel + ((pch ^ k_swz<D>(row)) << 3);
        off.v[i] = rel + ((pch ^ v_swz<D>(row)) << 3);
    }
}

// Key-major V tile in LDS: [D head-dim rows][8 pieces of 16 bytes]; a piece holds the eight keys one lane feeds to
// one P V MFMA.  The piece index is XORed with (row >> 1) & 7, which makes the 16 lanes of a ds_read_b128 phase hit
// 16 different 16-byte bank groups.
__device__ __forceinline__ int vt_swz(int d_row) { return (d_row >> 1) & 7; }

template <int D>
__device__ __forceinline__ void lane_offsets_vt(int vt_stride, int wave, int lane, LaneOffsets<D> &off) {
    using T = Tile<D>;
#pragma unroll
    for (int i = 0; i < T::NIV; ++i) {
        const int d_row = T::VROWS * wave + 8 * i + (lane >> 3);
        off.vt[i] = d_row * vt_stride + (((lane & 7) ^ vt_swz(d_row)) << 3);
    }
}

template <int D>
__device__ __forceinline__ void issue_tile_load(const __bf16 *gbase, const int (&off)[Tile<D>::NI], unsigned char *lds,
                                                int buf_off, int wave) {
    using T = Tile<D>;
#pragma unroll
    for (int i = 0; i < T::NI; ++i) {
        lds_direct_load_16(gbase + off[i], lds + buf_off + (RW * wave + T::RPI * i) * (D * 2));
    }
}

// Byte addresses inside an LDS tile are written as (per-lane constant XOR small constant) + constant, so that
// a handful of registers plus the instructions' immediate offsets cover every operand read.
struct LaneLds {
    int k;   // K operand: row r, chunk (swizzle(r) ^ h); XOR (s << 5) selects k step s
    int v;   // V^T operand: this lane's address row / column of the transposing read; XOR (db << 6) selects the column block
    int vt;  // V^T operand out of a key-major tile: row r, piece (swizzle(r) ^ h); XOR ((2 * sb + hf) << 5) selects the
             // 16-key group, + db * 4096 the block of 32 head-dim rows
};

template <int D>
__device__ __forceinline__ LaneLds lane_lds(int lane) {
    const int r = lane & 31, h = lane >> 5;
    const int grp = lane >> 4, li = lane & 15;
    // transposing read: lane (grp, li) supplies the address of key 4*(grp/2) + li/4, columns 16*(grp%2) + 4*(li%4) .. +3
    // and receives keys 4*(grp/2) .. +3 of column 16*(grp%2) + li
    const int t_row = 4 * (grp >> 1) + (li >> 2);
    const int t_col = 16 * (grp & 1) + 4 * (li & 3);
    LaneLds L;
    L.k = r * (D * 2) + ((k_swz<D>(r) ^ h) << 4);
    L.v = t_row * (D * 2) + (((t_col >> 3) ^ v_swz<D>(t_row)) << 4) + ((t_col & 7) << 1);
    L.vt = r * 128 + ((h ^ vt_swz(r)) << 4);
    return L;
}

// S^T (two 32-key blocks) for QB query blocks: sacc[qb][kb] += K[kb] Q[qb]^T
template <int D>
__device__ __forceinline__ void score_mfma(const unsigned char *lds, int buf_off, const LaneLds &ll,
                                           const bf16x8 (&qreg)[QB][Tile<D>::KS], f32x16 (&sacc)[QB][2]) {
    using T = Tile<D>;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 16; ++g) sacc[qb][kb][g] = 0.f;
#pragma unroll
    for (int s = 0; s < T::KS; ++s) {
        const int a_s = ll.k ^ (s << 5);   // logical chunk 2s + h of row r
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(lds + a_s + (buf_off + kb * 32 * (D * 2)));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                sacc[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[qb][s], sacc[qb][kb], 0, 0, 0);
        }
    }
}

// O^T += V^T P^T
template <int D>
__device__ __forceinline__ void pv_mfma(const unsigned char *lds, int buf_off, const LaneLds &ll,
                                        const bf16x8 (&pb)[QB][2][2], f32x16 (&oacc)[QB][Tile<D>::DB]) {
    using T = Tile<D>;
#pragma unroll
    for (int db = 0; db < T::DB; ++db) {
        const int a_db = ll.v ^ (db << 6);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int o0 = buf_off + (kb * 32 + hf * 16) * (D * 2), o1 = o0 + 8 * (D * 2);
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lds + a_db + o0));
                const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lds + a_db + o1));
                const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[qb][kb][hf], oacc[qb][db], 0, 0, 0);
            }
    }
}

// Online-softmax state of one lane's query rows.  m_ref is the reference maximum (raw score units) the
// exponentials are taken against; l_part is this lane's part of the row sum (the lane pair is added up at
// the end).
struct RowState {
    float m_ref[QB], l_part[QB];
    f32x4 l_sum[QB];    // pipelined kernel: row sums kept by sum_half(): lanes 0..15, registers 0 (query = lane) and 1 (+ 16)
};

// Row maxima of a score tile; returns true if some lane's row exceeds its reference by more than the threshold.
__device__ __forceinline__ bool tile_max(const f32x16 (&sacc)[QB][2], const RowState &st, float sl, float (&tmax)[QB]) {
    bool raise = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float mx = sacc[qb][0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 16; ++g) mx = fmaxf(mx, sacc[qb][kb][g]);
        mx = fmaxf(mx, other_half(mx));
        tmax[qb] = mx;
        raise |= (mx - st.m_ref[qb]) * sl > RESCALE_THRESHOLD_LOG2;
    }
    return __builtin_amdgcn_ballot_w64(raise) != 0;   // wave-uniform
}

// Raises the reference maxima to the tile maxima and rescales the row sums and the output accumulators (generic
// kernel).  Rarely taken: see RESCALE_THRESHOLD_LOG2.
template <int D>
__device__ __forceinline__ void raise_reference(RowState &st, const float (&tmax)[QB], f32x16 (&oacc)[QB][Tile<D>::DB],
                                                float sl) {
    using T = Tile<D>;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float m_new = fmaxf(st.m_ref[qb], tmax[qb]);
        // (old - new) first: equal references (also the -1e30 start value) must give exactly 2^0
        const float alpha = __builtin_amdgcn_exp2f((st.m_ref[qb] - m_new) * sl);
        st.m_ref[qb] = m_new;
        st.l_part[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < T::DB; ++db)
#pragma unroll
            for (int g = 0; g < 16; ++g) oacc[qb][db][g] *= alpha;
    }
}

// The pipelined kernel's version.  mx are the LANE's maxima of the pending scores; the two lanes of a row are combined
// here.  The output accumulators live in accumulation registers and are only ever touched by the inline-assembly
// MFMAs of pv_mfma_raw() and by this routine, which scales them in place, also in assembly: left to the compiler, the
// copies to VGPRs that a plain multiply needs get hoisted out of this block into the loop around it, where they would
// drain the MFMA pipe on every tile.
template <int D>
__device__ __forceinline__ void raise_reference_pl(RowState &st, const float (&mx)[QB], f32x16 (&oacc)[QB][Tile<D>::DB],
                                                   float sl) {
    using T = Tile<D>;
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMA results reach the register file
    // The accumulators are re-defined here as far as the compiler can tell: the per-register copies it makes for the
    // statements below then depend on this block and cannot be hoisted in front of the branch that guards it (where
    // they would run on every tile).
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        asm volatile("" : "+a"(st.l_sum[qb]));
#pragma unroll
        for (int db = 0; db < T::DB; ++db) asm volatile("" : "+a"(oacc[qb][db]));
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float m_new = fmaxf(st.m_ref[qb], fmaxf(mx[qb], other_half(mx[qb])));
        // (old - new) first: equal references (also the -1e30 start value) must give exactly 2^0
        const float alpha = __builtin_amdgcn_exp2f((st.m_ref[qb] - m_new) * sl);
        st.m_ref[qb] = m_new;
        // the row sums: lane j < 16 holds query j in register 0 and query j + 16 in register 1
        const float alpha_hi = __shfl(alpha, (threadIdx.x & 15) + 16);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float acc = st.l_sum[qb][i], tmp;
            asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                         : "+a"(acc), "=&v"(tmp)
                         : "v"(i == 0 ? alpha : alpha_hi));
            st.l_sum[qb][i] = acc;
        }
#pragma unroll
        for (int db = 0; db < T::DB; ++db)
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                float acc = oacc[qb][db][g], tmp;
                asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                             : "+a"(acc), "=&v"(tmp)
                             : "v"(alpha));
                oacc[qb][db][g] = acc;
            }
    }
    asm volatile("s_nop 7" ::: "memory");
    // Register spills around this block are reloaded from scratch memory.  Waiting for them here keeps the compiler
    // from placing its own s_waitcnt vmcnt(0) after the block rejoins the loop, where it would also wait for the
    // LDS-direct tile loads in flight (the hardware counter is shared) on every tile.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0) only
}

// O^T += V^T P^T with the accumulator in accumulation registers, whatever the build's default for MFMA results is.
// The compiler does not know that this statement is an MFMA: nothing but further pv_mfma_raw() statements and
// raise_reference_pl() may touch the accumulators until accumulators_settle() has run.
__device__ __forceinline__ void pv_mfma_raw(f32x16 &acc, const bf16x8 &v_op, const u32x4 &p_op) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(v_op), "v"(p_op));
}
// Waits until the last pv_mfma_raw() results are in the register file; later accesses stay behind it.
template <int D>
__device__ __forceinline__ void accumulators_settle(f32x16 (&oacc)[QB][Tile<D>::DB], RowState &st) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(oacc[0][0]));
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) asm volatile("" : "+a"(st.l_sum[qb]));
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < Tile<D>::DB; ++db)
            if (qb + db > 0) asm volatile("" : "+a"(oacc[qb][db]));
}

// p = 2^((s - m_ref) * scale * log2 e) rounded to bf16 in the B-operand layout of P V.  The row sum adds up the
// ROUNDED values (v_dot2c_f32_bf16 against (1, 1)), so that O = sum(p v) / sum(p) is normalised by exactly the
// weights that were multiplied: a row dominated by one key returns that key's V row up to output rounding.
__device__ __forceinline__ void exp_and_pack(const f32x16 (&sacc)[QB][2], bf16x8 (&pb)[QB][2][2], RowState &st, float sl) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float msl = st.m_ref[qb] * sl;
        float rsum = st.l_part[qb];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 16; g += 2) {
                bf16x2 pk;
                pk[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][g], sl, -msl));
                pk[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][g + 1], sl, -msl));
                rsum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, rsum, false);
                pb[qb][kb][g / 8][g % 8] = pk[0];
                pb[qb][kb][g / 8][g % 8 + 1] = pk[1];
            }
        st.l_part[qb] = rsum;
    }
}

// ---- pieces of the pipelined loop, which advances in sub-tiles of 32 keys -------------------------------------
// Source order below is the intended issue order: every MFMA group is followed by a slice of independent VALU
// work, and the order is pinned with scheduling barriers, because one wave per SIMD has nobody else to fill its
// MFMA latency.
#define KSA_STEP_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int D>
__device__ __forceinline__ bf16x8 read_k_operand(const unsigned char *lds, int lk, int s) {
    return *reinterpret_cast<const bf16x8 *>(lds + (lk ^ (s << 5)));
}

// V^T operand (32 head-dim rows x 16 keys) out of a key-major tile: one 16-byte read per lane
__device__ __forceinline__ bf16x8 read_vt_operand(const unsigned char *lds, int lvt, int hf, int db) {
    return *reinterpret_cast<const bf16x8 *>(lds + ((lvt ^ (hf << 5)) + db * 4096));
}

// The scores are consumed by VALU code (exp2, max), so the score MFMAs should leave them in ordinary VGPRs: with the
// results in accumulation registers every score costs a v_accvgpr_read, and such a read while other MFMAs are in
// flight was measured to cost about as much as an exponential.  The library is built with the compiler option that
// gives MFMA results and accumulator inputs VGPRs (-mllvm -amdgpu-mfma-vgpr-form), which covers this kernel's output
// accumulators as well; register allocation, copies and the wait states an MFMA result needs before VALU code may
// read it all stay with the compiler.
__device__ __forceinline__ void score_mfma_first(f32x16 &acc, const bf16x8 &k_op, const bf16x8 &q_op) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_op, q_op, f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0);
}
__device__ __forceinline__ void score_mfma_next(f32x16 &acc, const bf16x8 &k_op, const bf16x8 &q_op) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_op, q_op, acc, 0, 0, 0);
}
// Reads of the tuple written after this statement stay behind it, i.e. in the slot they were written for.
__device__ __forceinline__ void scores_ready(f32x16 &acc) { asm volatile("" : "+v"(acc)); }

// Scores of one 32-key block alone (pipeline fill).
template <int D>
__device__ __forceinline__ void qk_only(const unsigned char *lds, int k_off, const LaneLds &ll,
                                        const bf16x8 (&qreg)[QB][Tile<D>::KS], f32x16 (&s_out)[QB]) {
    using T = Tile<D>;
    const int lk = ll.k + k_off;
#pragma unroll
    for (int s = 0; s < T::KS; ++s) {
        const bf16x8 ka = read_k_operand<D>(lds, lk, s);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (s == 0)
                score_mfma_first(s_out[qb], ka, qreg[qb][s]);
            else
                score_mfma_next(s_out[qb], ka, qreg[qb][s]);
        }
    }
}

// One instruction's worth (1 KiB per wave) of a tile load.
// (gbase wave-uniform, off_b the lane's byte offset from it, lds_wave the wave's first LDS byte of the buffer)
template <int D>
__device__ __forceinline__ void issue_tile_load_part(const __bf16 *gbase, unsigned off_b, unsigned lds_wave, int i) {
    using T = Tile<D>;
    lds_direct_load_16_s(gbase, off_b, lds_wave + T::RPI * i * (D * 2));
}

template <int D>
__device__ __forceinline__ void issue_vt_load_part(const __bf16 *gbase, unsigned off_b, unsigned lds_wave, int i) {
    lds_direct_load_16_s(gbase, off_b, lds_wave + 8 * i * 128);
}

// What the synchronising sub-tile of a tile does besides its arithmetic: wait for this wave's pieces of the next
// tile, meet the other waves, and request the tile after that.
template <int D>
struct TileSync {
    const __bf16 *kg, *vg;          // global addresses (wave-uniform) of the first row of the tile to request
    const unsigned *k_off, *v_off;  // the lane's byte offsets from them, one per load instruction
    unsigned k_dst, v_dst;          // LDS byte addresses of this wave's share of the buffers it goes to
};

// v_max3_f32 without the NaN-quieting self-maxima that fmaxf expands to
__device__ __forceinline__ float max3(float a, float b, float c) {
    float x;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(x) : "v"(a), "v"(b), "v"(c));
    return x;
}

// Row sums by the matrix unit: acc(16x16) += A(16x32) P^T(32x16) with the eight packed weights of one 16-key half as
// the B operand, exactly as they enter P V.  As B of the 16x16x32 MFMA, lane l supplies column l % 16, k group l / 16;
// the lanes of column j are j, j + 16, j + 32, j + 48, which hold the weights of query j (lane halves 0 and 1: groups
// 0 and 2) and of query j + 16 (groups 1 and 3).  A is an indicator matrix: row 0 is one on groups 0 and 2, row 1 on
// groups 1 and 3, all else zero (`ind`: all ones in lanes 0, 32, 17 and 49).  Result: lane j < 16 holds in register 0
// the sum over all sixteen weights of query j, in register 1 that of query j + 16, in fp32, of the ROUNDED weights, so
// O = sum(p v) / sum(p) is normalised by what was multiplied and a row dominated by one key returns that key's V row
// up to output rounding.  (Adding the fp32 weights before rounding costs more issue time and, with outlier keys, output
// errors above the tolerance; v_dot2c_f32_bf16 on pairs costs 16 cycles of issue per pair; the 4x4x4 MFMA sums only
// four weights for the same 16 cycles in the matrix pipe.)
// Like pv_mfma_raw(), the accumulator stays in accumulation registers and the compiler does not know that this is an
// MFMA: `ind` must be a register that no VALU instruction has just written (the kernel pins it once), and the packed
// weights come from two slots before.
__device__ __forceinline__ void sum_half(f32x4 &acc, const u32x4 &ind, const u32x4 &p_op) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(ind), "v"(p_op));
}
// two fp32 weights rounded to bf16, packed (first in the low half)
__device__ __forceinline__ unsigned pack_pair(float w0, float w1) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 pk = {(__bf16)w0, (__bf16)w1};
    return __builtin_bit_cast(unsigned, pk);
}

// One sub-tile (32 keys) of the pipelined loop, written in issue order as a sequence of slots.  A slot is one MFMA
// plus a slice of independent VALU work and ends with a scheduling fence.  A wave issues in order and every
// instruction, MFMA included, occupies the SIMD's one vector issue port (about 5 cycles for a plain VALU instruction,
// 10 for an exponential, 16 for v_dot2c_f32_bf16, 4 for an MFMA, whose 32 cycles in the matrix pipe run in the
// background): the loop is bound by the sum of those, so the code below is written to need few instructions.
//   score slots (KS * QB)         s_next = K[next block] Q^T
//   P V slots (2 * DB * QB)       O^T += V^T P^T, 16-key half by 16-key half
//   VALU stream, spread over the slots:
//     weight e of the current block in stages, F  x = s * sl - m_ref * sl,  X  w = exp2(x),  C  pack a pair to bf16,
//     L  add a packed 16-key half to the row sums (sum_half), in consecutive slots (a dependent instruction directly
//     behind its producer stalls the wave); first the 16-key half the first P V slots need, then the other half;
//     R(j)  row maximum over two of the next scores (at least four MFMAs behind the last score MFMA), with the
//     scores clipped to the row's visible key range first when the run is MASKED.
// The scale stays a multiply per score: folded into Q (rounded to bf16 again) it would perturb a score by 2^-9 of
// its magnitude, which the outlier-key workload turns into output errors above the tolerance.
// sv_cur / sv_next are the scores as plain VGPR values (QB x 16 per lane).  K operands: steps 0 .. RING-1 of this
// sub-tile arrive in ka (read from LDS during the previous sub-tile), the others are read RING steps ahead into the
// register just used, and so are the V operands: every LDS read is issued at least RING steps before its use.  With
// SYNC the per-tile barrier and the requests for the tile after next sit at the start of the P V slots.  Returns true
// if some lane's next scores exceed its reference maximum by more than the threshold; mx_out holds the lane's maxima
// (the lane pair of a row is only combined when a raise happens).
// TRACK = false: the reference maximum is fixed for the whole work item (see static_reference() in the kernel): no row
// maxima, no raise decision; a MASKED run still clips the next scores in the same slots.
template <int D, bool SYNC, bool MASKED, bool TRACK, class Hook>
__device__ __forceinline__ bool subtile(unsigned char *lds, const LaneLds &ll, const bf16x8 (&qreg)[QB][Tile<D>::KS],
                                        f32x16 (&sv_next)[QB], const f32x16 (&sv_cur)[QB], bf16x8 (&ka)[Tile<D>::RING],
                                        int k_off, int v_off, int sb, int k_next_off, f32x16 (&oacc)[QB][Tile<D>::DB],
                                        RowState &st, const u32x4 &ind, float sl, float raise_margin,
                                        float (&mx_out)[QB], const TileSync<D> &sync, int next_key0, const int (&vis_lo)[QB],
                                        const int (&vis_span)[QB], Hook hook) {
    using T = Tile<D>;
    constexpr int NSTEP = 2 * T::DB;              // (hf, db) pairs of the P V phase
    static_assert(NSTEP == T::KS, "one V operand is fetched per score step");
    constexpr int N1 = T::KS * QB;                // score slots
    constexpr int NH = QB * T::DB;                // P V slots per 16-key half
    constexpr int N2 = 2 * NH;
    constexpr int NE = QB * 16;                   // weights per lane
    constexpr int E_SLOTS = N1 + NH - 3;          // slots that start a weight: the last C stage sits two slots before slot
                                                  // N1 + NH (a raw MFMA must not read a register a VALU instruction has
                                                  // only just written)
    constexpr int R_FIRST = N1 + 4;               // first slot that may read sv_next (four MFMAs behind its last MFMA)
    constexpr int R_SLOTS = N1 + N2 - 3 - R_FIRST;   // the row maxima are complete two slots before the end, where the
                                                      // "raise the reference?" decision is taken: in the shadow of the
                                                      // last MFMAs rather than behind them, with the matrix pipe idle
    constexpr int NR = QB * 8;                    // row-maximum units (two scores each)
    static_assert(E_SLOTS >= 1 && R_SLOTS >= 1, "the phases are too short for the pipelined VALU stream");
    static_assert((NE / 2 - 1) * E_SLOTS / NE + 2 <= N1 - 2, "the first half's weights are not packed in time");
    static_assert(E_SLOTS - 1 + 4 <= N1 + N2 - 1, "the last row-sum step does not fit into the sub-tile");
    static_assert(1 + T::NI + T::NIV <= N2, "the tile requests do not fit into the P V slots");
    constexpr int RING = T::RING;                 // operands in flight per kind
    const int lk = ll.k + k_off, lv = (ll.vt ^ (sb << 6)) + v_off, lkn = ll.k + k_next_off;
    float msl[QB], mx[QB];
    int mask_base[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        msl[qb] = st.m_ref[qb] * sl;
        mx[qb] = -INFINITY;
        mask_base[qb] = MASKED ? next_key0 - vis_lo[qb] : 0;
    }
    u32x4 p[QB][2];                               // packed weight pairs: the B operand of P V
    bf16x8 va[RING];
    float xs[NE], ws[NE];
    // weight e = hf * (QB * 8) + qb * 8 + i  ->  score register 8 * hf + i of query block qb
    auto slot_of_e = [](int e) { return e * E_SLOTS / NE; };
    auto slot_of_r = [](int j) { return R_FIRST + j * R_SLOTS / NR; };
    auto valu_slice = [&](int u) {
        // exponentials and multiply-adds first, alternating: a transcendental keeps its unit busy for several issue slots
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (slot_of_e(e | 1) + 1 == u) {   // X (both weights of a pair in the slot of the odd one)
                ws[e] = __builtin_amdgcn_exp2f(xs[e]);
                asm volatile("" : "+v"(ws[e]));
                KSA_STEP_FENCE();
            }
            if (slot_of_e(e | 1) == u) {   // F
                const int hf = e / (QB * 8), qb = (e / 8) % QB, i = e % 8;
                xs[e] = fmaf(sv_cur[qb][8 * hf + i], sl, -msl[qb]);
                asm volatile("" : "+v"(xs[e]));
                KSA_STEP_FENCE();
            }
        }
        // L in the middle of the slot: the matrix pipe takes one MFMA at a time and a wave that issues one while the
        // pipe is busy waits for it, so the small MFMA sits about 30 cycles of VALU work behind the slot's big MFMA and
        // has 10 to 20 cycles of VALU work between itself and the next slot's.  Two slots behind the pack: a raw MFMA
        // must not read a register that a VALU instruction has only just written.
#pragma unroll
        for (int e = 7; e < NE; e += 8)
            if (slot_of_e(e) + 4 == u) {
                const int hf = e / (QB * 8), qb = (e / 8) % QB;
                sum_half(st.l_sum[qb], ind, p[qb][hf]);
                KSA_STEP_FENCE();
            }
#pragma unroll
        for (int e = 1; e < NE; e += 2)
            if (slot_of_e(e) + 2 == u) {   // C
                const int hf = e / (QB * 8), qb = (e / 8) % QB, i = e % 8;
                p[qb][hf][i / 2] = pack_pair(ws[e - 1], ws[e]);
            }
#pragma unroll
        for (int j = 0; j < NR; ++j)
            if (slot_of_r(j) == u) {
                const int qb = j / 8, g = 2 * (j % 8);
                if (MASKED) {
                    // key of score register g: next_key0 + 4 * (lane / 32) + 8 * (g / 4) + g % 4; visible iff it lies in
                    // [lo, lo + span); vis_lo holds lo - 4 * (lane / 32)
#pragma unroll
                    for (int x = g; x < g + 2; ++x) {
                        const unsigned rel = (unsigned)(mask_base[qb] + (8 * (x / 4) + x % 4));
                        sv_next[qb][x] = rel < (unsigned)vis_span[qb] ? sv_next[qb][x] : -INFINITY;
                    }
                }
                if constexpr (TRACK) mx[qb] = max3(mx[qb], sv_next[qb][g], sv_next[qb][g + 1]);
            }
    };
    // ---- score slots ----
#pragma unroll
    for (int u = 0; u < N1; ++u) {
        const int sk = u / QB, qb = u % QB;
        if (sk == 0)
            score_mfma_first(sv_next[qb], ka[sk % RING], qreg[qb][sk]);
        else
            score_mfma_next(sv_next[qb], ka[sk % RING], qreg[qb][sk]);
        if (qb == QB - 1) {
            if (sk + RING < T::KS) ka[sk % RING] = read_k_operand<D>(lds, lk, sk + RING);
            if (sk >= T::KS - RING) {
                const int x = sk - (T::KS - RING);
                va[x] = read_vt_operand(lds, lv, x / T::DB, x % T::DB);
            }
        }
        valu_slice(u);
        // the caller's scalar bookkeeping for the NEXT sub-tile (tile addresses, loop state) rides in the shadow of
        // this sub-tile's second MFMA instead of sitting between two sub-tiles with the matrix pipe idle
        if (u == 1) hook();
        KSA_STEP_FENCE();
    }
    // ---- P V slots ----
    bool raise_any = false;
#pragma unroll
    for (int u = 0; u < N2; ++u) {
        const int x = u / QB, qb = u % QB;
        const int hf = x / T::DB, db = x % T::DB;
        pv_mfma_raw(oacc[qb][db], va[x % RING], p[qb][hf]);
        // the V operand RING steps ahead goes into the register this step has just used
        if (qb == QB - 1 && x + RING < NSTEP) va[x % RING] = read_vt_operand(lds, lv, (x + RING) / T::DB, (x + RING) % T::DB);
        if (SYNC) {
            if (u == 0) {
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's pieces of the next tile have landed
                // ... and everyone's; nobody still reads the buffer loaded next.  A bare s_barrier: __syncthreads() would
                // also drain this wave's LDS operand reads in flight (lgkmcnt(0)), which belong to the current tile and
                // may stay in flight.  The "memory" clobber keeps the reads of the published tile behind it.
                asm volatile("s_barrier" ::: "memory");
            }
            // the tile after next, one instruction per slot
            if (u >= 1 && u - 1 < T::NI) issue_tile_load_part<D>(sync.kg, sync.k_off[u - 1], sync.k_dst, u - 1);
            if (u >= 1 + T::NI && u - 1 - T::NI < T::NIV)
                issue_vt_load_part<D>(sync.vg, sync.v_off[u - 1 - T::NI], sync.v_dst, u - 1 - T::NI);
        }
        // the first RING K operands of the following sub-tile, in the second half of the slots
#pragma unroll
        for (int x = 0; x < RING; ++x)
            if (NH + x * NH / RING == u) ka[x] = read_k_operand<D>(lds, lkn, x);
        if (N1 + u == R_FIRST) {
            // from here on the next scores may be read
#pragma unroll
            for (int q2 = 0; q2 < QB; ++q2) scores_ready(sv_next[q2]);
        }
        valu_slice(N1 + u);
        if (TRACK && u == N2 - 2) {
            bool raise = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                mx_out[qb] = mx[qb];
                raise |= mx[qb] > st.m_ref[qb] + raise_margin;   // (mx - m_ref) * sl > threshold
            }
            raise_any = __builtin_amdgcn_ballot_w64(raise) != 0;
        }
        KSA_STEP_FENCE();
    }
    return raise_any;
}

// What a wave does in place of a sub-tile of a masked stretch when none of its rows sees a key of the block it would
// take weights from nor of the block it would score (block-diagonal summary rows, window edges): no MFMA, no
// exponential.  It keeps the pipeline state the neighbouring sub-tiles rely on: the next scores are all "masked", the
// first RING K operands of the following block are read, and with SYNC it waits for its tile loads, meets the other
// waves at the tile's one barrier and issues its share of the requests for the tile after next.
template <int D, bool SYNC>
__device__ __forceinline__ void idle_subtile(unsigned char *lds, const LaneLds &ll, f32x16 (&sv_next)[QB],
                                             bf16x8 (&ka)[Tile<D>::RING], int k_next_off, float (&mx_out)[QB],
                                             const TileSync<D> &sync) {
    using T = Tile<D>;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int g = 0; g < 16; ++g) sv_next[qb][g] = -INFINITY;
        mx_out[qb] = -INFINITY;
    }
    if (SYNC) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's pieces of the next tile have landed
        __syncthreads();
#pragma unroll
        for (int i = 0; i < T::NI; ++i) issue_tile_load_part<D>(sync.kg, sync.k_off[i], sync.k_dst, i);
#pragma unroll
        for (int i = 0; i < T::NIV; ++i) issue_vt_load_part<D>(sync.vg, sync.v_off[i], sync.v_dst, i);
    }
#pragma unroll
    for (int x = 0; x < T::RING; ++x) ka[x] = read_k_operand<D>(lds, ll.k + k_next_off, x);
}

// PIPELINED = true: work items all of whose key runs satisfy the conditions of the pipelined loop (the scheduler
// marks them); false: the remaining items, walked with the plain loop.  Two instantiations rather than one kernel
// with both loops keep the register allocation of the pipelined loop free of the plain loop's temporaries.
template <int D, bool PIPELINED>
__global__ __launch_bounds__(NW * 64) void ksa_prefill_kernel(const PrefillArgs a) {
    using T = Tile<D>;
    // three K tiles, then three V tiles: the pipelined loop loads two tiles ahead with one barrier per tile
    // ... and the staging area of the epilogue
    __shared__ __attribute__((aligned(1024))) unsigned char lds[6 * T::BYTES + NW * 32 * T::STAGE_ROW];
    constexpr int K0 = 0, V0 = 3 * T::BYTES;

    const KsaWgEntry ent = a.entries[blockIdx.x];
    if (ent.item < 0) return;
    const KsaWorkItem &item = a.items[ent.item];
    if ((item.pipelined != 0) != PIPELINED) return;
    // The runs' few words are copied into scalar registers here: read through the reference at the start of each run
    // they would be fetched from memory again (the tile requests are opaque memory operations to the compiler), one
    // more memory round trip in front of every run's first tile request.
    static_assert(KSA_MAX_SEGMENTS == 2, "run fields are selected with one compare");
    int run_space[KSA_MAX_SEGMENTS], run_begin[KSA_MAX_SEGMENTS], run_end[KSA_MAX_SEGMENTS];
    int run_full_lo[KSA_MAX_SEGMENTS], run_full_hi[KSA_MAX_SEGMENTS];
#pragma unroll
    for (int x = 0; x < KSA_MAX_SEGMENTS; ++x) {
        run_space[x] = item.seg[x].space, run_begin[x] = item.seg[x].begin, run_end[x] = item.seg[x].end;
        run_full_lo[x] = item.seg[x].full_lo, run_full_hi[x] = item.seg[x].full_hi;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this wave's query head and its block of 32*QB rows of the query tile
    const int b = ent.batch, hq = ent.q_head + (wave & (a.stack - 1)), hkv = ent.q_head / a.group;
    const int wrow = wave >> a.stack_shift;
    const int r = lane & 31, h = lane >> 5;
    const LaneLds ll = lane_lds<D>(lane);

    const int q_space = item.q_space, q_begin = item.q_begin, q_end = item.q_begin + item.q_count;
    const int n_seg = item.n_seg;

    // ---- per-lane query rows: visible ranges (Eq. 3) and the Q operand -------------------------
    int lo_t[QB], hi_t[QB], lo_s[QB], hi_s[QB];   // text / summary ranges
    int q_aug[QB];
    bool q_valid[QB];
    bf16x8 qreg[QB][T::KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int idx = q_begin + (wrow * QB + qb) * 32 + r;
        q_valid[qb] = idx < q_end;
        const int idc = q_valid[qb] ? idx : q_end - 1;
        q_aug[qb] = aug_row(a, q_space, idc);
        if (q_space == KSA_SPACE_TEXT) {
            const int j = div_by(idc, a.c, a.c_shift);
            const int first = j - a.C > 0 ? j - a.C : 0;
            lo_s[qb] = 0;
            hi_s[qb] = first * a.m;
            lo_t[qb] = first * a.c;
            hi_t[qb] = idc + 1;
        } else {
            const int j = div_by(idc, a.m, a.m_shift);
            lo_s[qb] = a.self_only ? idc : j * a.m;
            hi_s[qb] = idc + 1;
            lo_t[qb] = j * a.c;
            hi_t[qb] = (j + 1) * a.c;
        }
        if (!q_valid[qb]) {
            lo_s[qb] = lo_t[qb] = 0x7fffffff;
            hi_s[qb] = hi_t[qb] = 0;
        }
        const __bf16 *qp = a.q + b * a.qs[0] + (int64_t)q_aug[qb] * a.qs[1] + hq * a.qs[2] + h * 8;
#pragma unroll
        for (int s = 0; s < T::KS; ++s) {
            if (q_valid[qb])
                qreg[qb][s] = *reinterpret_cast<const bf16x8 *>(qp + s * 16);
            else
                qreg[qb][s] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    // union of the wave's rows' ranges per space: a masked tile outside it is skipped by the whole wave
    int wlo_t = lo_t[0], whi_t = hi_t[0], wlo_s = lo_s[0], whi_s = hi_s[0];
#pragma unroll
    for (int qb = 1; qb < QB; ++qb) {
        wlo_t = min(wlo_t, lo_t[qb]), whi_t = max(whi_t, hi_t[qb]);
        wlo_s = min(wlo_s, lo_s[qb]), whi_s = max(whi_s, hi_s[qb]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        wlo_t = min(wlo_t, __shfl_xor(wlo_t, off)), whi_t = max(whi_t, __shfl_xor(whi_t, off));
        wlo_s = min(wlo_s, __shfl_xor(wlo_s, off)), whi_s = max(whi_s, __shfl_xor(whi_s, off));
    }
    wlo_t = __builtin_amdgcn_readfirstlane(wlo_t), whi_t = __builtin_amdgcn_readfirstlane(whi_t);
    wlo_s = __builtin_amdgcn_readfirstlane(wlo_s), whi_s = __builtin_amdgcn_readfirstlane(whi_s);

    const __bf16 *kbase = a.k + b * a.ks[0] + hkv * a.ks[2];
    const __bf16 *vbase = a.v + b * a.ks[0] + hkv * a.ks[2];
    // ---- the first key tiles of the first run are requested right behind the Q rows ----------------------
    // A workgroup owns its compute unit alone (LDS, registers), so nothing hides its start-up: the Q rows come from
    // HBM (about 4 us on the loaded chip), and the first two key tiles another 2 us if they were only requested once
    // the Q rows are there.  Requested here they travel together.  Nothing else touches the LDS ring before the run's
    // own set-up in the loop below, which repeats this arithmetic and skips the requests.
    if constexpr (PIPELINED) {
        const int space = run_space[0], seg_begin = run_begin[0], seg_end = run_end[0];
        const int second = seg_end - seg_begin > BN ? 1 : 0;
        LaneOffsets<D> off;
        lane_offsets<D>(a, space, seg_begin, 0x7fffffff, wave, lane, aug_row(a, space, seg_begin), off);
        const int vt_stride = space == KSA_SPACE_TEXT ? a.nt_pad : a.ns_pad;
        lane_offsets_vt<D>(vt_stride, wave, lane, off);
        const __bf16 *vtbase = a.vt + (space == KSA_SPACE_TEXT ? 0 : a.vt_sum_off) +
                               ((int64_t)(b * a.n_kv_heads + hkv) * D) * vt_stride + seg_begin;
        const unsigned lds0 = (unsigned)(size_t)lds;
        const unsigned k_wave = lds0 + K0 + RW * wave * (D * 2), v_wave = lds0 + V0 + T::VROWS * wave * 128;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int tt = t == 0 ? 0 : second;
            const __bf16 *kg = kbase + (int64_t)aug_row(a, space, seg_begin + tt * BN) * a.ks[1], *vg = vtbase + tt * BN;
#pragma unroll
            for (int i = 0; i < T::NI; ++i) issue_tile_load_part<D>(kg, (unsigned)off.k[i] * 2u, k_wave + t * T::BYTES, i);
#pragma unroll
            for (int i = 0; i < T::NIV; ++i) issue_vt_load_part<D>(vg, (unsigned)off.vt[i] * 2u, v_wave + t * T::BYTES, i);
        }
    }

    // ---- the reference of the softmax -----------------------------------------------------------------
    // Online softmax needs a reference m_i per row with s_ij - m_i bounded above.  The usual choice is the running
    // row maximum (TRACK below: row maxima of every block, a raise of the reference with a rescale of the accumulators
    // when a block exceeds it).  Where it is provably safe the pipelined kernel fixes the reference up front instead:
    // |s_ij| = |q_i . k_j| <= |q_i| max_j |k_j| =: B_i (Cauchy-Schwarz; the largest K row norm of the KV head comes from
    // the preparation pass), so with m_i = B_i - 32 / (scale log2 e) every exponent (s_ij - m_i) scale log2 e is at
    // most 32, and at least 32 - 2 B_i scale log2 e.  If B_i scale log2 e <= 60 for every row of the wave, the exponents
    // lie in [-88, 32]: every weight is a normal number in bf16 and fp32, whatever the data, the fp32 sums of p and of
    // p v stay finite unless |v| times the number of keys exceeds 2^95 (2^119 with the running maximum), and a product
    // p v can only be lost to underflow where |v| < 2^-38 -- and there are no row maxima, no raise decision and no
    // rescale in the loop (3 - 4 % of the time of the 128K workload).  The result is the same softmax: the reference
    // cancels in O = sum(p v) / sum(p) and is added back in the log-sum-exp.  Waves whose bound is larger (keys or
    // queries of unusual size) or not a number take the tracking variant; both variants execute the same barriers,
    // so the waves of a workgroup may differ.
    float m_static[QB];
    bool static_ok = false;
    if constexpr (PIPELINED) {
        const float kmax2 = a.knorm[b * a.n_kv_heads + hkv];
        bool ok = true;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float n2 = 0.f;
#pragma unroll
            for (int s = 0; s < T::KS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) n2 = fmaf((float)qreg[qb][s][e], (float)qreg[qb][s][e], n2);
            n2 += other_half(n2);                                        // the lane pair of a row holds its two halves
            const float bound = __builtin_sqrtf(n2 * kmax2) * 1.002f;    // raw score units; the factor covers fp32 rounding
            ok &= bound * a.scale_log2e <= 60.f;                         // false for NaN
            m_static[qb] = bound - 32.f / a.scale_log2e;
        }
        static_ok = __builtin_amdgcn_ballot_w64(!ok) == 0;
    } else {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) m_static[qb] = 0.f;
    }

    // Everything from the accumulators to the stores, once per variant (two copies of the code that share nothing but
    // the prologue above: a choice inside the loops would join the variants with the accumulators live).
    auto body = [&](auto track_tag) {
    constexpr bool TRACK = decltype(track_tag)::value;
    // ---- accumulators -------------------------------------------------------------------------
    f32x16 oacc[QB][T::DB];
    RowState st;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        st.m_ref[qb] = TRACK ? -1e30f : m_static[qb];
        st.l_part[qb] = 0.f;
        st.l_sum[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int db = 0; db < T::DB; ++db)
#pragma unroll
            for (int g = 0; g < 16; ++g) oacc[qb][db][g] = 0.f;
    }

    // the A operand of sum_half(); opaque from here on: a value the compiler can see through would be re-materialised by
    // VALU moves right in front of the raw MFMAs that read it, and the compiler inserts no wait states for those
    const unsigned ind1 = (lane == 0 || lane == 32 || lane == 17 || lane == 49) ? 0x3f803f80u : 0u;
    u32x4 ind = {ind1, ind1, ind1, ind1};
    asm volatile("" : "+v"(ind));
    const float sl = a.scale_log2e;
    const float raise_margin = RESCALE_THRESHOLD_LOG2 / sl;   // the rescale threshold in raw score units

    for (int seg = 0; seg < n_seg; ++seg) {
        const int space = seg == 0 ? run_space[0] : run_space[1];
        const int seg_begin = seg == 0 ? run_begin[0] : run_begin[1], seg_end = seg == 0 ? run_end[0] : run_end[1];
        // tiles inside [full_lo, full_hi) are seen whole by every row of the query tile; the others are masked
        const int full_lo = seg == 0 ? run_full_lo[0] : run_full_lo[1], full_hi = seg == 0 ? run_full_hi[0] : run_full_hi[1];
        auto tile_masked = [&](int key0) { return !(key0 >= full_lo && key0 + BN <= full_hi); };
        const int n_tiles = (seg_end - seg_begin + BN - 1) / BN;
        // Are the lanes' row offsets the same for every tile of the run?  Yes when every tile starts at the same
        // phase of the chunk pattern (64 % period == 0), or never crosses a chunk (period % 64 == 0, aligned).
        const int period = space == KSA_SPACE_TEXT ? a.c : a.m;
        const bool invariant = (BN % period == 0) || (period % BN == 0 && seg_begin % BN == 0);
        LaneOffsets<D> off;
        if (invariant) lane_offsets<D>(a, space, seg_begin, 0x7fffffff, wave, lane, aug_row(a, space, seg_begin), off);

        // union of the visible ranges of the wave's rows in this index space: a masked tile outside it has nothing for
        // this wave
        const int wlo = space == KSA_SPACE_TEXT ? wlo_t : wlo_s, whi = space == KSA_SPACE_TEXT ? whi_t : whi_s;
        if constexpr (PIPELINED) {
            // (the scheduler guarantees: lane offsets invariant over the run, seg_begin % 16 == 0, and the run's last
            // tile ends inside its index space, so every row of every tile exists)
            // ================= pipelined loop over a run of tiles =======================================
            // The loop advances in sub-tiles of 32 keys (2t and 2t+1 for the halves of LDS tile t); see subtile().
            // The accumulators are only touched by VALU in the rare "raise the reference" block between sub-tiles.
            // LDS tile t lives in buffer t % 3; tile t+2 is requested right after the one barrier of tile t.
            // A MASKED run differs in one place: every score is clipped to its row's visible key range when it is
            // looked at for the row maximum.  (Every row of every tile exists: the run ends inside its index space.)
            auto tile_base = [&](int t) { return (int64_t)aug_row(a, space, seg_begin + t * BN) * a.ks[1]; };
            constexpr int HALF = 32 * (D * 2);   // byte offset of the second 32-key block of a tile
            // V comes from the key-major copy: rows of one (batch, KV head, index space), keys contiguous
            const int vt_stride = space == KSA_SPACE_TEXT ? a.nt_pad : a.ns_pad;
            const __bf16 *vtbase = a.vt + (space == KSA_SPACE_TEXT ? 0 : a.vt_sum_off) +
                                   ((int64_t)(b * a.n_kv_heads + hkv) * D) * vt_stride + seg_begin;
            lane_offsets_vt<D>(vt_stride, wave, lane, off);
            // the lane's byte offsets from the wave-uniform tile addresses, and the wave's share of an LDS buffer
            unsigned k_offb[T::NI], v_offb[T::NIV];
#pragma unroll
            for (int i = 0; i < T::NI; ++i) k_offb[i] = (unsigned)off.k[i] * 2u;
#pragma unroll
            for (int i = 0; i < T::NIV; ++i) v_offb[i] = (unsigned)off.vt[i] * 2u;
            const unsigned lds0 = (unsigned)(size_t)lds;
            const unsigned k_wave = lds0 + K0 + RW * wave * (D * 2), v_wave = lds0 + V0 + T::VROWS * wave * 128;
            auto issue_tile = [&](int t, int buf_off) {
                const __bf16 *kg = kbase + tile_base(t), *vg = vtbase + t * BN;
#pragma unroll
                for (int i = 0; i < T::NI; ++i) issue_tile_load_part<D>(kg, k_offb[i], k_wave + buf_off, i);
#pragma unroll
                for (int i = 0; i < T::NIV; ++i) issue_vt_load_part<D>(vg, v_offb[i], v_wave + buf_off, i);
            };
            // visible key range of each of the lane's rows inside this run: [lo, lo + span), lo stored minus 4 * h
            int vis_lo[QB], vis_span[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const int lo = max(space == KSA_SPACE_TEXT ? lo_t[qb] : lo_s[qb], seg_begin);
                const int hi = min(space == KSA_SPACE_TEXT ? hi_t[qb] : hi_s[qb], seg_end);
                vis_lo[qb] = lo - 4 * h;
                vis_span[qb] = max(hi - lo, 0);
            }
            // A run is up to three stretches of tiles: masked ones (a window edge), FULL ones, masked ones (the causal
            // diagonal, the summary edge).  The pipeline is filled once per run; a stretch is a loop over "produce the
            // scores of tile tn" = the second sub-tile of tile tn - 1 (scores of the first half of tile tn) followed by the
            // first sub-tile of tile tn (scores of its second half), instantiated with or without the clipping of those
            // scores.  (One loop with the choice made per tile costs register copies at every join of the two variants.)
            {
                const int second = n_tiles > 1 ? 1 : 0;
                if (seg > 0) {                       // (the first run's tiles were requested together with the Q rows)
                    __syncthreads();                 // earlier readers of the LDS buffers are done
                    issue_tile(0, 0);
                    issue_tile(second, T::BYTES);
                }
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
                f32x16 sv_a[QB], sv_b[QB];
                float mxl[QB];                       // the lane's maxima of the pending scores
                bool raise = false;
                qk_only<D>(lds, K0, ll, qreg, sv_a);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) scores_ready(sv_a[qb]);
                const bool first_masked = tile_masked(seg_begin);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if (first_masked) {
#pragma unroll
                        for (int g = 0; g < 16; ++g) {
                            const unsigned rel = (unsigned)(seg_begin - vis_lo[qb] + (8 * (g / 4) + g % 4));
                            sv_a[qb][g] = rel < (unsigned)vis_span[qb] ? sv_a[qb][g] : -INFINITY;
                        }
                    }
                    float mx = -INFINITY;
                    if constexpr (TRACK) {
#pragma unroll
                        for (int g = 0; g < 16; g += 2) mx = max3(mx, sv_a[qb][g], sv_a[qb][g + 1]);
                        raise |= mx > st.m_ref[qb] + raise_margin;
                    }
                    mxl[qb] = mx;
                }
                if (TRACK && seg == 0) {
                    // nothing has been accumulated yet, so the reference maximum simply starts at the first block's row
                    // maximum: no rescale of the (zero) accumulators and row sums.  A row that sees none of these keys
                    // keeps its start value and is raised by the first block it does see.
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        st.m_ref[qb] = fmaxf(st.m_ref[qb], fmaxf(mxl[qb], other_half(mxl[qb])));
                    raise = false;
                }
                if constexpr (TRACK) raise = __builtin_amdgcn_ballot_w64(raise) != 0;
                bf16x8 ka_pre[T::RING];
#pragma unroll
                for (int s = 0; s < T::RING; ++s) ka_pre[s] = read_k_operand<D>(lds, ll.k + K0 + HALF, s);
                int b_cur = 0, b_nxt = T::BYTES, b_ld = 2 * T::BYTES;   // buffer offsets of tiles tn, tn+1, tn+2
                TileSync<D> sync;
                sync.k_off = k_offb;
                sync.v_off = v_offb;
                sync.kg = kbase, sync.vg = vtbase, sync.k_dst = k_wave, sync.v_dst = v_wave;
                // does some row of this wave see a key of the tile that starts at key k0?
                auto wave_sees = [&](int k0) { return k0 < whi && k0 + BN > wlo; };
                // Global addresses of tile min(t, n_tiles - 1) for the request two tiles ahead (past the end of the run the
                // last tile is requested again, into a free buffer).  Runs whose tiles all start at the same phase of the
                // chunk pattern advance by a constant number of augmented rows per tile.
                // (straight-line scalar code on purpose: it is executed inside a sub-tile's MFMA slot, see subtile(); the
                // scheduler only marks items pipelined whose chunk length and summary count are powers of two, so the row
                // of a compact index is two shifts, a multiply and two adds)
                const int r_sh = space == KSA_SPACE_TEXT ? a.c_shift : a.m_shift;
                const int r_msk = period - 1, r_add = space == KSA_SPACE_TEXT ? 0 : a.c;
                auto aim = [&](int t) {
                    const int tt = t < n_tiles ? t : n_tiles - 1;
                    const int u = seg_begin + tt * BN;
                    const int row = (u >> r_sh) * a.w + (u & r_msk) + r_add;
                    sync.kg = kbase + (int64_t)row * a.ks[1];
                    sync.vg = vtbase + tt * BN;
                };
                auto stretch = [&](auto masked_tag, int tn_begin, int tn_end) {
                    constexpr bool MASKED = decltype(masked_tag)::value;
                    for (int tn = tn_begin; tn < tn_end; ++tn) {
                        const int key0 = seg_begin + tn * BN;
                        // what the first sub-tile of tile tn requests (tile tn + 2) and where it goes: b_ld after the
                        // rotation below, i.e. the buffer tile tn - 1 leaves
                        auto prepare_request = [&]() {
                            aim(tn + 2);
                            sync.k_dst = k_wave + (tn > 0 ? b_cur : b_ld);
                            sync.v_dst = v_wave + (tn > 0 ? b_cur : b_ld);
                        };
                        if (tn > 0) {
                            // ---- second sub-tile of tile tn-1: weights from sv_b, scores of the first half of tile tn into
                            // sv_a (for tn = n_tiles they come from a buffer that holds no new tile and are never used)
                            if (MASKED && !wave_sees(key0 - BN) && !wave_sees(key0)) {
                                idle_subtile<D, false>(lds, ll, sv_a, ka_pre, K0 + b_nxt + HALF, mxl, sync);
                                prepare_request();
                                raise = false;
                            } else {
                                if (TRACK && raise) raise_reference_pl<D>(st, mxl, oacc, sl);
                                raise = subtile<D, false, MASKED, TRACK>(lds, ll, qreg, sv_a, sv_b, ka_pre, K0 + b_nxt, V0 + b_cur,
                                                                  1, K0 + b_nxt + HALF, oacc, st, ind, sl, raise_margin, mxl,
                                                                  sync, key0, vis_lo, vis_span, prepare_request) &&
                                        (tn < n_tiles);
                            }
                            const int b_old = b_cur;
                            b_cur = b_nxt, b_nxt = b_ld, b_ld = b_old;
                        } else {
                            prepare_request();
                        }
                        if (tn < n_tiles) {
                            // (no wait for the loads of tile tn+1 here: they get until the barrier inside the sub-tile)
                            // ---- first sub-tile of tile tn: weights from sv_a, scores of its second half into sv_b ----
                            if (MASKED && !wave_sees(key0)) {
                                idle_subtile<D, true>(lds, ll, sv_b, ka_pre, K0 + b_nxt, mxl, sync);
                                raise = false;
                            } else {
                                if (TRACK && raise) raise_reference_pl<D>(st, mxl, oacc, sl);
                                raise = subtile<D, true, MASKED, TRACK>(lds, ll, qreg, sv_b, sv_a, ka_pre, K0 + b_cur + HALF,
                                                                 V0 + b_cur, 0, K0 + b_nxt, oacc, st, ind, sl, raise_margin,
                                                                 mxl, sync, key0 + 32, vis_lo, vis_span, [] {});
                            }
                        }
                    }
                };
                // tiles [f_lo, f_hi) of the run are FULL
                int f_lo = full_lo > seg_begin ? (full_lo - seg_begin + BN - 1) / BN : 0;
                int f_hi = full_hi > seg_begin ? (full_hi - seg_begin) / BN : 0;
                f_hi = min(f_hi, n_tiles);
                if (f_hi <= f_lo) f_lo = f_hi = 0;
                // index n_tiles (the last second sub-tile alone) goes with the last stretch
                if (f_lo > 0) stretch(std::true_type{}, 0, f_lo);
                if (f_hi > f_lo) stretch(std::false_type{}, f_lo, f_hi < n_tiles ? f_hi : n_tiles + 1);
                if (f_hi < n_tiles) stretch(std::true_type{}, f_hi, n_tiles + 1);
                // the request repeated for the last tile is still in flight: let it land before anyone reuses LDS
                __builtin_amdgcn_s_waitcnt(0x0F70);
                accumulators_settle<D>(oacc, st);
            }
        } else {
        // ================= plain loop: MASKED runs, short runs, odd chunk shapes ============================
        for (int kt = seg_begin; kt < seg_end; kt += BN) {
            const int t_lo = kt, t_hi = min(kt + BN, seg_end);
            // the wave has nothing visible in this tile (block-diagonal summary rows, window edges): skip the math
            const bool masked = tile_masked(kt);
            const bool active = !masked || (t_lo < whi && t_hi > wlo);
            const bool ragged = kt + BN > seg_end;
            const int base_aug = aug_row(a, space, kt);
            if (!invariant || ragged) lane_offsets<D>(a, space, kt, seg_end - 1, wave, lane, base_aug, off);
            __syncthreads();
            issue_tile_load<D>(kbase + (int64_t)base_aug * a.ks[1], off.k, lds, K0, wave);
            issue_tile_load<D>(vbase + (int64_t)base_aug * a.ks[1], off.v, lds, V0, wave);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (!active) continue;
            f32x16 sacc[QB][2];
            score_mfma<D>(lds, K0, ll, qreg, sacc);
            if (masked) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int lo = space == KSA_SPACE_TEXT ? lo_t[qb] : lo_s[qb];
                    const int hi = space == KSA_SPACE_TEXT ? hi_t[qb] : hi_s[qb];
                    const int elo = max(lo, seg_begin), ehi = min(hi, seg_end);
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int g = 0; g < 16; ++g) {
                            const int key = kt + kb * 32 + 8 * (g / 4) + 4 * h + (g % 4);
                            if (key < elo || key >= ehi) sacc[qb][kb][g] = -INFINITY;
                        }
                }
            }
            bf16x8 pb[QB][2][2];
            float tmax[QB];
            if (tile_max(sacc, st, sl, tmax)) raise_reference<D>(st, tmax, oacc, sl);
            exp_and_pack(sacc, pb, st, sl);
            pv_mfma<D>(lds, V0, ll, pb, oacc);
        }
        }
    }

    // ---- epilogue: O = O^T / l, LSE ---------------------------------------------------------------
    // The accumulators hold O transposed: a lane owns one query row and, per register group, four consecutive head-dim
    // values, so storing them directly would scatter 8-byte pieces over 32 rows per instruction.  Each wave instead
    // passes its 32-row blocks through a private LDS staging area (rows padded by 16 bytes against bank conflicts) and
    // writes whole rows: one store instruction covers 1 KiB of contiguous 16-byte pieces.  Only this wave touches the
    // area, and a wave's LDS accesses complete in order, so no barrier is needed.
    {
        constexpr int ROWB = T::STAGE_ROW;
        unsigned char *stg = lds + 6 * T::BYTES + wave * (32 * ROWB);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float l_row;
            if (PIPELINED) {   // lane j < 16 holds the sums of queries j (register 0) and j + 16 (register 1)
                const float s0 = __shfl(st.l_sum[qb][0], r & 15), s1 = __shfl(st.l_sum[qb][1], r & 15);
                l_row = (r & 16) ? s1 : s0;
            } else {
                l_row = st.l_part[qb] + other_half(st.l_part[qb]);
            }
            const float inv = 1.0f / l_row;   // rows past the end of the tile: never stored
#pragma unroll
            for (int db = 0; db < T::DB; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    bf16x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(oacc[qb][db][g4 * 4 + e] * inv);
                    *reinterpret_cast<bf16x4 *>(stg + r * ROWB + (db * 32 + g4 * 8 + h * 4) * 2) = pk;
                }
            const int row0 = q_begin + (wrow * QB + qb) * 32;
            // the lane's piece of row 0 of its (batch, head); a row's address is this plus augmented row x row stride.
            // The pipelined instantiation only sees chunk shapes that are powers of two (the scheduler's condition), so
            // the row map is two shifts and a multiply-add per store rather than the general map with its divisions
            // (60 instructions per store, 16 stores per wave, with the matrix pipe idle).
            const int piece = lane % T::CH;
            __bf16 *const obase = a.o + b * a.os[0] + hq * a.os[2] + piece * 8;
            const int e_sh = q_space == KSA_SPACE_TEXT ? a.c_shift : a.m_shift;
            const int e_msk = (q_space == KSA_SPACE_TEXT ? a.c : a.m) - 1, e_add = q_space == KSA_SPACE_TEXT ? 0 : a.c;
#pragma unroll
            for (int i = 0; i < 32 / T::RPI; ++i) {
                const int row = T::RPI * i + lane / T::CH;
                const u32x4 x = *reinterpret_cast<const u32x4 *>(stg + row * ROWB + piece * 16);
                const int idx = row0 + row;
                if (idx < q_end) {
                    const int arow = PIPELINED ? (idx >> e_sh) * a.w + (idx & e_msk) + e_add : aug_row(a, q_space, idx);
                    *reinterpret_cast<u32x4 *>(obase + (int64_t)arow * a.os[1]) = x;
                }
            }
            if (a.lse && h == 0 && q_valid[qb]) {
                // log-sum-exp = (m_ref scale log2 e + log2 l) ln 2 with l = f 2^e split first.  With the fixed reference
                // the two terms are large and of opposite sign (a row of 10^5 keys: -12 and +29 in the exponent
                // domain, Q = 0: -32 and +49), and adding them as they are would cost two or three bits; m_ref scale
                // log2 e is the rounded product the weights were computed with.
                float msl = st.m_ref[qb] * sl;
                asm volatile("" : "+v"(msl));   // (not contracted with the sum below)
                const float t = msl + (float)__builtin_amdgcn_frexp_expf(l_row);
                a.lse[((int64_t)b * a.n_q_heads + hq) * a.aug_len + q_aug[qb]] =
                    fmaf(t, 0.6931471805599453f, __logf(__builtin_amdgcn_frexp_mantf(l_row)));
            }
        }
    }
    };
    if constexpr (PIPELINED) {
        if (static_ok)
            body(std::false_type{});
        else
            body(std::true_type{});
    } else {
        body(std::true_type{});
    }
}

// Key-major copy of V for the pipelined loop.  The P V MFMA wants, per lane, eight keys of one head-dim column; V is
// stored the other way round (a key's head-dim values are contiguous), and the transposing LDS read that bridges the
// two runs at half the rate of a plain 16-byte read.  This pass therefore writes, per (batch, KV head, index space),
//   vt[d][64 * t + 8 * pc + e] = V[key 64 * t + 32 * sb + 16 * hf + 8 * (e / 4) + 4 * h + e % 4][d],
//   pc = 4 * sb + 2 * hf + h,
// i.e. rows of keys in the compact index space, each run of eight keys ordered the way the score MFMA leaves the
// weights in a lane's registers (lane half h of the 16-key group hf of the 32-key block sb), so that one 16-byte
// piece is exactly one lane's operand.  One workgroup transposes one 64-key tile through LDS; keys past the end of
// the space are written as zeros.
template <int D>
__global__ __launch_bounds__(256) void ksa_vt_kernel(const PrefillArgs a, int tiles_text) {
    constexpr int CH = D / 8;
    __shared__ __attribute__((aligned(16))) unsigned short raw[64][D + 8];
    typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
    const int b = blockIdx.z, hkv = blockIdx.y, tid = threadIdx.x;
    int t = blockIdx.x, space = KSA_SPACE_TEXT;
    if (t >= tiles_text) t -= tiles_text, space = KSA_SPACE_SUMMARY;
    const int n_space = space == KSA_SPACE_TEXT ? a.n_text : a.n_sum;
    const int stride = space == KSA_SPACE_TEXT ? a.nt_pad : a.ns_pad;
    const int k0 = t * 64;
    const __bf16 *vb = a.v + b * a.ks[0] + hkv * a.ks[2];
    for (int idx = tid; idx < 64 * CH; idx += 256) {
        const int row = idx / CH, ch = idx % CH;
        u16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
        if (k0 + row < n_space)
            x = *reinterpret_cast<const u16x8 *>(vb + (int64_t)aug_row(a, space, k0 + row) * a.ks[1] + ch * 8);
        *reinterpret_cast<u16x8 *>(&raw[row][ch * 8]) = x;
    }
    __syncthreads();
    __bf16 *out = const_cast<__bf16 *>(a.vt) + (space == KSA_SPACE_TEXT ? 0 : a.vt_sum_off) +
                  ((int64_t)(b * a.n_kv_heads + hkv) * D) * stride + k0;
    for (int idx = tid; idx < D * 8; idx += 256) {
        const int d = idx >> 3, pc = idx & 7;
        const int first = 32 * (pc >> 2) + 16 * ((pc >> 1) & 1) + 4 * (pc & 1);
        u16x8 x;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = raw[first + 8 * (e / 4) + e % 4][d];
        *reinterpret_cast<u16x8 *>(out + (int64_t)d * stride + 8 * pc) = x;
    }
    // The same pass takes the largest squared row norm of the tile's K rows (for the attention kernel's static softmax
    // reference): one value per (batch, KV head, tile), reduced per (batch, KV head) by ksa_knorm_reduce_kernel.
    {
        __shared__ float wave_best[4];
        const __bf16 *kb = a.k + b * a.ks[0] + hkv * a.ks[2];
        float best = 0.f;
        for (int idx = tid; idx < 64 * CH; idx += 256) {
            const int row = idx / CH, ch = idx % CH;
            float s2 = 0.f;
            if (k0 + row < n_space) {
                const bf16x8 x = *reinterpret_cast<const bf16x8 *>(kb + (int64_t)aug_row(a, space, k0 + row) * a.ks[1] + ch * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) s2 = fmaf((float)x[e], (float)x[e], s2);
            }
#pragma unroll
            for (int dd = CH / 2; dd > 0; dd >>= 1) s2 += __shfl_xor(s2, dd);   // the CH lanes of a row are neighbours
            best = fmaxf(best, s2);
        }
#pragma unroll
        for (int dd = 32; dd > 0; dd >>= 1) best = fmaxf(best, __shfl_xor(best, dd));
        if ((tid & 63) == 0) wave_best[tid >> 6] = best;
        __syncthreads();
        if (tid == 0)
            a.knorm_tiles[((int64_t)(b * a.n_kv_heads + hkv)) * gridDim.x + blockIdx.x] =
                fmaxf(fmaxf(wave_best[0], wave_best[1]), fmaxf(wave_best[2], wave_best[3]));
    }
}

// knorm[(batch, KV head)] = max over that head's tiles of knorm_tiles.  A NaN anywhere gives NaN (which sends the
// attention kernel to its tracking variant).
__global__ __launch_bounds__(256) void ksa_knorm_reduce_kernel(const float *tiles, float *out, int n_tiles) {
    __shared__ float wave_best[4];
    const float *src = tiles + (int64_t)blockIdx.x * n_tiles;
    float best = 0.f;
    bool bad = false;
    for (int i = threadIdx.x; i < n_tiles; i += 256) {
        const float x = src[i];
        bad |= !(x == x);
        best = fmaxf(best, x);
    }
    if (bad) best = __builtin_nanf("");
#pragma unroll
    for (int dd = 32; dd > 0; dd >>= 1) {
        const float o = __shfl_xor(best, dd);
        best = (best != best || o != o) ? __builtin_nanf("") : fmaxf(best, o);
    }
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = wave_best[0];
        for (int w = 1; w < 4; ++w) r = (r != r || wave_best[w] != wave_best[w]) ? __builtin_nanf("") : fmaxf(r, wave_best[w]);
        out[blockIdx.x] = r;
    }
}

}  // namespace

namespace {
// workspace: [key-major copy of V][largest squared K row norm per (batch, KV head, 64-key tile)][... per (batch, KV head)]
int64_t vt_bytes(const ksa_params &p) {
    const int64_t n_sum = (int64_t)(p.n_text / p.chunk_len) * p.n_summary;
    const int64_t keys = (p.n_text + 63) / 64 * 64 + (n_sum + 63) / 64 * 64;
    return (int64_t)p.batch * p.n_kv_heads * p.head_dim * keys * 2;   // a multiple of 128 * head_dim bytes
}
int64_t key_tiles(const ksa_params &p) {
    const int64_t n_sum = (int64_t)(p.n_text / p.chunk_len) * p.n_summary;
    return (p.n_text + 63) / 64 + (n_sum + 63) / 64;
}
}  // namespace

size_t ksa_prefill_workspace_size(const ksa_params &p) {
    const int64_t heads = (int64_t)p.batch * p.n_kv_heads;
    return (size_t)(vt_bytes(p) + (heads * key_tiles(p) + heads) * (int64_t)sizeof(float));
}


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
    a.stack = L.head_stack;
    a.stack_shift = log2_exact(L.head_stack);
    if (a.stack_shift < 0 || L.head_stack > KSA_MAX_HEAD_STACK || a.group % L.head_stack != 0) return KSA_ERR_INVALID_ARG;
    a.n_q_heads = L.p.n_q_heads;
    a.self_only = (L.p.flags & KSA_FLAG_SUMMARY_SELF_ONLY) ? 1 : 0;
    a.aug_len = L.aug_len;
    a.scale = L.p.softmax_scale;
    a.scale_log2e = L.p.softmax_scale * 1.4426950408889634f;
    a.n_kv_heads = L.p.n_kv_heads;
    a.n_text = L.p.n_text;
    a.n_sum = (L.p.n_text / L.p.chunk_len) * L.p.n_summary;
    a.nt_pad = (a.n_text + 63) / 64 * 64;
    a.ns_pad = (a.n_sum + 63) / 64 * 64;
    a.vt = static_cast<const __bf16 *>(L.workspace);
    a.knorm_tiles = reinterpret_cast<float *>(static_cast<unsigned char *>(L.workspace) + vt_bytes(L.p));
    a.knorm = a.knorm_tiles + (int64_t)L.p.batch * L.p.n_kv_heads * key_tiles(L.p);
    a.vt_sum_off = (int64_t)L.p.batch * L.p.n_kv_heads * L.p.head_dim * a.nt_pad;
    if (!L.workspace || L.workspace_bytes < ksa_prefill_workspace_size(L.p)) return KSA_ERR_WORKSPACE_TOO_SMALL;
    if (L.n_entries <= 0) return KSA_OK;
    // lane offsets inside one tile are 32-bit element offsets: a tile of 64 rows of one index space spans at
    // most (64 / period + 2) chunks of the augmented sequence
    {
        const int64_t period = a.m > 0 && a.m < a.c ? a.m : a.c;
        if (L.kv_strides[1] * ((BN / period + 2) * (int64_t)a.w) >= ((int64_t)1 << 31)) return KSA_ERR_UNSUPPORTED;
        // ... and so are the ones into the key-major copy of V (head_dim rows of nt_pad or ns_pad keys)
        if ((int64_t)L.p.head_dim * (a.nt_pad > a.ns_pad ? a.nt_pad : a.ns_pad) >= ((int64_t)1 << 31)) return KSA_ERR_UNSUPPORTED;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (L.phases & 1) {
        const int tiles_text = a.nt_pad / 64, tiles_sum = a.ns_pad / 64;
        const dim3 grid(tiles_text + tiles_sum, L.p.n_kv_heads, L.p.batch);
        if (L.p.head_dim == 128)
            hipLaunchKernelGGL(ksa_vt_kernel<128>, grid, dim3(256), 0, st, a, tiles_text);
        else if (L.p.head_dim == 64)
            hipLaunchKernelGGL(ksa_vt_kernel<64>, grid, dim3(256), 0, st, a, tiles_text);
        else
            return KSA_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(ksa_knorm_reduce_kernel, dim3(L.p.batch * L.p.n_kv_heads), dim3(256), 0, st, a.knorm_tiles, a.knorm,
                           tiles_text + tiles_sum);
        if (hipGetLastError() != hipSuccess) return KSA_ERR_HIP;
    }
    if (!(L.phases & 2)) return KSA_OK;
    // the pipelined items' workgroups first, then those of the remaining items: one launch each
    const dim3 block(NW * 64), grid_p(L.n_pipelined_entries), grid_g(L.n_entries - L.n_pipelined_entries);
    PrefillArgs g = a;
    g.entries = a.entries + L.n_pipelined_entries;
    if (L.p.head_dim == 128) {
        if (grid_p.x > 0) hipLaunchKernelGGL((ksa_prefill_kernel<128, true>), grid_p, block, 0, st, a);
        if (grid_g.x > 0) hipLaunchKernelGGL((ksa_prefill_kernel<128, false>), grid_g, block, 0, st, g);
    } else if (L.p.head_dim == 64) {
        if (grid_p.x > 0) hipLaunchKernelGGL((ksa_prefill_kernel<64, true>), grid_p, block, 0, st, a);
        if (grid_g.x > 0) hipLaunchKernelGGL((ksa_prefill_kernel<64, false>), grid_g, block, 0, st, g);
    } else {
        return KSA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? KSA_OK : KSA_ERR_HIP;
}
