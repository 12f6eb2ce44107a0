// Device-side pieces shared by the prefill forward and backward kernels: vector types, the row maps of the
// augmented sequence and the global -> LDS load.  Header-only, included by .hip files.
#ifndef KSA_DEVICE_H_
#define KSA_DEVICE_H_

#include <hip/hip_runtime.h>

#include "ksa.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T) __attribute__((address_space(3))) T *

__device__ __forceinline__ int div_by(int x, int d, int shift) { return shift >= 0 ? (x >> shift) : (x / d); }

// Augmented row (Eq. 1) of compact text index / summary ordinal idx.  Args carries c, m, w = c + m and the
// shifts c_shift, m_shift (log2 when a power of two, else -1).
template <class Args>
__device__ __forceinline__ int aug_row(const Args &a, int space, int idx) {
    if (space == KSA_SPACE_TEXT) {
        const int j = div_by(idx, a.c, a.c_shift);
        return j * a.w + (idx - j * a.c);
    }
    const int j = div_by(idx, a.m, a.m_shift);
    return j * a.w + a.c + (idx - j * a.m);
}

// global -> LDS without VGPR staging: every lane fetches 16 bytes from its own global address and the wave's 64
// pieces land back to back (lane order) from the wave-uniform LDS address `dst`.
// Written as inline assembly on purpose: for the builtin the compiler assumes that any later LDS read may alias the
// data in flight and puts s_waitcnt vmcnt(0) in front of it, which serialises the loads with the MFMA work they are
// meant to overlap.  Here the waits are explicit (s_waitcnt before the workgroup barrier that publishes a tile).
// M0 carries the LDS address; no other code of these kernels uses M0.
__device__ __forceinline__ void lds_direct_load_16(const __bf16 *src, const unsigned char *dst) {
    const unsigned lds_addr = __builtin_amdgcn_readfirstlane((unsigned)(size_t)dst);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory");
}

// lds_direct_load_16() with a wave-uniform base address in scalar registers plus a per-lane unsigned byte offset:
// nothing but the load itself goes through the vector issue port.
__device__ __forceinline__ void lds_direct_load_16_s(const __bf16 *sbase, unsigned voff_bytes, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff_bytes), "s"(sbase), "s"(lds_addr)
                 : "memory");
}

inline int log2_exact(int x) {
    if (x <= 0 || (x & (x - 1))) return -1;
    int s = 0;
    while ((1 << s) < x) ++s;
    return s;
}

}  // namespace

#endif
