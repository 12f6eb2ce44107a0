// Measurement probes for bench.py (libksa_probe.so; not part of libksa): what one MI355X sustains on the two resources
// the KSA kernels are bound by, measured on the same box and in the same process as the kernels themselves.
//   ksa_probe_mfma  a loop of nothing but v_mfma_f32_32x32x16_bf16 (the instruction of the prefill kernel) on every
//                   SIMD of the chip, operands N(0,1)-like bf16 values that differ per lane: the "achievable" matrix
//                   rate under the board's power management, and the core clock it settles at;
//   ksa_probe_read  a streaming read of a caller buffer with the decode kernel's access pattern (16 bytes per lane,
//                   non-temporal): the "achievable" HBM read bandwidth.
// Both synchronise the device and time with HIP events; they are probes, not kernels of the hot path.
#include <hip/hip_runtime.h>

#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int CHAINS = 8;   // independent accumulators per wave: 8 x 16 registers

// Every wave runs `iters` rounds of CHAINS MFMAs (one per accumulator).  operands: 16 bytes per (lane, operand).
__global__ __launch_bounds__(512) void mfma_loop_kernel(const u32x4 *operands, int iters, float *sink, long long *clocks) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    const bf16x8 a = __builtin_bit_cast(bf16x8, operands[2 * (tid & 4095)]);
    const bf16x8 b = __builtin_bit_cast(bf16x8, operands[2 * (tid & 4095) + 1]);
    f32x16 c[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; ++i)
#pragma unroll
        for (int g = 0; g < 16; ++g) c[i][g] = 0.f;
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < CHAINS; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < CHAINS; ++i)
#pragma unroll
        for (int g = 0; g < 16; ++g) s += c[i][g];
    if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; practically never true
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = t1 - t0;       // shader clock cycles
        clocks[2 * blockIdx.x + 1] = w1 - w0;   // ticks of the constant 100 MHz counter
    }
}

// Every workgroup streams one contiguous span (as a decode workgroup does), eight 16-byte loads in flight per lane.
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *src, long long n_vec, unsigned *sink) {
    const long long per = (n_vec + gridDim.x - 1) / gridDim.x;
    const long long lo = per * blockIdx.x, hi = lo + per < n_vec ? lo + per : n_vec;
    unsigned acc = 0;
    long long i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        u32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u][0] ^ x[u][1] ^ x[u][2] ^ x[u][3];
    }
    for (; i < hi; i += 256) {
        const u32x4 x = __builtin_nontemporal_load(src + i);
        acc ^= x[0] ^ x[1] ^ x[2] ^ x[3];
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;
}

}  // namespace

extern "C" {

// Runs the MFMA loop on `blocks` workgroups of 256 * waves_per_simd threads (blocks = 0: one per compute unit) for
// `iters` rounds, `repeats` launches back to back after one warm-up launch.  Returns 0 and writes the sustained rate
// in TFLOP/s (bf16, dense) and the mean core clock in MHz over the timed launches; negative on a HIP error.
int ksa_probe_mfma(int blocks, int waves_per_simd, int iters, int repeats, float *tflops, float *core_mhz) {
    if (!tflops || !core_mhz || iters <= 0 || repeats <= 0 || (waves_per_simd != 1 && waves_per_simd != 2)) return -1;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -4;
    if (blocks <= 0) blocks = prop.multiProcessorCount;
    const int threads = 256 * waves_per_simd;
    // operand pool: 4096 lanes x 2 operands x 16 bytes of bf16 values of magnitude 0.25 .. 4, a fixed pseudo-random pattern
    const int n_words = 4096 * 2 * 4;
    unsigned *h = new unsigned[n_words];
    unsigned x = 0x12345u;
    for (int i = 0; i < n_words; ++i) {
        unsigned w = 0;
        for (int half = 0; half < 2; ++half) {
            x = x * 1664525u + 1013904223u;
            // sign, exponent 125 .. 128 (magnitudes 0.25 .. 4), seven random mantissa bits
            const unsigned sign = (x >> 31) << 15, expo = (125u + ((x >> 20) & 3u)) << 7, mant = (x >> 8) & 0x7fu;
            w |= (sign | expo | mant) << (16 * half);
        }
        h[i] = w;
    }
    u32x4 *d_op = nullptr;
    float *d_sink = nullptr;
    long long *d_clk = nullptr;
    int rc = 0;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipMalloc(&d_op, n_words * 4) != hipSuccess || hipMalloc(&d_sink, 64) != hipSuccess ||
        hipMalloc(&d_clk, sizeof(long long) * 2 * blocks) != hipSuccess ||
        hipMemcpy(d_op, h, n_words * 4, hipMemcpyHostToDevice) != hipSuccess || hipEventCreate(&e0) != hipSuccess ||
        hipEventCreate(&e1) != hipSuccess)
        rc = -4;
    if (rc == 0) {
        hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(threads), 0, nullptr, d_op, iters, d_sink, d_clk);
        (void)hipEventRecord(e0, nullptr);
        for (int r = 0; r < repeats; ++r)
            hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(threads), 0, nullptr, d_op, iters, d_sink, d_clk);
        (void)hipEventRecord(e1, nullptr);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) {
            rc = -4;
        } else {
            const double flops = (double)blocks * (threads / 64) * (double)iters * CHAINS * 32768.0 * repeats;
            *tflops = (float)(flops / (ms * 1e-3) / 1e12);
            long long *hc = new long long[2 * blocks];
            if (hipMemcpy(hc, d_clk, sizeof(long long) * 2 * blocks, hipMemcpyDeviceToHost) == hipSuccess) {
                double cyc = 0, wall = 0;
                for (int i = 0; i < blocks; ++i) cyc += (double)hc[2 * i], wall += (double)hc[2 * i + 1];
                *core_mhz = wall > 0 ? (float)(cyc / wall * 100.0) : 0.f;
            } else {
                rc = -4;
            }
            delete[] hc;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(d_op), (void)hipFree(d_sink), (void)hipFree(d_clk);
    delete[] h;
    return rc;
}

// Streams `bytes` (a multiple of 16) from the device buffer `src` `repeats` times after one warm-up pass and writes
// the read bandwidth in GB/s.  The buffer should be larger than the chip's last-level cache (256 MB).
int ksa_probe_read(const void *src, long long bytes, int repeats, float *gbs) {
    if (!src || !gbs || bytes < 16 || bytes % 16 != 0 || repeats <= 0) return -1;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -4;
    unsigned *d_sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = 0;
    if (hipMalloc(&d_sink, 64) != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = -4;
    if (rc == 0) {
        const dim3 grid(prop.multiProcessorCount * 6), block(256);
        const u32x4 *p = static_cast<const u32x4 *>(src);
        hipLaunchKernelGGL(read_kernel, grid, block, 0, nullptr, p, bytes / 16, d_sink);
        (void)hipEventRecord(e0, nullptr);
        for (int r = 0; r < repeats; ++r) hipLaunchKernelGGL(read_kernel, grid, block, 0, nullptr, p, bytes / 16, d_sink);
        (void)hipEventRecord(e1, nullptr);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
            rc = -4;
        else
            *gbs = (float)((double)bytes * repeats / (ms * 1e-3) / 1e9);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(d_sink);
    return rc;
}

}  // extern "C"
