// Calibration kernels for the benchmark (libpp_calib.so; not part of libpp's C ABI):
// the integer vector rate the chip sustains on the instruction mix of the partition DP's inner
// loop, at a chosen number of resident waves per SIMD, and a plain copy of known size that the
// HBM traffic counters are scaled by.
#include <hip/hip_runtime.h>
#include <stdint.h>

// Every wave runs `iters` trips of 8 rounds of 16 v_max_i32 and 8 v_min3_i32 on independent
// registers (the mix of the tiled DP kernel: one max and half a three-operand min per (cell,
// split) pair): 192 vector instructions per trip, written as inline assembly so that the count
// is exact.
__global__ __launch_bounds__(256) void k_calib_valu(int *out, int iters, int seed) {
    int x[8], g[4], t[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0x7fffffff - seed * (i + 1) - (int)threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) g[i] = seed * (i + 3) + (int)threadIdx.x;
    for (int it = 0; it < iters; ++it) {
        // 8 rounds per trip through the loop, so that the branch does not weigh (the DP's rows
        // are straight-line code of a few hundred instructions as well)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                asm volatile("v_max_i32 %0, %1, %2" : "=v"(t[i]) : "v"(g[i & 3]), "v"(x[(i + 1) & 7]));
#pragma unroll
            for (int i = 0; i < 8; ++i)
                asm volatile("v_min3_i32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(t[2 * i]), "v"(t[2 * i + 1]));
        }
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s ^= x[i];
    if (s == 0x12345678) out[0] = s;  // keeps the arithmetic alive; practically never true
}

__global__ __launch_bounds__(256) void k_calib_copy(const int4 *src, int4 *dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

extern "C" {

// Vector instructions one wave issues per trip through the loop of k_calib_valu.
int pp_calib_valu_insts_per_iter(void) { return 192; }

// Enqueues k_calib_valu with `blocks` workgroups of 256 threads (4 waves: one per SIMD of a
// compute unit, so blocks = compute units * k keeps k waves per SIMD resident).  out: one
// int32 of device memory.  Returns 0 or the HIP error code.
int pp_calib_valu(int blocks, int iters, int seed, int32_t *out, void *stream) {
    hipLaunchKernelGGL(k_calib_valu, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters, seed);
    return (int)hipGetLastError();
}

// Enqueues a copy of `bytes` (a multiple of 16) from src to dst (device pointers).
int pp_calib_copy(const void *src, void *dst, size_t bytes, void *stream) {
    hipLaunchKernelGGL(k_calib_copy, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const int4 *)src,
                       (int4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}

int pp_calib_compute_units(void) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

int pp_calib_clock_khz(void) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) return 0;
    return khz;
}
}
