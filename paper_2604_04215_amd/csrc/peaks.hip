// libdlm_peaks: achievable-peak micro-benchmarks (device copy, one-pass read, register-only MFMA loop).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlm_peaks.h"

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <int NT>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const u32x4 v = (NT & 1) ? __builtin_nontemporal_load(src + i) : src[i];
    if (NT & 2) __builtin_nontemporal_store(v, dst + i);
    else dst[i] = v;
}

template <bool NT>
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const size_t i = base + q * 256;
        const size_t ic = i < n16 ? i : n16 - 1;     // clamped: the loads stay unconditional
        v[q] = NT ? __builtin_nontemporal_load(src + ic) : src[ic];
    }
    uint32_t x = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) x ^= v[q][0] ^ v[q][1] ^ v[q][2] ^ v[q][3];
    // one word per workgroup, from a lane chosen by the data: the loads cannot be dropped
    if (threadIdx.x == (x & 255u)) sink[blockIdx.x] = x;
}

__global__ __launch_bounds__(256) void mfma_kernel(int iters, const u32x4* __restrict__ operands, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[8], b[8];
    if (operands) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            union { u32x4 u; bf16x8 v; } x, y;
            x.u = operands[(2 * k) * 64 + lane];
            y.u = operands[(2 * k + 1) * 64 + lane];
            a[k] = x.v;
            b[k] = y.v;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                a[k][i] = (__bf16)(0.001f * (float)((lane + i + k) & 7));
                b[k][i] = (__bf16)(0.002f * (float)((lane * 3 + i + k) & 7));
            }
    }
    f32x16 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[k][i] = 0.f;
    for (int it = 0; it < iters; it += 8) {      // iters is a multiple of 8: every register index below is a constant
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[(k + u) & 7], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[k][i];
    if (lane == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
}

template <int MODE>
__global__ __launch_bounds__(512) void overlap_kernel(int iters, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.01f * (float)((lane + i) & 7));
        b[i] = (__bf16)(0.02f * (float)((lane * 3 + i) & 7));
    }
    f32x16 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[k][i] = 0.f;
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(lane + i);
    const bool do_m = MODE == 0 || (MODE == 2 && w < 4);
    const bool do_v = MODE == 1 || (MODE == 2 && w >= 4);
    for (int it = 0; it < iters; ++it) {
        if (MODE == 3) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) x[4 * k + i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[4 * k + i], 0.5f, -1.0f));
            }
        } else {
            if (do_m) {
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
            }
            if (do_v) {
#pragma unroll
                for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], 0.5f, -1.0f));
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[k][i];
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
    if (lane == 0) sink[blockIdx.x * 8 + w] = s;
}

int launched() { return hipGetLastError() == hipSuccess ? 0 : -4; }
bool ok16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int dlm_peak_copy(const void* src, void* dst, size_t bytes, int nt, void* stream) {
    if (!ok16(src) || !ok16(dst) || bytes == 0 || bytes % 16 || nt < 0 || nt > 3) return -1;
    const size_t n16 = bytes / 16, n_wg = (n16 + 255) / 256;
    if (n_wg > 0x7fffffffu) return -1;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)n_wg), blk(256);
    const u32x4* s = (const u32x4*)src;
    u32x4* d = (u32x4*)dst;
    switch (nt) {
        case 0: hipLaunchKernelGGL(copy_kernel<0>, grid, blk, 0, st, s, d, n16); break;
        case 1: hipLaunchKernelGGL(copy_kernel<1>, grid, blk, 0, st, s, d, n16); break;
        case 2: hipLaunchKernelGGL(copy_kernel<2>, grid, blk, 0, st, s, d, n16); break;
        default: hipLaunchKernelGGL(copy_kernel<3>, grid, blk, 0, st, s, d, n16); break;
    }
    return launched();
}

extern "C" int dlm_peak_read(const void* src, size_t bytes, int nt, uint32_t* sink, void* stream) {
    if (!ok16(src) || !sink || bytes == 0 || bytes % 16) return -1;
    const size_t n16 = bytes / 16, n_wg = (n16 + 1023) / 1024;
    if (n_wg > 0x7fffffffu) return -1;
    hipStream_t st = (hipStream_t)stream;
    if (nt) hipLaunchKernelGGL(read_kernel<true>, dim3((unsigned)n_wg), dim3(256), 0, st, (const u32x4*)src, n16, sink);
    else hipLaunchKernelGGL(read_kernel<false>, dim3((unsigned)n_wg), dim3(256), 0, st, (const u32x4*)src, n16, sink);
    return launched();
}

extern "C" int dlm_peak_mfma(int n_wg, int iters, const void* operands, float* sink, void* stream) {
    if (n_wg <= 0 || iters <= 0 || iters % 8 || !sink || (operands && !ok16(operands))) return -1;
    hipLaunchKernelGGL(mfma_kernel, dim3((unsigned)n_wg), dim3(256), 0, (hipStream_t)stream, iters, (const u32x4*)operands, sink);
    return launched();
}

extern "C" int dlm_peak_overlap(int mode, int n_wg, int iters, float* sink, void* stream) {
    if (mode < 0 || mode > 3 || n_wg <= 0 || iters <= 0 || !sink) return -1;
    const dim3 grid((unsigned)n_wg), blk(512);
    hipStream_t st = (hipStream_t)stream;
    switch (mode) {
        case 0: hipLaunchKernelGGL(overlap_kernel<0>, grid, blk, 0, st, iters, sink); break;
        case 1: hipLaunchKernelGGL(overlap_kernel<1>, grid, blk, 0, st, iters, sink); break;
        case 2: hipLaunchKernelGGL(overlap_kernel<2>, grid, blk, 0, st, iters, sink); break;
        default: hipLaunchKernelGGL(overlap_kernel<3>, grid, blk, 0, st, iters, sink); break;
    }
    return launched();
}
