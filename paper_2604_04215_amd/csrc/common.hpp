// Shared host/device helpers of libdlm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "dlm.h"

namespace dlm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int WAVE = 64;

// ---- error reporting (host) -------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);
int check_hip(hipError_t e, const char* what);

int lm_set_variant(int v);   // lmhead.hip
int lm_set_block(int v);     // lmhead.hip
int lm_set_nt(int v);        // lmhead.hip
int lm_set_cus(int v);       // lmhead.hip
int copy_set_unroll(int v);  // commit.hip
extern int g_attn_remap;     // attn.hip: bit 0 forward + dQ, bit 1 longest key range first, bit 2 dK / dV passes

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- XCD-aware 1-D grids ------------------------------------------------------
// Workgroups go round-robin to the 8 XCDs, each with an L2 of its own.  Workgroups that read the same operands (the
// nx tiles of one (sequence, KV head) "group") are given consecutive slots of ONE XCD, so those operands come from
// HBM once and every other tile hits that L2.  When the group count is not a multiple of 8 each group's tiles are
// dealt to sp XCDs (interleaved, so the parts do equal work under a causal mask) and no XCD idles.
struct GridRemap {
    int nx;    // tiles per group; 0 = plain 3-D grid (tile, KV head, sequence)
    int sp;    // XCDs a group is dealt to
    int nxp;   // tiles per part = ceil(nx / sp)
    int rev;   // 1: tiles are handed out last to first (longest key range first under a causal mask)
};
inline GridRemap no_remap() { return GridRemap{0, 1, 1, 0}; }
// returns the 1-D grid size, 0 when it does not fit a launch
inline int64_t set_remap(GridRemap& m, int64_t n_groups, int nx, bool rev) {
    int gcd8 = 8;
    while (n_groups % gcd8) gcd8 >>= 1;
    const int sp = 8 / gcd8 < nx ? 8 / gcd8 : nx;
    m.nx = nx;
    m.sp = sp;
    m.nxp = (nx + sp - 1) / sp;
    m.rev = rev ? 1 : 0;
    const int64_t n_wg = (n_groups * sp + 7) / 8 * 8 * m.nxp;
    return n_wg <= 0x7fffffff ? n_wg : 0;
}

// ---- device helpers ---------------------------------------------------------
// fp32 -> bf16, round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    union { bf16x2_t v; uint32_t u; } x;
    x.v[0] = (__bf16)lo;
    x.v[1] = (__bf16)hi;
    return x.u;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// raw v_exp_f32: exp2(-inf) = 0, no denormal range fix-up (results below 2^-126 flush to 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// decodes blockIdx.x of a remapped grid; false: this workgroup has no tile
__device__ __forceinline__ bool remap_decode(const GridRemap& m, int n_groups, int& grp, int& bx) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int sq = slot / m.nxp;
    const int vg = xcd + 8 * sq;
    grp = vg / m.sp;
    bx = (slot - sq * m.nxp) * m.sp + (vg - grp * m.sp);
    if (grp >= n_groups || bx >= m.nx) return false;
    if (m.rev) bx = m.nx - 1 - bx;
    return true;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

template <typename T>
__device__ __forceinline__ T shfl_xor(T v, int m) { return __shfl_xor(v, m, WAVE); }

}  // namespace dlm
