// dlm_lmhead_confidence: fused hidden x W_vocab^T with online max / arg-max /
// runner-up / sum-of-exp per row, so the [M, V] logits never leave the chip.
//
// Work decomposition (gfx950, MFMA 32x32x16 bf16):
//   * The product is computed transposed, Z^T = W H^T: vocabulary rows are the MFMA
//     A operand (matrix rows), hidden rows the B operand (matrix columns).  A lane then
//     holds 16 vocabulary entries of ONE hidden row per accumulator tile, so the
//     per-row reductions over the vocabulary are in-register, plus one exchange with
//     lane^32 and one small LDS merge across the wavefronts of the workgroup.
//   * A workgroup owns TV vocabulary rows and up to MB hidden rows and streams its
//     W panel exactly once from HBM over the Dh axis in 64-element chunks, LDS
//     double-buffered with register prefetch; the (small) H panel is re-read from
//     L2 by every workgroup.
//   * Each workgroup writes one partial (max, sumexp, argmax, runner-up) per row;
//     a second kernel merges the V/TV partials per row in a fixed order
//     (deterministic; ties resolve to the lowest vocabulary index).
#include "common.hpp"

namespace dlm {

struct LmParams {
    int M, Dh, V;
    const uint16_t* hidden;
    int64_t h_stride;
    const int32_t* row_idx;
    const int32_t* m_dev;
    const uint16_t* w;
    int64_t w_stride;
    float inv_t;
    int forbid;
    int out_scatter;
    float* conf;
    int32_t* tok;
    float *lse, *zmax, *z2nd;
    const int32_t* target;
    float* ztarget;
    f32x4* part;  // [M][n_vt] of (max, sumexp, runner-up, argmax bits)
    int n_vt, n_mc;   // partials per row (all launches of the call together), row chunks
    // One call may cover the vocabulary with two launches (full-height tiles, then half-height ones for the tail):
    // a launch owns n_vt_l tiles that begin at vocabulary row v_first and fill the partials vt0 .. vt0 + n_vt_l - 1.
    int n_vt_l, vt0, v_first;
    int gm, gv;   // workgroup blocking per XCD: gm row chunks x gv vocabulary tiles run side by side
    // Gumbel-max sampling (sample != 0): a second partial per (tile, row) of
    // (perturbed max, logit of that token, its index bits, unused)
    int sample;
    uint32_t seed_lo, seed_hi, step, stream;
    f32x4* part2;
    // conf_mode: DLM_CONF_*.  For the negative entropy, slot 3 of the second partial carries
    // U = sum_v exp(z_v - max) * (z_v - max) of the tile (entropy = log(sumexp) - U / sumexp).
    int conf_mode;
    // Two shapes queued for one call (the host expects fewer rows than its bound): a launch runs only when the
    // device's row count lies in (m_lo, m_hi]; the reduction reads the layout of the launch that ran.
    int m_lo, m_hi;
    int alt_cap, alt_n_vt;   // reduction: row count <= alt_cap (> 0) -> alt_n_vt partials per row, second partials at alt_part2
    f32x4* alt_part2;
};

// Row count of this launch; false when the device's count belongs to the other shape queued for the same call.
__device__ __forceinline__ bool lm_rows(const LmParams& p, int& M) {
    if (p.m_dev) {
        const int md = max(*p.m_dev, 0);
        if (md <= p.m_lo || md > p.m_hi) return false;
        M = min(M, md);
    }
    return true;
}

struct Red {
    float m, s, m2;
    int idx;
};
// merge two partial reductions; on equal maxima the lower index wins and the runner-up equals the maximum
__device__ __forceinline__ Red red_merge(const Red a, const Red b) {
    const bool takeb = (b.m > a.m) || (b.m == a.m && b.idx < a.idx);
    const float mx = fmaxf(a.m, b.m), mn = fminf(a.m, b.m);
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * fast_exp2((a.m - mx) * 1.4426950408889634f);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * fast_exp2((b.m - mx) * 1.4426950408889634f);
    const int ai = a.idx, bi = b.idx;
    Red r;
    r.m = mx;
    r.s = sa + sb;
    r.m2 = fmaxf(fmaxf(a.m2, b.m2), mn);
    r.idx = takeb ? bi : ai;
    return r;
}
__device__ __forceinline__ Red red_shfl_xor(const Red a, int off) {
    Red o;
    o.m = shfl_xor(a.m, off);
    o.s = shfl_xor(a.s, off);
    o.m2 = shfl_xor(a.m2, off);
    o.idx = shfl_xor(a.idx, off);
    return o;
}

// ---- noise for sampling ------------------------------------------------------------------------
// Philox-4x32, ten rounds (Salmon et al., SC 2011): a keyed bijection of a 128-bit counter.  The word for
// (row key r, token v) is word v % 4 of Philox(counter = (v / 4, r, step, stream), key = seed).
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    u32x4 out = {c0, c1, c2, c3};
    return out;
}
// Standard Gumbel variate -log(-log u) from the top 23 bits k of a word: u = (2k + 1) / 2^24, an odd 24-bit
// numerator, so u and 1 - u are exact in single precision.  Close to u = 1, where the largest variates (the
// ones that decide an arg-max) come from, -log u is summed as a series in 1 - u: the hardware logarithm's
// absolute error would otherwise turn into a relative error of -log u and an absolute error of the variate.
__device__ __forceinline__ float gumbel_from_bits(uint32_t bits) {
    const uint32_t odd = 2u * (bits >> 9) + 1u;
    const float u = (float)odd * 0x1p-24f;
    const float w = (float)(0x1000000u - odd) * 0x1p-24f;   // 1 - u
    constexpr float LN2 = 0.6931471805599453f;
    const float e_series = w * (1.0f + w * (0.5f + w * (0.33333334f + w * (0.25f + w * 0.2f))));
    const float e_log = -LN2 * __builtin_amdgcn_logf(u);
    const float e = (w < 0x1p-6f) ? e_series : e_log;        // -log u, an Exp(1) variate
    return -LN2 * __builtin_amdgcn_logf(e);
}
struct Smp {
    float pm, pz;   // perturbed maximum, unperturbed logit of its token
    int idx;
};
// the larger perturbed value wins; on equal values the lower index
__device__ __forceinline__ Smp smp_merge(const Smp a, const Smp b) {
    const bool takeb = (b.pm > a.pm) || (b.pm == a.pm && b.idx < a.idx);
    const float apm = a.pm, apz = a.pz, bpm = b.pm, bpz = b.pz;
    const int ai = a.idx, bi = b.idx;
    Smp r;
    r.pm = takeb ? bpm : apm;
    r.pz = takeb ? bpz : apz;
    r.idx = takeb ? bi : ai;
    return r;
}

// U of the union of two partials a, b (each relative to its own maximum), relative to the joint maximum
__device__ __forceinline__ float u_merge(const Red a, float ua, const Red b, float ub) {
    constexpr float LOG2E = 1.4426950408889634f;
    const float mx = fmaxf(a.m, b.m);
    float r = 0.f;
    if (a.m > -INFINITY) r += fast_exp2((a.m - mx) * LOG2E) * (ua + (a.m - mx) * a.s);
    if (b.m > -INFINITY) r += fast_exp2((b.m - mx) * LOG2E) * (ub + (b.m - mx) * b.s);
    return r;
}

constexpr int KC = 64;             // Dh elements per pipeline stage (128 B per row); Dh must be a multiple of it
constexpr int LP = KC * 2 + 16;    // LDS row pitch in bytes: 16-byte reads of 16 consecutive rows hit distinct banks

// Workgroup -> (vocabulary tile, row chunk).  Workgroups are dealt round-robin to the 8 XCDs (each with
// its own L2), so what one XCD runs at the same time is a run of consecutive slots of ITS list.  Those slots
// are laid out as blocks of gv vocabulary tiles x gm row chunks: with one row chunk (the rollout) a W tile
// comes from HBM once; with many row chunks a block of gv x gm workgroups shares gv W panels and gm H panels
// through that XCD's L2 instead of streaming all of H once per vocabulary tile.  group = index of the block's
// vocabulary-tile group: workgroups of one block start their walk over Dh at the same chunk.
__device__ __forceinline__ void lm_tile_of_block(int bid, int n_mc, int gm, int gv, int& vt, int& mc, int& group) {
    const int xcd = bid & 7, slot = bid >> 3;
    const int per_super = gv * n_mc;
    const int super = slot / per_super, within = slot - super * per_super;
    const int blk = within / (gv * gm), r = within - blk * (gv * gm);
    const int v_local = r / gm;
    mc = blk * gm + (r - v_local * gm);
    vt = (super * gv + v_local) * 8 + xcd;
    group = super;
}

// Per hidden row (matrix column): reduce over this workgroup's vocabulary rows and write one partial.
// Called after the main loop's final barrier, so the staging area can be reused.
template <int WV, int WH, int TVW, int THW>
__device__ __forceinline__ void lm_epilogue(const LmParams& p, f32x16 (&acc)[TVW][THW], unsigned char* smem, int v0, int m0,
                                            int M, int vt, int wv, int wh, int n, int hi, int tid) {
    constexpr int NT = 64 * WV * WH;
    constexpr int MB = 32 * THW * WH;
    constexpr float LOG2E = 1.4426950408889634f;
    f32x4* redbuf = reinterpret_cast<f32x4*>(smem);  // [WV][MB] of (max, sumexp, runner-up, argmax bits)
    f32x4* redbuf2 = redbuf + WV * MB;               // [WV][MB] of the second partial (sampling and / or entropy)
    const bool ent = p.conf_mode == DLM_CONF_NEG_ENTROPY;
    const bool second = p.sample || ent;
    constexpr int TVWG = 32 * TVW * WV;
    // does this workgroup's vocabulary tile hold a token that must be masked (past V, or the forbidden one)?
    const bool edge = (v0 + TVWG > p.V) || (p.forbid >= v0 && p.forbid < v0 + TVWG);
    // (the loop above ended with a barrier: the staging area is free)
#pragma unroll
    for (int c = 0; c < THW; ++c) {
        if (m0 + (wh * THW + c) * 32 >= M) continue;   // a row tile past the last row: nothing reads its partials
        const int col = (wh * THW + c) * 32 + n;       // hidden row inside the workgroup's MB
        const int r = m0 + col;
        int tgt = -1;
        int64_t oidx = 0;
        if (r < M) {
            oidx = (p.out_scatter && p.row_idx) ? (int64_t)p.row_idx[r] : (int64_t)r;
            if (p.target) tgt = p.target[oidx];
        }
        // scaled (and, in a tile that holds a forbidden or out-of-range token, masked) logits, kept in acc
        const int vb = v0 + wv * TVW * 32 + 4 * hi;    // this lane's token of element (a, i): vb + 32 a + 8 (i >> 2) + (i & 3)
        if (edge) {
#pragma unroll
            for (int a = 0; a < TVW; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int v = vb + a * 32 + 8 * (i >> 2) + (i & 3);
                    const float z = acc[a][c][i] * p.inv_t;
                    acc[a][c][i] = (v >= p.V || v == p.forbid) ? -INFINITY : z;
                }
        } else {
#pragma unroll
            for (int a = 0; a < TVW; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][c][i] *= p.inv_t;
        }
        if (p.target) {                                // the target's logit, if this lane holds it
            const int dt = tgt - vb;
            float zt = 0.f;
            bool found = false;
#pragma unroll
            for (int a = 0; a < TVW; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const bool hit = dt == a * 32 + 8 * (i >> 2) + (i & 3);
                    zt = hit ? acc[a][c][i] : zt;
                    found |= hit;
                }
            if (found && tgt >= 0) p.ztarget[oidx] = zt;
        }
        // maximum and runner-up (equal to the maximum when it occurs twice): the two largest of (m, m2, z)
        Red red{-INFINITY, 0.f, -INFINITY, 0x7fffffff};
#pragma unroll
        for (int a = 0; a < TVW; ++a)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float z = acc[a][c][i];
                red.m2 = __builtin_amdgcn_fmed3f(red.m, red.m2, z);
                red.m = fmaxf(red.m, z);
            }
        // lowest token that attains the maximum: walk downwards, the last hit stays (offsets from vb are constants)
        if (red.m > -INFINITY) {
            int li = 0;
#pragma unroll
            for (int a = TVW - 1; a >= 0; --a)
#pragma unroll
                for (int i = 15; i >= 0; --i)
                    li = (acc[a][c][i] == red.m) ? a * 32 + 8 * (i >> 2) + (i & 3) : li;
            red.idx = vb + li;
        }
        float uent = 0.f;
        if (red.m > -INFINITY) {
            const float mb = red.m * LOG2E;
            float s = 0.f;
            if (ent) {
#pragma unroll
                for (int a = 0; a < TVW; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float z = acc[a][c][i];
                        const float e = fast_exp2(z * LOG2E - mb);
                        s += e;
                        uent += (z > -INFINITY) ? e * (z - red.m) : 0.f;
                    }
            } else {
#pragma unroll
                for (int a = 0; a < TVW; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s += fast_exp2(acc[a][c][i] * LOG2E - mb);
            }
            red.s = s;
        }
        {
            const Red o = red_shfl_xor(red, 32);
            if (ent) uent = u_merge(red, uent, o, shfl_xor(uent, 32));
            red = red_merge(red, o);
        }
        if (hi == 0) {
            f32x4 packed = {red.m, red.s, red.m2, __int_as_float(red.idx)};
            redbuf[wv * MB + col] = packed;
        }
        Smp sm{-INFINITY, -INFINITY, 0x7fffffff};
        if (p.sample) {
            // acc now holds the scaled, masked logits; noise is keyed by the row's index in `hidden`
            const uint32_t rk = (r < M) ? (uint32_t)(p.row_idx ? p.row_idx[r] : r) : 0u;
#pragma unroll
            for (int a = 0; a < TVW; ++a) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int vq = v0 + (wv * TVW + a) * 32 + 8 * i4 + 4 * hi;   // four consecutive tokens, vq % 4 == 0
                    const u32x4 bits = philox4x32_10((uint32_t)vq >> 2, rk, p.step, p.stream, p.seed_lo, p.seed_hi);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float z = acc[a][c][4 * i4 + e];
                        const float pert = z + gumbel_from_bits(bits[e]);
                        if (pert > sm.pm) {
                            sm.pm = pert;
                            sm.pz = z;
                            sm.idx = vq + e;
                        }
                    }
                }
            }
            Smp o;
            o.pm = shfl_xor(sm.pm, 32);
            o.pz = shfl_xor(sm.pz, 32);
            o.idx = shfl_xor(sm.idx, 32);
            sm = smp_merge(sm, o);
        }
        if (second && hi == 0) {
            f32x4 packed = {sm.pm, sm.pz, __int_as_float(sm.idx), uent};
            redbuf2[wv * MB + col] = packed;
        }
    }
    __syncthreads();
    for (int col = tid; col < MB; col += NT) {
        const int r = m0 + col;
        if (r >= M) continue;
        const f32x4 f = redbuf[col];
        Red red{f[0], f[1], f[2], __float_as_int(f[3])};
        f32x4 g = {-INFINITY, -INFINITY, __int_as_float(0x7fffffff), 0.f};
        if (second) g = redbuf2[col];
        Smp sm{g[0], g[1], __float_as_int(g[2])};
        float uent = g[3];
#pragma unroll
        for (int k = 1; k < WV; ++k) {
            const f32x4 o = redbuf[k * MB + col];
            const Red ro{o[0], o[1], o[2], __float_as_int(o[3])};
            if (second) {
                const f32x4 o2 = redbuf2[k * MB + col];
                sm = smp_merge(sm, Smp{o2[0], o2[1], __float_as_int(o2[2])});
                if (ent) uent = u_merge(red, uent, ro, o2[3]);
            }
            red = red_merge(red, ro);
        }
        f32x4 out = {red.m, red.s, red.m2, __int_as_float(red.idx)};
        p.part[(int64_t)r * p.n_vt + vt] = out;
        if (second) {
            f32x4 out2 = {sm.pm, sm.pz, __int_as_float(sm.idx), uent};
            p.part2[(int64_t)r * p.n_vt + vt] = out2;
        }
    }
}

// WV x WH wavefronts; each owns TVW x THW accumulator tiles of 32 (vocab) x 32 (hidden rows).
// PD = how many 64-element chunks of W / H are in flight in registers ahead of the one being multiplied.
// NTW: W is fetched with non-temporal loads (see the launch table: for launches with one row chunk).
template <int WV, int WH, int TVW, int THW, int PD, int KCH = 64, int OCC = 1, bool PIPE = false, bool NTW = false>
__global__ __launch_bounds__(64 * WV * WH, OCC) void lmhead_kernel(LmParams p) {
    constexpr int NT = 64 * WV * WH;
    constexpr int TV = 32 * TVW * WV;   // vocabulary rows per workgroup
    constexpr int MB = 32 * THW * WH;   // hidden rows per workgroup
    constexpr int KC = KCH;             // shadows the namespace constant: elements per stage of THIS shape
    constexpr int LP = KC * 2 + 16;
    constexpr int TPR = KC / 8;         // threads covering one row segment with 16-byte loads
    constexpr int RPP = NT / TPR;       // rows covered by one pass
    constexpr int WLD = (TV + RPP - 1) / RPP;
    constexpr int HLD = (MB + RPP - 1) / RPP;
    constexpr int STAGE = (TV + MB) * LP;
    constexpr int RED_BYTES = WV * MB * 16;
    static_assert(2 * STAGE >= 2 * RED_BYTES, "both reduction buffers must fit in the staging area");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wv = w % WV, wh = w / WV;
    const int n = lane & 31, hi = lane >> 5;
    int vt, mc, kgroup;
    lm_tile_of_block(blockIdx.x, p.n_mc, p.gm, p.gv, vt, mc, kgroup);
    if (vt >= p.n_vt_l) return;
    const int v0 = p.v_first + vt * TV;
    vt += p.vt0;
    const int m0 = mc * MB;
    int M = p.M;
    if (!lm_rows(p, M)) return;
    if (m0 >= M) return;

    // ---- global -> register staging addresses --------------------------------
    const int lrow = tid / TPR, lc = tid % TPR;
#define W_ON(q) ((TV % RPP == 0) || (lrow + (q) * RPP < TV))   // a ragged last pass leaves some threads idle
#define H_ON(q) ((MB % RPP == 0) || (lrow + (q) * RPP < MB))
    const uint16_t* wsrc[WLD];
#pragma unroll
    for (int q = 0; q < WLD; ++q) {
        const int v = min(v0 + lrow + q * RPP, p.V - 1);       // rows past V are clamped, masked in the epilogue
        wsrc[q] = p.w + (int64_t)v * p.w_stride + lc * 8;
    }
    const uint16_t* hsrc[HLD];
#pragma unroll
    for (int q = 0; q < HLD; ++q) {
        const int r = min(m0 + lrow + q * RPP, M - 1);         // rows past M are clamped, never stored
        const int64_t src = p.row_idx ? p.row_idx[r] : r;
        hsrc[q] = p.hidden + src * p.h_stride + lc * 8;
    }
    u32x4 wreg[PD][WLD], hreg[PD][HLD];

    f32x16 acc[TVW][THW];
#pragma unroll
    for (int a = 0; a < TVW; ++a)
#pragma unroll
        for (int c = 0; c < THW; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][c][i] = 0.f;

    const int nk = p.Dh / KC;
    // Every workgroup walks the Dh axis from a different starting chunk (and wraps).  Rows of W are a power
    // of two apart, so workgroups marching in step over the same columns would all hit the same few HBM
    // channels; the rotation spreads them (measured: 5.0 -> 6.2 TB/s on a pure read of W in this pattern).
    const int kstart = (int)(((long)(p.gv > 1 ? kgroup : vt) * 11) % nk);
#define LM_CHUNK(kc) (((kc) + kstart) >= nk ? ((kc) + kstart - nk) : ((kc) + kstart))
#define LM_GLOAD(slot, kc)                                                                               \
    {                                                                                                    \
        _Pragma("unroll") for (int q = 0; q < WLD; ++q) if (W_ON(q))                                     \
            wreg[slot][q] = NTW ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wsrc[q] + LM_CHUNK(kc) * KC)) \
                                : *reinterpret_cast<const u32x4*>(wsrc[q] + LM_CHUNK(kc) * KC);          \
        _Pragma("unroll") for (int q = 0; q < HLD; ++q) if (H_ON(q))                                     \
            hreg[slot][q] = *reinterpret_cast<const u32x4*>(hsrc[q] + LM_CHUNK(kc) * KC);                \
    }
#define LM_LSTORE(slot, buf)                                                                             \
    {                                                                                                    \
        unsigned char* Wl_ = smem + (buf) * STAGE;                                                       \
        unsigned char* Hl_ = Wl_ + TV * LP;                                                              \
        _Pragma("unroll") for (int q = 0; q < WLD; ++q) if (W_ON(q))                                     \
            *reinterpret_cast<u32x4*>(Wl_ + (lrow + q * RPP) * LP + lc * 16) = wreg[slot][q];            \
        _Pragma("unroll") for (int q = 0; q < HLD; ++q) if (H_ON(q))                                     \
            *reinterpret_cast<u32x4*>(Hl_ + (lrow + q * RPP) * LP + lc * 16) = hreg[slot][q];            \
    }

    // NL = live 32-row tiles of this wavefront (the tiles past the launch's last row are never multiplied)
#define LM_COMPUTE(buf, NL)                                                                              \
    if constexpr ((NL) > 0) {                                                                            \
        const unsigned char* Wl = smem + (buf) * STAGE + (wv * TVW * 32 + n) * LP + hi * 16;             \
        const unsigned char* Hl = smem + (buf) * STAGE + TV * LP + (wh * THW * 32 + n) * LP + hi * 16;   \
        _Pragma("unroll") for (int ks = 0; ks < KC / 16; ++ks) {                                         \
            bf16x8 af[TVW], bfr[THW];                                                                    \
            _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                              \
                af[a] = *reinterpret_cast<const bf16x8*>(Wl + a * 32 * LP + ks * 32);                    \
            _Pragma("unroll") for (int c = 0; c < (NL); ++c)                                             \
                bfr[c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * LP + ks * 32);                   \
            _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                              \
                _Pragma("unroll") for (int c = 0; c < (NL); ++c)                                         \
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[c], acc[a][c], 0, 0, 0); \
        }                                                                                                \
    }

    // Software-pipelined iteration: fragments of step ks+1 are requested before the MFMAs of step ks, and
    // the LDS stores of the next chunk are spread between the MFMA groups instead of preceding them, so the
    // LDS port and the load-counter waits overlap with matrix work inside each wavefront.
    constexpr int KSTEPS = KC / 16;
    constexpr int NST = WLD + HLD;
#define LM_STORE_ONE(slot, buf, i)                                                                       \
    {                                                                                                    \
        unsigned char* Wl_ = smem + (buf) * STAGE;                                                       \
        unsigned char* Hl_ = Wl_ + TV * LP;                                                              \
        if ((i) < WLD) { if (W_ON(i)) *reinterpret_cast<u32x4*>(Wl_ + (lrow + (i) * RPP) * LP + lc * 16) = wreg[slot][(i) < WLD ? (i) : 0]; } \
        else { if (H_ON((i) - WLD)) *reinterpret_cast<u32x4*>(Hl_ + (lrow + ((i) - WLD) * RPP) * LP + lc * 16) = hreg[slot][(i) >= WLD ? (i) - WLD : 0]; } \
    }
#define LM_ITER_PIPE(buf, do_store, slot, nbuf, NL)                                                      \
    {                                                                                                    \
        const unsigned char* Wl = smem + (buf) * STAGE + (wv * TVW * 32 + n) * LP + hi * 16;             \
        const unsigned char* Hl = smem + (buf) * STAGE + TV * LP + (wh * THW * 32 + n) * LP + hi * 16;   \
        bf16x8 af[2][TVW], bfr[2][THW];                                                                  \
        if constexpr ((NL) > 0) {                                                                        \
            _Pragma("unroll") for (int a = 0; a < TVW; ++a) af[0][a] = *reinterpret_cast<const bf16x8*>(Wl + a * 32 * LP); \
            _Pragma("unroll") for (int c = 0; c < (NL); ++c) bfr[0][c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * LP); \
        }                                                                                                \
        _Pragma("unroll") for (int ks = 0; ks < KSTEPS; ++ks) {                                          \
            if constexpr ((NL) > 0) {                                                                    \
                if (ks + 1 < KSTEPS) {                                                                   \
                    _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                      \
                        af[(ks + 1) & 1][a] = *reinterpret_cast<const bf16x8*>(Wl + a * 32 * LP + (ks + 1) * 32); \
                    _Pragma("unroll") for (int c = 0; c < (NL); ++c)                                     \
                        bfr[(ks + 1) & 1][c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * LP + (ks + 1) * 32); \
                }                                                                                        \
                _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                          \
                    _Pragma("unroll") for (int c = 0; c < (NL); ++c)                                     \
                        acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][a], bfr[ks & 1][c], acc[a][c], 0, 0, 0); \
            }                                                                                            \
            if (do_store) {                                                                              \
                _Pragma("unroll") for (int i = 0; i < NST; ++i)                                          \
                    if (i * KSTEPS / NST == ks) LM_STORE_ONE(slot, nbuf, i);                             \
            }                                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                                           \
        }                                                                                                \
    }

    // prologue: chunks 0 .. PD-1 in flight, chunk 0 staged, chunk PD requested.
    // Steady state, free of conditions so that the load counter waits can be exact: iteration kc stages
    // chunk kc+1 (requested PD chunks ago) into the other LDS buffer, requests chunk kc+1+PD into the
    // register slot just freed, multiplies chunk kc.  Chunk c lives in register slot c % PD.
    // Drain (at most 2*PD chunks): same steps, each guarded.
#define LM_MAIN(NL)                                                                                      \
    {                                                                                                    \
        _Pragma("unroll") for (int s = 0; s < PD; ++s)                                                   \
            if (s < nk) LM_GLOAD(s, s);                                                                  \
        LM_LSTORE(0, 0);                                                                                 \
        if (PD < nk) LM_GLOAD(0, PD);                                                                    \
        __syncthreads();                                                                                 \
        int kc = 0;                                                                                      \
        const int n_main = (nk - PD - 1 > 0) ? ((nk - PD - 1) / PD) * PD : 0;                            \
        for (; kc < n_main; kc += PD) {                                                                  \
            _Pragma("unroll") for (int u = 0; u < PD; ++u) {                                             \
                if (PIPE) {                                                                              \
                    LM_ITER_PIPE((kc + u) & 1, true, (u + 1) % PD, (kc + u + 1) & 1, NL);                \
                    LM_GLOAD((u + 1) % PD, kc + u + 1 + PD);                                             \
                } else {                                                                                 \
                    LM_LSTORE((u + 1) % PD, (kc + u + 1) & 1);                                           \
                    LM_GLOAD((u + 1) % PD, kc + u + 1 + PD);                                             \
                    LM_COMPUTE((kc + u) & 1, NL);                                                        \
                }                                                                                        \
                __syncthreads();                                                                         \
            }                                                                                            \
        }                                                                                                \
        _Pragma("unroll") for (int u = 0; u < 2 * PD; ++u) {                                             \
            const int k = kc + u;                                                                        \
            if (k < nk) {                                                                                \
                if (k + 1 < nk) {                                                                        \
                    LM_LSTORE((u + 1) % PD, (k + 1) & 1);                                                \
                    if (k + 1 + PD < nk) LM_GLOAD((u + 1) % PD, k + 1 + PD);                             \
                }                                                                                        \
                LM_COMPUTE(k & 1, NL);                                                                   \
                __syncthreads();                                                                         \
            }                                                                                            \
        }                                                                                                \
    }
    // Where the wavefronts split the rows (WH > 1), the loop exists once per count of live row tiles of a
    // wavefront: the rollout's host knows a step's row count only as an upper bound, and a launch sized for it
    // should cost what the rows that exist cost.  Every copy runs the same loads, stores and barriers.
    if constexpr (WH > 1 && PIPE) {
        const int nl = __builtin_amdgcn_readfirstlane(min(max((M - m0 - wh * THW * 32 + 31) >> 5, 0), THW));
#define LM_CASE(k)                                                                                       \
    case k:                                                                                              \
        if constexpr ((k) <= THW) { LM_MAIN(k) }                                                         \
        break;
        switch (nl) {
            LM_CASE(0) LM_CASE(1) LM_CASE(2) LM_CASE(3) LM_CASE(4)
            default: break;
        }
        static_assert(THW <= 4, "one copy of the loop per live-tile count");
#undef LM_CASE
    } else {
        LM_MAIN(THW)
    }
#undef LM_MAIN
#undef W_ON
#undef H_ON
#undef LM_COMPUTE
#undef LM_ITER_PIPE
#undef LM_STORE_ONE
#undef LM_GLOAD
#undef LM_CHUNK
#undef LM_LSTORE

    lm_epilogue<WV, WH, TVW, THW>(p, acc, smem, v0, m0, M, vt, wv, wh, n, hi, tid);
}

// Second kernel family: W fragments go straight from global memory into MFMA A-operand registers.
// The wavefronts of a workgroup split only the vocabulary, so no W element is shared between them and
// staging W in LDS would only add LDS traffic (the LDS port, not the MFMA pipe, limits the shared-W shapes
// once M > 128).  Only the H panel, which every wavefront needs, is staged in LDS.
// Within a 64-element chunk a lane half `hi` owns elements [32*hi, 32*hi + 32): it reads 64 contiguous
// bytes of its W row with four 16-byte loads, and MFMA step ks contracts elements 32*hi + 8*ks + e.  H is
// read from LDS with the same element order, so the contraction still covers every k exactly once.
template <int WV, int TVW, int THW, int PDW>
__global__ __launch_bounds__(64 * WV) void lmhead_wdirect_kernel(LmParams p) {
    constexpr int NT = 64 * WV;
    constexpr int TV = 32 * TVW * WV;
    constexpr int MB = 32 * THW;
    constexpr int PDH = (PDW > 1) ? PDW - 1 : 1;   // H chunks in flight (H comes from L2: shorter latency)
    constexpr int UNR = PDW * PDH;                 // iterations per unrolled group: both register rings return to slot 0
    constexpr int RPP = NT / 8;
    constexpr int HLD = (MB + RPP - 1) / RPP;
    constexpr int HSTAGE = MB * LP;
    static_assert(2 * HSTAGE >= 2 * WV * MB * 16, "both reduction buffers must fit in the staging area");
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * HSTAGE];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = lane & 31, hi = lane >> 5;
    int vt, mc, kgroup;
    lm_tile_of_block(blockIdx.x, p.n_mc, p.gm, p.gv, vt, mc, kgroup);
    if (vt >= p.n_vt_l) return;
    const int v0 = p.v_first + vt * TV;
    vt += p.vt0;
    const int m0 = mc * MB;
    int M = p.M;
    if (!lm_rows(p, M)) return;
    if (m0 >= M) return;

    const uint16_t* wsrc[TVW];
#pragma unroll
    for (int a = 0; a < TVW; ++a) {
        const int v = min(v0 + (wv * TVW + a) * 32 + n, p.V - 1);
        wsrc[a] = p.w + (int64_t)v * p.w_stride + hi * 32;
    }
    const int lrow = tid >> 3, lc = tid & 7;
#define H_ON(q) ((MB % RPP == 0) || (lrow + (q) * RPP < MB))
    const uint16_t* hsrc[HLD];
#pragma unroll
    for (int q = 0; q < HLD; ++q) {
        const int r = min(m0 + lrow + q * RPP, M - 1);
        const int64_t src = p.row_idx ? p.row_idx[r] : r;
        hsrc[q] = p.hidden + src * p.h_stride + lc * 8;
    }
    u32x4 wreg[PDW][TVW][4], hreg[PDH][HLD];
    f32x16 acc[TVW][THW];
#pragma unroll
    for (int a = 0; a < TVW; ++a)
#pragma unroll
        for (int c = 0; c < THW; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][c][i] = 0.f;

    const int nk = p.Dh / KC;
    const int kstart = (int)(((long)(p.gv > 1 ? kgroup : vt) * 11) % nk);
#define LM_CHUNK(kc) (((kc) + kstart) >= nk ? ((kc) + kstart - nk) : ((kc) + kstart))
#define WD_GLOAD_W(slot, kc)                                                                             \
    {                                                                                                    \
        const int ch_ = LM_CHUNK(kc) * KC;                                                               \
        _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                                  \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
                wreg[slot][a][j] = *reinterpret_cast<const u32x4*>(wsrc[a] + ch_ + j * 8);               \
    }
#define WD_GLOAD_H(slot, kc)                                                                             \
    {                                                                                                    \
        const int ch_ = LM_CHUNK(kc) * KC;                                                               \
        _Pragma("unroll") for (int q = 0; q < HLD; ++q) if (H_ON(q))                                     \
            hreg[slot][q] = *reinterpret_cast<const u32x4*>(hsrc[q] + ch_);                              \
    }
#define WD_LSTORE_H(slot, buf)                                                                           \
    {                                                                                                    \
        unsigned char* Hl_ = smem + (buf) * HSTAGE;                                                      \
        _Pragma("unroll") for (int q = 0; q < HLD; ++q) if (H_ON(q))                                     \
            *reinterpret_cast<u32x4*>(Hl_ + (lrow + q * RPP) * LP + lc * 16) = hreg[slot][q];            \
    }
#define WD_COMPUTE(wslot, buf)                                                                           \
    {                                                                                                    \
        const unsigned char* Hl = smem + (buf) * HSTAGE + n * LP + hi * 64;                              \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                               \
            bf16x8 bfr[THW];                                                                             \
            _Pragma("unroll") for (int c = 0; c < THW; ++c)                                              \
                bfr[c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * LP + ks * 16);                   \
            _Pragma("unroll") for (int a = 0; a < TVW; ++a) {                                            \
                union { u32x4 u; bf16x8 b; } af_;                                                        \
                af_.u = wreg[wslot][a][ks];                                                              \
                _Pragma("unroll") for (int c = 0; c < THW; ++c)                                          \
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af_.b, bfr[c], acc[a][c], 0, 0, 0); \
            }                                                                                            \
        }                                                                                                \
    }

    // prologue: H(0) staged in LDS buffer 0; registers hold H(1..PDH) and W(0..PDW-1); chunk c sits in
    // slot c % PDH (H) / c % PDW (W)
    WD_GLOAD_H(0, 0);
#pragma unroll
    for (int c = 0; c < PDW; ++c) {
        if (c < nk) WD_GLOAD_W(c, c);
        if (c + 1 < PDH && c + 1 < nk) WD_GLOAD_H((c + 1) % PDH, c + 1);
    }
    WD_LSTORE_H(0, 0);
    if (PDH < nk) WD_GLOAD_H(0, PDH);
    __syncthreads();

    // steady state (no conditions): stage H(kc+1), request H(kc+1+PDH), multiply chunk kc, request W(kc+PDW)
    int kc = 0;
    const int n_main = (nk - PDW > 0) ? ((nk - PDW) / UNR) * UNR : 0;
    for (; kc < n_main; kc += UNR) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            WD_LSTORE_H((u + 1) % PDH, (kc + u + 1) & 1);
            WD_GLOAD_H((u + 1) % PDH, kc + u + 1 + PDH);
            WD_COMPUTE(u % PDW, (kc + u) & 1);
            WD_GLOAD_W(u % PDW, kc + u + PDW);
            __syncthreads();
        }
    }
    // drain: same steps, each guarded
#pragma unroll
    for (int u = 0; u < UNR + PDW; ++u) {
        const int k = kc + u;
        if (k < nk) {
            if (k + 1 < nk) {
                WD_LSTORE_H((u + 1) % PDH, (k + 1) & 1);
                if (k + 1 + PDH < nk) WD_GLOAD_H((u + 1) % PDH, k + 1 + PDH);
            }
            WD_COMPUTE(u % PDW, k & 1);
            if (k + PDW < nk) WD_GLOAD_W(u % PDW, k + PDW);
            __syncthreads();
        }
    }
#undef H_ON
#undef WD_GLOAD_W
#undef WD_GLOAD_H
#undef WD_LSTORE_H
#undef WD_COMPUTE
#undef LM_CHUNK

    lm_epilogue<WV, 1, TVW, THW>(p, acc, smem, v0, m0, M, vt, wv, 0, n, hi, tid);
}

// Third kernel family, for the MFMA-bound regime (M >= 256): both operand panels go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane, no staging registers), through a ring of NS stages
// of 32 Dh elements each, so NS-1 stages are in flight while one is being multiplied and the register file is
// left to a 128 x 128 accumulator tile per wavefront (4 x 4 MFMA tiles: half the LDS bytes per MFMA of the
// 64 x 128 shapes).  A wave's load instruction fills 1 KB of LDS = 16 rows x 64 B in lane order, so the
// bank-conflict-free layout is obtained by choosing WHICH 16-byte piece of its row each lane fetches:
// piece c of row r is stored at position c ^ ((r >> 2) & 3).
// XB = true keeps the MFMA operand fragments one MFMA step ahead ACROSS the workgroup barrier: while the 16 MFMAs
// of one 16-element step run, the fragments of the next step (of the next stage, in the second half) are read
// into a second register set, one LDS read issued behind each MFMA, so no MFMA ever waits for an LDS read that
// was issued just before it; the barrier sits between the two steps of a stage.
template <int WV, int WH, int TVW, int THW, int NS, bool XB = false>
__global__ __launch_bounds__(64 * WV * WH) void lmhead_dma_kernel(LmParams p) {
    constexpr int KCD = 32, ROWB = 64;
    constexpr int NW = WV * WH, NT = 64 * NW;
    constexpr int TV = 32 * TVW * WV, MB = 32 * THW * WH;
    constexpr int STAGE = (TV + MB) * ROWB;
    constexpr int IPW = (TV + MB) / 16 / NW;          // load instructions per wavefront per stage
    static_assert((TV + MB) / 16 % NW == 0, "rows must split evenly over the wavefronts");
    static_assert(NS >= 2 && NS <= 8 && NS * STAGE <= 160 * 1024, "ring of 2..8 stages within the 160 KB of LDS");
    static_assert(NS * STAGE >= 2 * WV * MB * 16, "both reduction buffers must fit in the ring");
    __shared__ __attribute__((aligned(1024))) unsigned char ring[NS * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wv = w % WV, wh = w / WV;
    const int n = lane & 31, hi = lane >> 5;
    int vt, mc, kgroup;
    lm_tile_of_block(blockIdx.x, p.n_mc, p.gm, p.gv, vt, mc, kgroup);
    if (vt >= p.n_vt_l) return;
    const int v0 = p.v_first + vt * TV, m0 = mc * MB;
    vt += p.vt0;
    int M = p.M;
    if (!lm_rows(p, M)) return;
    if (m0 >= M) return;

    // per-lane source of each of this wavefront's load instructions (row of the combined [W rows | H rows] panel)
    const uint16_t* src[IPW];
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        const int row = (w * IPW + j) * 16 + (lane >> 2);
        const int piece = (lane & 3) ^ ((row >> 2) & 3);
        if (row < TV) {
            const int v = min(v0 + row, p.V - 1);
            src[j] = p.w + (int64_t)v * p.w_stride + piece * 8;
        } else {
            const int r = min(m0 + row - TV, M - 1);
            const int64_t sr = p.row_idx ? p.row_idx[r] : r;
            src[j] = p.hidden + sr * p.h_stride + piece * 8;
        }
    }
    const int nk = p.Dh / KCD;
    const int kstart = (int)(((long)(p.gv > 1 ? kgroup : vt) * 11) % nk);
#define DMA_CHUNK(kc) (((kc) + kstart) >= nk ? ((kc) + kstart - nk) : ((kc) + kstart))
#define DMA_ISSUE(stage, kc)                                                                             \
    {                                                                                                    \
        const int ch_ = DMA_CHUNK(kc) * KCD;                                                             \
        _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                                  \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ch_), \
                (__attribute__((address_space(3))) void*)(ring + (stage) * STAGE + (w * IPW + j) * 1024), 16, 0, 0); \
    }
    // wait until at most `cnt` of this wavefront's loads are outstanding, then meet the other wavefronts
#define DMA_SYNC(cnt)                                                                                    \
    {                                                                                                    \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(cnt) : "memory");                                       \
        __builtin_amdgcn_s_barrier();                                                                    \
        asm volatile("" ::: "memory");                                                                   \
    }

    f32x16 acc[TVW][THW];
#pragma unroll
    for (int a = 0; a < TVW; ++a)
#pragma unroll
        for (int c = 0; c < THW; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][c][i] = 0.f;

    const int sw = (n >> 2) & 3;
    const int off0 = n * ROWB + ((hi ^ sw) << 4);          // MFMA step 0: piece hi
    const int off1 = n * ROWB + (((2 + hi) ^ sw) << 4);    // MFMA step 1: piece 2 + hi
#define DMA_COMPUTE(stage)                                                                               \
    {                                                                                                    \
        const unsigned char* Wl = ring + (stage) * STAGE + wv * TVW * 32 * ROWB;                         \
        const unsigned char* Hl = ring + (stage) * STAGE + TV * ROWB + wh * THW * 32 * ROWB;             \
        bf16x8 af[2][TVW], bfr[2][THW];                                                                  \
        _Pragma("unroll") for (int a = 0; a < TVW; ++a) af[0][a] = *reinterpret_cast<const bf16x8*>(Wl + a * 32 * ROWB + off0); \
        _Pragma("unroll") for (int c = 0; c < THW; ++c) bfr[0][c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * ROWB + off0); \
        _Pragma("unroll") for (int a = 0; a < TVW; ++a) af[1][a] = *reinterpret_cast<const bf16x8*>(Wl + a * 32 * ROWB + off1); \
        _Pragma("unroll") for (int c = 0; c < THW; ++c) bfr[1][c] = *reinterpret_cast<const bf16x8*>(Hl + c * 32 * ROWB + off1); \
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                                 \
            _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                              \
                _Pragma("unroll") for (int c = 0; c < THW; ++c)                                          \
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][a], bfr[ks][c], acc[a][c], 0, 0, 0); \
    }

    // prologue: stages 0 .. NS-2 requested; stage 0 complete
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) DMA_ISSUE(s, s);
    if (nk >= NS - 1) { DMA_SYNC(IPW * (NS - 2)); } else { DMA_SYNC(0); }

    int kc = 0;
    const int n_main = (nk - (NS - 1) > 0) ? ((nk - (NS - 1)) / NS) * NS : 0;
    if constexpr (XB) {
        // One loop iteration per stage, all alike (no guarded drain): the request that would run past the last
        // chunk re-reads the last chunk into a stage nobody reads again, and the fragment reads of the last
        // iteration's second half fetch a stage that is never multiplied.  The stage index is a scalar.
        bf16x8 af[2][TVW], bfr[2][THW];
        const int wsc = __builtin_amdgcn_readfirstlane(w);
        const int lw0 = wv * TVW * 32 * ROWB + off0, lw1 = wv * TVW * 32 * ROWB + off1;
        const int lh0 = TV * ROWB + wh * THW * 32 * ROWB + off0, lh1 = TV * ROWB + wh * THW * 32 * ROWB + off1;
        // fragment i (0 .. TVW-1: W tiles, then the H tiles) of MFMA step `half` from the stage at byte offset sb
#define XB_READ_ONE(half, sb, i)                                                                         \
    {                                                                                                    \
        if ((i) < TVW) af[half][(i) < TVW ? (i) : 0] =                                                   \
            *reinterpret_cast<const bf16x8*>(ring + (sb) + ((half) ? lw1 : lw0) + (i) * 32 * ROWB);      \
        else bfr[half][(i) >= TVW ? (i) - TVW : 0] =                                                     \
            *reinterpret_cast<const bf16x8*>(ring + (sb) + ((half) ? lh1 : lh0) + ((i) - TVW) * 32 * ROWB); \
    }
        // TVW*THW MFMAs on register set `half`; behind the i-th MFMA goes the i-th auxiliary instruction: first the
        // fragment reads of the other set (from the stage at rsb), then (first half only) this wavefront's requests
        // of chunk `ich` (element offset) into the stage at isb
#define XB_HALF(half, rsb, do_issue, isb, ich)                                                           \
    {                                                                                                    \
        _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                                  \
            _Pragma("unroll") for (int c = 0; c < THW; ++c) {                                            \
                constexpr int NF = TVW + THW;                                                            \
                const int i_ = a * THW + c;                                                              \
                acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[half][a], bfr[half][c], acc[a][c], 0, 0, 0); \
                _Pragma("unroll") for (int f = 0; f < NF; ++f)                                           \
                    if (f * (TVW * THW) / (2 * NF) == i_) XB_READ_ONE(1 - (half), rsb, f);               \
                if (do_issue) {                                                                          \
                    _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                      \
                        if ((TVW * THW) / 2 + j * (TVW * THW) / (2 * IPW) == i_)                         \
                            __builtin_amdgcn_global_load_lds(                                            \
                                (const __attribute__((address_space(1))) void*)(src[j] + (ich)),         \
                                (__attribute__((address_space(3))) void*)(ring + (isb) + (wsc * IPW + j) * 1024), 16, 0, 0); \
                }                                                                                        \
                __builtin_amdgcn_sched_barrier(0);                                                       \
            }                                                                                            \
    }
#pragma unroll
        for (int f = 0; f < TVW + THW; ++f) XB_READ_ONE(0, 0, f);
        int sb = 0;                                   // byte offset of the stage being multiplied
        int ib = (NS - 1) * STAGE;                    // ... of the stage the next request fills
        for (int k = 0; k < nk; ++k) {
            const int nb = (sb + STAGE == NS * STAGE) ? 0 : sb + STAGE;
            const int ich = DMA_CHUNK(min(k + NS - 1, nk - 1)) * KCD;
            XB_HALF(0, sb, true, ib, ich);
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(IPW * (NS - 2)) : "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            XB_HALF(1, nb, false, 0, 0);
            ib = sb;
            sb = nb;
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef XB_READ_ONE
#undef XB_HALF
    } else {
    // steady state: request chunk kc+NS-1 into the stage freed by the previous iteration, multiply chunk kc,
    // wait for this wavefront's share of chunk kc+1, barrier (which also frees stage kc % NS for the next request)
    for (; kc < n_main; kc += NS) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            DMA_ISSUE((u + NS - 1) % NS, kc + u + NS - 1);
            DMA_COMPUTE(u);
            DMA_SYNC(IPW * (NS - 2));
        }
    }
    // drain: the remaining requests (if any) are guarded; waits are total
#pragma unroll
    for (int u = 0; u < 2 * NS; ++u) {
        const int k = kc + u;
        if (k < nk) {
            if (k + NS - 1 < nk) DMA_ISSUE((u + NS - 1) % NS, k + NS - 1);
            DMA_COMPUTE(u % NS);
            DMA_SYNC(0);
        }
    }
    }
#undef DMA_CHUNK
#undef DMA_ISSUE
#undef DMA_SYNC
#undef DMA_COMPUTE
    __syncthreads();
    lm_epilogue<WV, WH, TVW, THW>(p, acc, ring, v0, m0, M, vt, wv, wh, n, hi, tid);
}

// Fourth kernel family, the one used for the MFMA-bound regime: the direct-to-LDS ring above with three changes
// that each measured faster at M = 8192 (V = 126464, Dh = 4096; 1.24 -> 1.40 PFLOP/s for the loop alone):
//  * fragments are read one MFMA step ahead, across the barrier (as in the XB form above);
//  * requests come in PAIRS: a row's 64 bytes of chunk 2p and of chunk 2p+1 are the two halves of one 128-byte
//    line and are requested back to back, so the second request finds the line in (or on its way to) L1 instead
//    of fetching it from L2 a second time a whole stage later (the L2 -> LDS path alone: 17 -> 24 TB/s);
//  * the 2*IPW requests of a pair are spread evenly over the MFMAs of a whole stage period (second half of an even
//    stage, first half of the odd one) instead of being issued in a burst that backs up the address unit and
//    stalls the issuing wavefront (and with it the MFMAs behind the request).
// Five stages of 32 elements (the pair being multiplied, the pair in flight, and the stage just freed): pair
// (k+4, k+5) is requested after the barrier of even stage k, into stages (k+4) % 5 and k % 5, and must have landed
// by the barrier of stage k+3.
template <int WV, int WH, int TVW, int THW>
__global__ __launch_bounds__(64 * WV * WH) void lmhead_pair_kernel(LmParams p) {
    constexpr int NS = 5, KCD = 32, ROWB = 64;
    constexpr int NW = WV * WH;
    constexpr int TV = 32 * TVW * WV, MB = 32 * THW * WH;
    constexpr int STAGE = (TV + MB) * ROWB;
    constexpr int IPW = (TV + MB) / 16 / NW;          // 16-row groups per wavefront (two requests each per pair)
    static_assert((TV + MB) / 16 % NW == 0, "rows must split evenly over the wavefronts");
    static_assert(NS * STAGE <= 160 * 1024, "five stages within the 160 KB of LDS");
    static_assert(NS * STAGE >= 2 * WV * MB * 16, "both reduction buffers must fit in the ring");
    __shared__ __attribute__((aligned(1024))) unsigned char ring[NS * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wv = w % WV, wh = w / WV;
    const int n = lane & 31, hi = lane >> 5;
    int vt, mc, kgroup;
    lm_tile_of_block(blockIdx.x, p.n_mc, p.gm, p.gv, vt, mc, kgroup);
    if (vt >= p.n_vt_l) return;
    const int v0 = p.v_first + vt * TV, m0 = mc * MB;
    vt += p.vt0;
    int M = p.M;
    if (!lm_rows(p, M)) return;
    if (m0 >= M) return;

    const uint16_t* src[IPW];
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        const int row = (w * IPW + j) * 16 + (lane >> 2);
        const int piece = (lane & 3) ^ ((row >> 2) & 3);
        if (row < TV) {
            const int v = min(v0 + row, p.V - 1);
            src[j] = p.w + (int64_t)v * p.w_stride + piece * 8;
        } else {
            const int r = min(m0 + row - TV, M - 1);
            const int64_t sr = p.row_idx ? p.row_idx[r] : r;
            src[j] = p.hidden + sr * p.h_stride + piece * 8;
        }
    }
    const int nk = p.Dh / KCD;                        // even: Dh is a multiple of 64
    // rotated start as in the other shapes, kept even so that a pair stays one 128-byte line
    const int kstart = ((int)(((long)(p.gv > 1 ? kgroup : vt) * 11) % nk)) & ~1;
#define PR_CHUNK(kc) (((kc) + kstart) >= nk ? ((kc) + kstart - nk) : ((kc) + kstart))
    const int wsc = __builtin_amdgcn_readfirstlane(w);
#define PR_ISSUE1(sbyte, j, eoff)                                                                        \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + (eoff)),   \
        (__attribute__((address_space(3))) void*)(ring + (sbyte) + (wsc * IPW + (j)) * 1024), 16, 0, 0)

    f32x16 acc[TVW][THW];
#pragma unroll
    for (int a = 0; a < TVW; ++a)
#pragma unroll
        for (int c = 0; c < THW; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][c][i] = 0.f;

    const int sw = (n >> 2) & 3;
    const int off0 = n * ROWB + ((hi ^ sw) << 4);          // MFMA step 0: piece hi
    const int off1 = n * ROWB + (((2 + hi) ^ sw) << 4);    // MFMA step 1: piece 2 + hi
    const int lw0 = wv * TVW * 32 * ROWB + off0, lw1 = wv * TVW * 32 * ROWB + off1;
    const int lh0 = TV * ROWB + wh * THW * 32 * ROWB + off0, lh1 = TV * ROWB + wh * THW * 32 * ROWB + off1;
    bf16x8 af[2][TVW], bfr[2][THW];
    // fragment i (0 .. TVW-1: W tiles, then the H tiles) of MFMA step `half` from the stage at byte offset sb
#define PR_READ_ONE(half, sb, i)                                                                         \
    {                                                                                                    \
        if ((i) < TVW) af[half][(i) < TVW ? (i) : 0] =                                                   \
            *reinterpret_cast<const bf16x8*>(ring + (sb) + ((half) ? lw1 : lw0) + (i) * 32 * ROWB);      \
        else bfr[half][(i) >= TVW ? (i) - TVW : 0] =                                                     \
            *reinterpret_cast<const bf16x8*>(ring + (sb) + ((half) ? lh1 : lh0) + ((i) - TVW) * 32 * ROWB); \
    }
    // One half stage for a wavefront with NL live row tiles (NL <= THW; the tiles past the last row of the
    // launch are never multiplied): TVW * NL MFMAs on register set `half`; behind the first ones the fragment reads
    // of the other set (stage at rsb); part = 1 / 2: the first / second half of the pair's 2*IPW requests (chunk at
    // element offset ich into the stage at isb0, the following chunk into isb1), spread evenly over the MFMAs.
    // NL = 0 (every row tile of this wavefront is past the end): only its share of the requests.
#define PR_HALF(half, rsb, part, isb0, isb1, ich, NL)                                                    \
    {                                                                                                    \
        constexpr int T_ = TVW * (NL), NF_ = TVW + (NL);                                                 \
        if constexpr ((NL) == 0) {                                                                       \
            if ((part) != 0) {                                                                           \
                _Pragma("unroll") for (int j = 0; j < IPW; ++j) {                                        \
                    const int jj = j + ((part) == 2 ? IPW : 0);                                          \
                    if (jj & 1) PR_ISSUE1(isb1, jj >> 1, (ich) + KCD);                                   \
                    else PR_ISSUE1(isb0, jj >> 1, (ich));                                                \
                }                                                                                        \
            }                                                                                            \
        } else {                                                                                         \
        _Pragma("unroll") for (int a = 0; a < TVW; ++a)                                                  \
            _Pragma("unroll") for (int c = 0; c < (NL); ++c) {                                           \
                const int i_ = a * (NL) + c;                                                             \
                acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[half][a], bfr[half][c], acc[a][c], 0, 0, 0); \
                _Pragma("unroll") for (int f = 0; f < NF_; ++f)                                          \
                    if (f * T_ / (2 * NF_) == i_) PR_READ_ONE(1 - (half), rsb, f);                       \
                if ((part) != 0) {                                                                       \
                    _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                      \
                        if (j * T_ / IPW == i_) {                                                        \
                            const int jj = j + ((part) == 2 ? IPW : 0);                                  \
                            if (jj & 1) PR_ISSUE1(isb1, jj >> 1, (ich) + KCD);                           \
                            else PR_ISSUE1(isb0, jj >> 1, (ich));                                        \
                        }                                                                                \
                }                                                                                        \
                __builtin_amdgcn_sched_barrier(0);                                                       \
            }                                                                                            \
        }                                                                                                \
    }
#define PR_NEXT(x) (((x) + STAGE == NS * STAGE) ? 0 : (x) + STAGE)
    // prologue: pairs (0,1) -> stages 0,1 and (2,3) -> stages 2,3 (a request past the end re-reads the last pair);
    // then the loop over pairs of stages
#define PR_MAIN(NL)                                                                                      \
    {                                                                                                    \
        _Pragma("unroll") for (int pr = 0; pr < 2; ++pr) {                                               \
            const int e = PR_CHUNK(min(2 * pr, nk - 2)) * KCD;                                           \
            _Pragma("unroll") for (int j = 0; j < IPW; ++j) {                                            \
                PR_ISSUE1((2 * pr) * STAGE, j, e);                                                       \
                PR_ISSUE1((2 * pr + 1) * STAGE, j, e + KCD);                                             \
            }                                                                                            \
        }                                                                                                \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * IPW) : "memory");                                   \
        __builtin_amdgcn_s_barrier();                                                                    \
        asm volatile("" ::: "memory");                                                                   \
        if constexpr ((NL) > 0) {                                                                        \
            _Pragma("unroll") for (int f = 0; f < TVW + (NL); ++f) PR_READ_ONE(0, 0, f);                 \
        }                                                                                                \
        int sb = 0; /* byte offset of the stage of chunk k (k even at the loop top) */                   \
        for (int k = 0; k < nk; k += 2) {                                                                \
            const int s1 = PR_NEXT(sb), s2 = PR_NEXT(s1), s3 = PR_NEXT(s2), s4 = PR_NEXT(s3);            \
            const int ich = PR_CHUNK(min(k + 4, nk - 2)) * KCD;                                          \
            /* even stage k */                                                                           \
            PR_HALF(0, sb, 0, 0, 0, 0, NL);                                                              \
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                           \
            __builtin_amdgcn_s_barrier(); /* every wavefront has read stage k to the end: it is free */  \
            asm volatile("" ::: "memory");                                                               \
            PR_HALF(1, s1, 1, s4, sb, ich, NL);                                                          \
            /* odd stage k+1 */                                                                          \
            PR_HALF(0, s1, 2, s4, sb, ich, NL);                                                          \
            /* all but the pair just requested has landed: chunks k+2 and k+3 */                         \
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * IPW) : "memory");                    \
            __builtin_amdgcn_s_barrier();                                                                \
            asm volatile("" ::: "memory");                                                               \
            PR_HALF(1, s2, 0, 0, 0, 0, NL);                                                              \
            sb = s2;                                                                                     \
        }                                                                                                \
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                                      \
    }
    // Row tiles of this wavefront that hold a row of the launch: the loop exists once per count, so that the row
    // count of a step that the host only knows an upper bound of (device-side M) costs what its rows cost.  Every
    // copy runs the same barriers and the same requests.
    const int nl = __builtin_amdgcn_readfirstlane(min(max((M - m0 - wh * THW * 32 + 31) >> 5, 0), THW));
#define PR_CASE(k)                                                                                       \
    case k:                                                                                              \
        if constexpr ((k) <= THW) { PR_MAIN(k) }                                                         \
        break;
    switch (nl) {
        PR_CASE(0) PR_CASE(1) PR_CASE(2) PR_CASE(3) PR_CASE(4) PR_CASE(5) PR_CASE(6)
        default: break;
    }
    static_assert(THW <= 6, "one copy of the loop per live-tile count");
#undef PR_CASE
#undef PR_MAIN
#undef PR_CHUNK
#undef PR_ISSUE1
#undef PR_READ_ONE
#undef PR_HALF
#undef PR_NEXT
    __syncthreads();
    lm_epilogue<WV, WH, TVW, THW>(p, acc, ring, v0, m0, M, vt, wv, wh, n, hi, tid);
}

// One workgroup per row: merge the per-vocabulary-tile partials (contiguous per row) in a fixed order: every thread
// takes the tiles t = tid, tid + 256, ... (all loads issued before the first merge), then a fixed tree over the
// lanes and the four wavefronts.  The merge is associative and its tie rule (lowest index) does not depend on order.
__global__ __launch_bounds__(256) void lmhead_reduce_kernel(LmParams p) {
    __shared__ f32x4 s_red[4], s_smp[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = blockIdx.x;
    int M = p.M;
    int n_vt = p.n_vt;
    const f32x4* part2 = p.part2;
    if (p.m_dev) {
        const int md = max(*p.m_dev, 0);
        M = min(M, md);
        if (p.alt_cap > 0 && md <= p.alt_cap) {
            n_vt = p.alt_n_vt;
            part2 = p.alt_part2;
        }
    }
    if (r >= M) return;
    const bool ent = p.conf_mode == DLM_CONF_NEG_ENTROPY;
    const bool second = p.sample || ent;
    const f32x4* row = p.part + (int64_t)r * n_vt;
    const f32x4* row2 = part2 + (int64_t)r * n_vt;
    Red tot{-INFINITY, 0.f, -INFINITY, 0x7fffffff};
    Smp sm{-INFINITY, -INFINITY, 0x7fffffff};
    float uent = 0.f;
    for (int t0 = 0; t0 < n_vt; t0 += 1024) {
        f32x4 v[4], g[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int t = t0 + a * 256 + tid;
            v[a] = f32x4{-INFINITY, 0.f, -INFINITY, __int_as_float(0x7fffffff)};
            g[a] = f32x4{-INFINITY, -INFINITY, __int_as_float(0x7fffffff), 0.f};
            if (t < n_vt) {
                v[a] = row[t];
                if (second) g[a] = row2[t];
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const Red o{v[a][0], v[a][1], v[a][2], __float_as_int(v[a][3])};
            if (ent) uent = u_merge(tot, uent, o, g[a][3]);
            tot = red_merge(tot, o);
            if (p.sample) sm = smp_merge(sm, Smp{g[a][0], g[a][1], __float_as_int(g[a][2])});
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const Red o = red_shfl_xor(tot, off);
        if (ent) uent = u_merge(tot, uent, o, shfl_xor(uent, off));
        tot = red_merge(tot, o);
        if (p.sample) {
            Smp so;
            so.pm = shfl_xor(sm.pm, off);
            so.pz = shfl_xor(sm.pz, off);
            so.idx = shfl_xor(sm.idx, off);
            sm = smp_merge(sm, so);
        }
    }
    if (lane == 0) {
        s_red[w] = f32x4{tot.m, tot.s, tot.m2, __int_as_float(tot.idx)};
        s_smp[w] = f32x4{sm.pm, sm.pz, __int_as_float(sm.idx), uent};
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int k = 1; k < 4; ++k) {
            const f32x4 o = s_red[k], g = s_smp[k];
            const Red ro{o[0], o[1], o[2], __float_as_int(o[3])};
            if (ent) uent = u_merge(tot, uent, ro, g[3]);
            tot = red_merge(tot, ro);
            sm = smp_merge(sm, Smp{g[0], g[1], __float_as_int(g[2])});
        }
        const int64_t oidx = (p.out_scatter && p.row_idx) ? (int64_t)p.row_idx[r] : (int64_t)r;
        float conf;
        if (p.conf_mode == DLM_CONF_MARGIN) {
            // p(top-1) - p(top-2) = (1 - exp(z2nd - zmax)) / sum_v exp(z_v - zmax)
            conf = (1.0f - __expf(tot.m2 - tot.m)) / tot.s;
        } else if (ent) {
            conf = uent / tot.s - logf(tot.s);      // sum_v p_v log p_v
        } else if (p.sample) {
            // probability of the sampled token: exp(z_tok - lse) = exp(z_tok - zmax) / sum_v exp(z_v - zmax)
            conf = __expf(sm.pz - tot.m) / tot.s;
        } else {
            conf = 1.0f / tot.s;                    // exp(zmax - lse) = 1 / sum_v exp(z_v - zmax)
        }
        p.conf[oidx] = conf;
        p.tok[oidx] = p.sample ? sm.idx : tot.idx;
        if (p.lse) p.lse[oidx] = tot.m + logf(tot.s);
        if (p.zmax) p.zmax[oidx] = tot.m;
        if (p.z2nd) p.z2nd[oidx] = tot.m2;
    }
}

struct LmVariant {
    int tv, mb, threads;
    int half;   // table entry with the same rows and half the vocabulary tile height (for the tail of a launch), -1: none
    void (*launch)(dim3, hipStream_t, const LmParams&);
    // The same shape with W fetched by non-temporal loads, for launches with ONE row chunk, where every element of
    // W is used exactly once: W then streams through L2 without being kept.  Measured on one box, V = 126464,
    // Dh = 4096: 192 -> 170 us at M <= 64, 198 -> 180 at 96, 203 -> 188 at 128, 236 -> 228 at 160 - 192 rows.  With
    // several row chunks W is re-read from L2 and the hint costs 30 - 40 %; in the direct-to-LDS ring it undoes the
    // pairing of half-line requests (268 -> 305 us at 256 rows).  Null where the shape has no such form.
    void (*launch_nt)(dim3, hipStream_t, const LmParams&);
};
template <int WV, int WH, int TVW, int THW, int PD, int KCH = 64, int OCC = 1, bool PIPE = false, bool NTW = false>
static void launch_lm(dim3 grid, hipStream_t st, const LmParams& p) {
    hipLaunchKernelGGL((lmhead_kernel<WV, WH, TVW, THW, PD, KCH, OCC, PIPE, NTW>), grid, dim3(64 * WV * WH), 0, st, p);
}
#define LMP(WV, WH, TVW, THW, PD) {32 * TVW * WV, 32 * THW * WH, 64 * WV * WH, -1, launch_lm<WV, WH, TVW, THW, PD, 64, 1, true>, launch_lm<WV, WH, TVW, THW, PD, 64, 1, true, true>}
template <int WV, int TVW, int THW, int PDW>
static void launch_lmd(dim3 grid, hipStream_t st, const LmParams& p) {
    hipLaunchKernelGGL((lmhead_wdirect_kernel<WV, TVW, THW, PDW>), grid, dim3(64 * WV), 0, st, p);
}
#define LMD(WV, TVW, THW, PDW) {32 * TVW * WV, 32 * THW, 64 * WV, -1, launch_lmd<WV, TVW, THW, PDW>, nullptr}
template <int WV, int WH, int TVW, int THW, int NS, bool XB = false>
static void launch_lma(dim3 grid, hipStream_t st, const LmParams& p) {
    hipLaunchKernelGGL((lmhead_dma_kernel<WV, WH, TVW, THW, NS, XB>), grid, dim3(64 * WV * WH), 0, st, p);
}
#define LMA(WV, WH, TVW, THW, NS) {32 * TVW * WV, 32 * THW * WH, 64 * WV * WH, -1, launch_lma<WV, WH, TVW, THW, NS>, nullptr}
#define LMX(WV, WH, TVW, THW, NS) {32 * TVW * WV, 32 * THW * WH, 64 * WV * WH, -1, launch_lma<WV, WH, TVW, THW, NS, true>, nullptr}
template <int WV, int WH, int TVW, int THW>
static void launch_lmq(dim3 grid, hipStream_t st, const LmParams& p) {
    hipLaunchKernelGGL((lmhead_pair_kernel<WV, WH, TVW, THW>), grid, dim3(64 * WV * WH), 0, st, p);
}
#define LMQ(WV, WH, TVW, THW) {32 * TVW * WV, 32 * THW * WH, 64 * WV * WH, -1, launch_lmq<WV, WH, TVW, THW>, nullptr}
#define LMV(WV, WH, TVW, THW, PD) {32 * TVW * WV, 32 * THW * WH, 64 * WV * WH, -1, launch_lm<WV, WH, TVW, THW, PD>, launch_lm<WV, WH, TVW, THW, PD, 64, 1, false, true>}
static const LmVariant g_lm_variants[] = {
    // shapes the planner uses, by row count M (V = 126464, Dh = 4096 on MI355X, us per main-kernel launch in the
    // rollout, non-temporal W stream; entries 22, 20 above 256 rows):
    /*0*/ LMV(4, 1, 1, 1, 3),   // M <= 32   128 x 32 tile,  4 waves            ~161
    /*1*/ LMP(4, 1, 1, 2, 3),   // M <= 64   128 x 64,       4 waves            ~159
    /*2*/ LMP(8, 1, 1, 3, 3),   // M <= 96   256 x 96,       8 waves            ~166
    /*3*/ LMP(4, 2, 2, 2, 3),   // M <= 128  256 x 128,      8 waves            ~172
    /*4*/ LMP(4, 2, 2, 3, 2),   // M <= 192  256 x 192,      8 waves            ~203
    /*5*/ LMP(4, 2, 2, 4, 2),   // M <= 256  256 x 256,      8 waves            ~245
    // alternatives kept for tests and tuning sweeps
    /*6*/ LMV(2, 2, 2, 4, 3),   // 128 x 256, 4 waves, stores before the MFMA block
    /*7*/ LMD(4, 1, 1, 3),      // W fragments straight from global memory, 128 x 32
    /*8*/ LMD(4, 2, 4, 3),      // same, 256 x 128
    /*9*/ LMD(4, 2, 8, 2),      // same, 256 x 256
    /*10*/ LMA(2, 2, 4, 4, 4),  // direct-to-LDS ring, 256 x 256, 4 waves x (128 x 128), 4 stages
    /*11*/ LMA(2, 2, 4, 4, 3),  // same, 3 stages
    /*12*/ LMA(2, 4, 4, 2, 4),  // 8 waves x (128 x 64)
    /*13*/ LMA(4, 2, 2, 4, 4),  // 8 waves x (64 x 128)
    /*14*/ LMA(2, 2, 2, 4, 4),  // 128 x 256, 4 waves x (64 x 128)
    /*15*/ LMA(2, 2, 4, 2, 4),  // 256 x 128, 4 waves x (128 x 64)
    /*16*/ LMA(4, 4, 2, 2, 4),  // 256 x 256, 16 waves x (64 x 64): four wavefronts per SIMD, 118 registers each
    /*17*/ LMA(4, 4, 2, 2, 3),  // same, 3 stages      (both within 3 % of entry 5 from M = 224 to 8192)
    /*18*/ LMX(2, 2, 4, 4, 4),  // entry 10 with the operand fragments read one MFMA step ahead, across the barrier
    /*19*/ LMX(4, 2, 2, 4, 4),  // entry 13 likewise
    /*20*/ LMQ(2, 2, 4, 4),     // paired, evenly spread requests, 5 stages: 256 x 256, 4 waves x (128 x 128)
    /*21*/ LMQ(4, 2, 2, 4),     // same, 8 waves x (64 x 128): one 256-row chunk as fast as entry 5, with 1.47 x the HBM fetch
    /*22*/ LMQ(4, 1, 2, 6),     // 256 x 192, 4 waves x (64 x 192)
    /*23*/ LMQ(4, 1, 2, 4),     // 256 x 128, 4 waves x (64 x 128)
    // half-height forms of entries 2, 3, 4, 21 and 5 (128 vocabulary rows): the tail of a launch whose tile count leaves
    // at most half of the CUs busy in its last round (see launch_lm_shape)
    /*24*/ LMP(4, 1, 1, 3, 3),  // 128 x 96,  4 waves
    /*25*/ LMP(4, 2, 1, 2, 3),  // 128 x 128, 8 waves
    /*26*/ LMP(4, 2, 1, 3, 2),  // 128 x 192, 8 waves
    /*27*/ LMQ(4, 2, 1, 4),     // 128 x 256, paired ring, 8 waves x (32 x 128)
    /*28*/ LMP(4, 2, 1, 4, 2),  // 128 x 256, register-staged, 8 waves
};
// entry -> its half-height form
static int lm_half_of(int v) { return v == 2 ? 24 : v == 3 ? 25 : v == 4 ? 26 : v == 21 ? 27 : v == 5 ? 28 : -1; }
#undef LMV
#undef LMA
#undef LMX
#undef LMQ
#undef LMP
#undef LMD
constexpr int N_LM_VARIANTS = sizeof(g_lm_variants) / sizeof(g_lm_variants[0]);
constexpr int LM_MIN_TV = 128;   // smallest vocabulary tile of any variant: sizes the workspace
int g_lm_variant = -1;           // -1 = choose by M; otherwise force an entry of the table (dlm_set_option)
int g_lm_nt = 1;                 // 1 = non-temporal W loads when there is one row chunk (default); 0 = never (tuning)
int g_lm_block_gv = -1;          // -1 = automatic XCD blocking; 0 = none; n = n vocabulary tiles per block (tuning)
int g_lm_cus = 0;                // CUs the tail rule assumes: 0 = the device's count; -1 = no half-height tail (tuning, tests)

static int plan_lmhead(int M) {
    if (g_lm_variant >= 0) return g_lm_variant;
    if (M <= 32) return 0;
    if (M <= 64) return 1;
    if (M <= 96) return 2;
    if (M <= 128) return 3;
    if (M <= 192) return 4;
    if (M <= 256) return 5;         // one 256-row chunk, register-staged: as fast as the ring (entry 21), which fetches 1.3 - 1.5 x W here
    if (M <= 384) return 22;        // two 192-row chunks
    return 20;                      // 256-row chunks, one wavefront per SIMD with a 128 x 128 tile
}

static int validate_lm(const dlm_lmhead_args* a) {
    if (!a) return fail(DLM_ERR_INVALID_ARG, "lmhead: null args");
    if (a->struct_size != sizeof(dlm_lmhead_args))
        return fail(DLM_ERR_INVALID_ARG, "lmhead: struct_size %u != %zu", a->struct_size, sizeof(dlm_lmhead_args));
    if (a->M < 0 || a->Dh <= 0 || a->V <= 0) return fail(DLM_ERR_INVALID_ARG, "lmhead: bad sizes M=%d Dh=%d V=%d", a->M, a->Dh, a->V);
    if (a->Dh % KC) return fail(DLM_ERR_UNSUPPORTED, "lmhead: Dh=%d is not a multiple of %d", a->Dh, KC);
    if (a->forbid_token >= a->V) return fail(DLM_ERR_INVALID_ARG, "lmhead: forbid_token %d >= V", a->forbid_token);
    if (a->forbid_token >= 0 && a->V < 2) return fail(DLM_ERR_INVALID_ARG, "lmhead: forbid_token with V < 2 leaves no token");
    if (!(a->inv_temperature > 0.f) || a->inv_temperature > 3.0e38f) return fail(DLM_ERR_INVALID_ARG, "lmhead: inv_temperature must be positive and finite");
    if ((a->target == nullptr) != (a->ztarget == nullptr)) return fail(DLM_ERR_INVALID_ARG, "lmhead: target and ztarget go together");
    if (a->sample != 0 && a->sample != 1) return fail(DLM_ERR_INVALID_ARG, "lmhead: sample must be 0 or 1");
    if (a->conf_mode < DLM_CONF_TOKEN_PROB || a->conf_mode > DLM_CONF_NEG_ENTROPY)
        return fail(DLM_ERR_INVALID_ARG, "lmhead: unknown conf_mode %d", a->conf_mode);
    if (a->M == 0) return DLM_OK;
    if (!a->hidden || !a->w || !a->conf || !a->tok) return fail(DLM_ERR_INVALID_ARG, "lmhead: null hidden/w/conf/tok");
    if (!aligned16(a->hidden) || !aligned16(a->w)) return fail(DLM_ERR_UNSUPPORTED, "lmhead: hidden/w not 16-byte aligned");
    if ((a->hidden_stride_row | a->w_stride_row) % 8) return fail(DLM_ERR_UNSUPPORTED, "lmhead: strides must be multiples of 8");
    if (a->hidden_stride_row < a->Dh || a->w_stride_row < a->Dh) return fail(DLM_ERR_INVALID_ARG, "lmhead: row stride < Dh");
    return DLM_OK;
}

}  // namespace dlm

using namespace dlm;

// largest row count served by the shape plan_lmhead picks for M rows
static int plan_capacity(int M) {
    static const int caps[] = {32, 64, 96, 128, 192, 256, 384};
    for (int c : caps)
        if (M <= c) return c;
    return 0x7fffffff;
}

// Launches one kernel shape over n_vt_l vocabulary tiles that begin at row v_first (partials vt0 ...).
static int launch_lm_tiles(const LmVariant& var, LmParams& p, int n_vt_l, int vt0, int v_first, hipStream_t st) {
    p.n_vt_l = n_vt_l; p.vt0 = vt0; p.v_first = v_first;
    // several row chunks: blocks of gm x gv workgroups for the 32 CUs of an XCD; gm is the largest divisor of the
    // chunk count up to 8 (measured at V = 126464, Dh = 4096: +6 % at M >= 1024, +10..17 % at M = 512)
    p.gm = 1; p.gv = 1;
    if (p.n_mc >= 2) {
        for (int c = 8; c >= 1; --c)
            if (p.n_mc % c == 0) { p.gm = c; break; }
        p.gv = 32 / p.gm > 8 ? 8 : 32 / p.gm;
    }
    if (g_lm_block_gv >= 0) { p.gv = g_lm_block_gv > 0 ? g_lm_block_gv : 1; if (g_lm_block_gv == 0) p.gm = 1; }
    const int64_t n_vt8 = ((int64_t)(n_vt_l + 7) / 8 + p.gv - 1) / p.gv * p.gv;   // vocabulary tiles per XCD, padded to gv
    const int64_t n_wg = n_vt8 * 8 * p.n_mc;
    if (n_wg > 0x7fffffff) return fail(DLM_ERR_UNSUPPORTED, "lmhead: M * V too large for one launch");
    ((p.n_mc == 1 && var.launch_nt && g_lm_nt) ? var.launch_nt : var.launch)(dim3((unsigned)n_wg), st, p);
    return check_hip(hipGetLastError(), "lmhead_kernel launch");
}

static int device_cus() {
    static int cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        cus[dev] = (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
    }
    return cus[dev];
}

// Fills the layout fields of p for one kernel shape (p.M = the rows this launch may hold, m_bound = the caller's
// bound, which places the second partials) and launches it.
// Tail rule: the shapes for 65 - 256 rows run one workgroup per CU, so a launch costs ceil(tiles / CUs) rounds of
// equal length.  When the last round would occupy at most half of the CUs (V = 152064: 594 tiles = 2.32 rounds on 256
// CUs, V = 157184: 614 = 2.40), the tiles of that round are launched at half height instead (a second launch of the
// shape's 128-row form on twice as many tiles): 2.5 rounds' time instead of 3.
static int launch_lm_shape(int v_idx, LmParams& p, int m_bound, hipStream_t st) {
    const LmVariant& var = g_lm_variants[v_idx];
    const int n_full = (p.V + var.tv - 1) / var.tv;
    p.n_mc = (p.M + var.mb - 1) / var.mb;
    const int half = lm_half_of(v_idx);
    const int cus = g_lm_cus > 0 ? g_lm_cus : device_cus();
    const int tail = n_full % cus;
    if (g_lm_cus >= 0 && half >= 0 && p.n_mc == 1 && n_full > cus && tail > 0 && 2 * tail <= cus) {
        const int n_main = n_full - tail, v_split = n_main * var.tv;
        const int n_half = (p.V - v_split + var.tv / 2 - 1) / (var.tv / 2);
        p.n_vt = n_main + n_half;
        p.part2 = p.part + (size_t)p.n_vt * m_bound;
        int rc = launch_lm_tiles(var, p, n_main, 0, 0, st);
        if (rc != DLM_OK) return rc;
        return launch_lm_tiles(g_lm_variants[half], p, n_half, n_main, v_split, st);
    }
    p.n_vt = n_full;
    p.part2 = p.part + (size_t)p.n_vt * m_bound;
    return launch_lm_tiles(var, p, n_full, 0, 0, st);
}

extern "C" size_t dlm_lmhead_workspace_bytes(const dlm_lmhead_args* a) {
    if (!a || a->M <= 0 || a->V <= 0) return 0;
    const size_t n_vt = ((size_t)a->V + LM_MIN_TV - 1) / LM_MIN_TV;   // enough for every kernel shape
    return n_vt * (size_t)a->M * sizeof(f32x4) * ((a->sample || a->conf_mode == DLM_CONF_NEG_ENTROPY) ? 2 : 1);
}

// Enqueues the main kernel(s) and the reduction of one call; `workspace` holds the per-tile partials.
static int lmhead_enqueue(const dlm_lmhead_args* a, void* workspace, void* stream) {
    int rc;
    LmParams p;
    p.M = a->M; p.Dh = a->Dh; p.V = a->V;
    p.hidden = (const uint16_t*)a->hidden; p.h_stride = a->hidden_stride_row;
    p.row_idx = a->row_idx; p.m_dev = a->m_dev;
    p.w = (const uint16_t*)a->w; p.w_stride = a->w_stride_row;
    p.inv_t = a->inv_temperature; p.forbid = a->forbid_token; p.out_scatter = a->out_scatter;
    p.conf = a->conf; p.tok = a->tok; p.lse = a->lse; p.zmax = a->zmax; p.z2nd = a->z2nd;
    p.target = a->target; p.ztarget = a->ztarget;
    p.part = (f32x4*)workspace;
    p.sample = a->sample;
    p.conf_mode = a->conf_mode;
    p.seed_lo = (uint32_t)a->sample_seed; p.seed_hi = (uint32_t)(a->sample_seed >> 32);
    p.step = a->sample_step; p.stream = a->sample_stream;
    p.m_lo = -1; p.m_hi = 0x7fffffff;
    p.alt_cap = 0; p.alt_n_vt = 0; p.alt_part2 = nullptr;
    hipStream_t st = (hipStream_t)stream;

    // The caller's bound M sizes the launch, the device's count says how many rows there are.  When the caller
    // expects the count to fall in a smaller shape's range, that shape is queued first, guarded by "count <= its
    // capacity", and the bound's shape after it, guarded by the opposite: one of the two returns at once.
    const int v_safe = plan_lmhead(a->M);
    int v_try = v_safe, cap = 0;
    if (a->m_dev && a->M_expected > 0 && a->M_expected < a->M && g_lm_variant < 0) {
        cap = plan_capacity(a->M_expected);
        if (cap < a->M) v_try = plan_lmhead(cap);
    }
    if (v_try != v_safe) {
        LmParams q = p;
        q.M = cap;
        q.m_hi = cap;
        rc = launch_lm_shape(v_try, q, a->M, st);
        if (rc != DLM_OK) return rc;
        p.m_lo = cap;
        p.alt_cap = cap; p.alt_n_vt = q.n_vt; p.alt_part2 = q.part2;
    }
    rc = launch_lm_shape(v_safe, p, a->M, st);
    if (rc != DLM_OK) return rc;
    hipLaunchKernelGGL(lmhead_reduce_kernel, dim3(a->M), dim3(256), 0, st, p);
    return check_hip(hipGetLastError(), "lmhead_reduce_kernel launch");
}

extern "C" int dlm_lmhead_confidence(const dlm_lmhead_args* a, void* stream) {
    int rc = validate_lm(a);
    if (rc != DLM_OK) return rc;
    if (a->M == 0) return DLM_OK;
    const size_t need = dlm_lmhead_workspace_bytes(a);
    if (!a->workspace || a->workspace_bytes < need)
        return fail(DLM_ERR_WORKSPACE, "lmhead: workspace of %zu bytes needed, %zu given", need, a->workspace ? a->workspace_bytes : (size_t)0);
    if (!aligned16(a->workspace)) return fail(DLM_ERR_WORKSPACE, "lmhead: workspace not 16-byte aligned");
    return lmhead_enqueue(a, a->workspace, stream);
}

// ---- the variant that allocates nothing ------------------------------------------------------------------
// The per-tile partials live in a file-scope device array instead of a caller-provided workspace.  Every GPU the
// library runs on holds its own copy of the array (at its own address) until the process ends; the address is
// looked up once per device, with that device current, and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[DLM_LMHEAD_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];   // per device: device address of `scratch` (null until looked up)

extern "C" size_t dlm_lmhead_static_scratch_bytes(void) { return sizeof(scratch); }

extern "C" int dlm_lmhead_confidence_static(const dlm_lmhead_args* a, void* stream) {
    int rc = validate_lm(a);
    if (rc != DLM_OK) return rc;
    if (a->M == 0) return DLM_OK;
    const size_t need = dlm_lmhead_workspace_bytes(a);
    if (need > sizeof(scratch))
        return fail(DLM_ERR_WORKSPACE, "lmhead (static scratch): M=%d rows x V=%d needs %zu bytes of partials, the built-in "
                    "scratch holds %zu; use dlm_lmhead_confidence with a workspace", a->M, a->V, need, sizeof(scratch));
    int dev = -1;
    if ((rc = check_hip(hipGetDevice(&dev), "hipGetDevice")) != DLM_OK) return rc;
    if (dev < 0 || dev >= MAX_DEVICES) return fail(DLM_ERR_UNSUPPORTED, "lmhead (static scratch): device index %d", dev);
    void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        if ((rc = check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) != DLM_OK) return rc;
        if (!ptr || !aligned16(ptr)) return fail(DLM_ERR_HIP, "lmhead (static scratch): bad symbol address");
        __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);
    }
    return lmhead_enqueue(a, ptr, stream);
}

namespace dlm {
int lm_set_block(int v) {
    if (v < -1 || v > 8) return fail(DLM_ERR_INVALID_ARG, "set_option: lmhead_block must be -1..8");
    g_lm_block_gv = v;
    return DLM_OK;
}
int lm_set_cus(int v) {
    if (v < -1 || v > 4096) return fail(DLM_ERR_INVALID_ARG, "set_option: lmhead_cus must be -1..4096");
    g_lm_cus = v;
    return DLM_OK;
}
int lm_set_nt(int v) {
    if (v < 0 || v > 1) return fail(DLM_ERR_INVALID_ARG, "set_option: lmhead_nt must be 0 or 1");
    g_lm_nt = v;
    return DLM_OK;
}
int lm_set_variant(int v) {
    if (v < -1 || v >= N_LM_VARIANTS) return fail(DLM_ERR_INVALID_ARG, "set_option: lmhead_variant must be -1..%d", N_LM_VARIANTS - 1);
    g_lm_variant = v;
    return DLM_OK;
}
}  // namespace dlm
