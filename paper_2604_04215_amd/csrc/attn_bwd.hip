// dlm_block_attn_bwd: gradients of block attention (dQ, and dK / dV per KV segment).
//
// With P = softmax(scale Q K^T + mask), O = P V and an upstream gradient dO:
//   delta_r = sum_c dO[r,c] O[r,c]                  (= rowsum(dP * P))
//   dV = P^T dO,  dP = dO V^T,  dS = P * (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
// P is recomputed from Q, K and the forward pass's log-sum-exp; nothing of size Lq x Lk is stored.
//
// Three kernels, no atomics, every output element written exactly once (deterministic):
//   * attn_bwd_delta_kernel : delta per (sequence, head, query row).
//   * attn_bwd_dq_kernel    : a workgroup owns 128 rows (query, head in group) of one (sequence, KV head) and
//                             walks the key tiles of all segments, like the forward kernel.  Per 32-key tile and
//                             wavefront: S^T = K Q^T and dP^T = V dO^T (keys are the MFMA rows, so a lane holds 16
//                             keys of ONE query row and LSE / delta are per-lane scalars), dS^T in registers is
//                             already the B operand of dQ^T += K^T dS^T; K^T fragments come from LDS through the
//                             transposing 64-bit LDS read.
//   * attn_bwd_dkv_kernel   : the mirror image, run once for dV and once for dK.  A workgroup owns 128 keys of
//                             ONE segment of one (sequence, KV head), each wavefront 32 of them, and walks the
//                             32-row tiles of (query, head in group) rows that can see them: S = Q K^T and
//                             dP = dO V^T (rows are the MFMA rows, a lane holds 16 rows of ONE key), P and dS in
//                             registers are the B operands of dV^T += dO^T P and dK^T += Q^T dS; the sum over the
//                             heads of a group happens in the accumulators because the rows of all its heads pass
//                             through the same workgroup.
#include "common.hpp"

namespace dlm {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;

struct BwdSeg {
    const uint16_t *k, *v;
    uint16_t *dk, *dv;
    int len, pos0;
    int64_t sb, sh, st;
    int rule;
};

struct BwdParams {
    int B, Lq, Hq, Hkv, g, R;
    const uint16_t *q, *o, *dout;
    int64_t q_sb, q_st, q_sh, o_sb, o_st, o_sh, do_sb, do_st, do_sh;
    uint16_t* dq;
    int64_t dq_sb, dq_st, dq_sh;
    BwdSeg seg[3];
    const float* lse;
    float* delta;
    int bs, q_pos0;
    float scale, scale_log2;
    const int32_t* cu;
    int total;
};

__device__ __forceinline__ bf16x8 bw_as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } x;
    x.u = v;
    return x.b;
}

// index of (sequence b, head h, query row i) in the LSE / delta arrays; s0 = first token of the sequence (packed mode)
__device__ __forceinline__ int64_t stat_index(const BwdParams& p, int b, int h, int i, int s0) {
    return p.cu ? (int64_t)h * p.total + s0 + i : ((int64_t)b * p.Hq + h) * p.Lq + i;
}

// ---------------------------------------------------------------------------------------------------------
// delta[b, h, i] = sum_c dO * O.  D / 8 lanes per row, 16-byte loads.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(BwdParams p) {
    constexpr int LPR = D / 8;             // lanes per row
    constexpr int RPB = 256 / LPR;         // rows per workgroup
    const int b = blockIdx.z;
    int s0 = 0, sl = p.Lq;
    int64_t o_off = b * p.o_sb, do_off = b * p.do_sb;
    if (p.cu) {
        s0 = min(max(p.cu[b], 0), p.total);
        sl = max(min(min(p.cu[b + 1], p.total) - s0, p.Lq), 0);
        o_off = s0 * p.o_st;
        do_off = s0 * p.do_st;
    }
    const int row = blockIdx.x * RPB + threadIdx.x / LPR;   // row = i * Hq + h
    const int c = threadIdx.x % LPR;
    const int i = row / p.Hq, h = row - i * p.Hq;
    float acc = 0.f;
    if (i < sl) {
        const u32x4 a = *reinterpret_cast<const u32x4*>(p.o + o_off + i * p.o_st + (int64_t)h * p.o_sh + c * 8);
        const u32x4 d = *reinterpret_cast<const u32x4*>(p.dout + do_off + i * p.do_st + (int64_t)h * p.do_sh + c * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += bf16_bits_to_f32(a[e] & 0xffffu) * bf16_bits_to_f32(d[e] & 0xffffu);
            acc += bf16_bits_to_f32(a[e] >> 16) * bf16_bits_to_f32(d[e] >> 16);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) acc += shfl_xor(acc, off);
    if (i < sl && c == 0) p.delta[stat_index(p, b, h, i, s0)] = acc;
}

// ---------------------------------------------------------------------------------------------------------
template <int D, bool BC>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(BwdParams p, GridRemap rm) {
    constexpr int KP = D * 2 + 16;         // row-read image pitch (bytes)
    constexpr int TP = D * 2 + 64;         // transposing-read image pitch
    constexpr int C8 = D / 8;
    constexpr int NLD = (32 * C8) / 256;   // 16-byte chunks per thread per 32-row tile
    constexpr int OPB = D * 2 + 16;        // output staging row pitch (bytes)
    constexpr int TILES_BYTES = 2 * 32 * KP + 32 * TP, STAGE_BYTES = 4 * 32 * OPB + 4 * 32 * 8;
    __shared__ __attribute__((aligned(16))) unsigned char smem[TILES_BYTES > STAGE_BYTES ? TILES_BYTES : STAGE_BYTES];
    unsigned char* Krow = smem;
    unsigned char* Vrow = smem + 32 * KP;
    unsigned char* Ktr = smem + 2 * 32 * KP;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = lane & 31, hi = lane >> 5;
    int b = blockIdx.z, kvh = blockIdx.y, bx0 = blockIdx.x;
    if (rm.nx > 0) {
        int grp;
        if (!remap_decode(rm, p.B * p.Hkv, grp, bx0)) return;
        kvh = grp % p.Hkv;
        b = grp / p.Hkv;
    }
    const int r0 = bx0 * 128;

    int len0 = p.seg[0].len, len1 = p.seg[1].len, len2 = p.seg[2].len;
    int R = p.R, s0 = 0;
    int64_t q_off = b * p.q_sb, do_off = b * p.do_sb, dq_off = b * p.dq_sb, kv1_off = b * p.seg[1].sb;
    if (p.cu) {
        s0 = min(max(p.cu[b], 0), p.total);
        const int sl = max(min(min(p.cu[b + 1], p.total) - s0, p.Lq), 0);
        R = p.g * sl;
        if (r0 >= R) return;
        len1 = min(len1, sl);
        q_off = s0 * p.q_st;
        do_off = s0 * p.do_st;
        dq_off = s0 * p.dq_st;
        kv1_off = s0 * p.seg[1].st;
    }
    int F0 = 0, F1 = 0, F2 = 0, ho0 = 0, ho1 = 0, ho2 = 0;
    bool same0 = false, same1 = false, same2 = false;
    if (BC) {
        const int rows_end = min(r0 + 128, R);
        const int lim = ((p.q_pos0 + (rows_end - 1) / p.g) / p.bs + 1) * p.bs;
        const int first = ((p.q_pos0 + r0 / p.g) / p.bs) * p.bs;
        ho0 = (p.seg[0].rule == DLM_SEG_EARLIER_BLOCKS) ? p.bs : 0;
        ho1 = (p.seg[1].rule == DLM_SEG_EARLIER_BLOCKS) ? p.bs : 0;
        ho2 = (p.seg[2].rule == DLM_SEG_EARLIER_BLOCKS) ? p.bs : 0;
        same0 = p.seg[0].rule == DLM_SEG_SAME_BLOCK;
        same1 = p.seg[1].rule == DLM_SEG_SAME_BLOCK;
        same2 = p.seg[2].rule == DLM_SEG_SAME_BLOCK;
        len0 = max(0, min(len0, lim - ho0 - p.seg[0].pos0));
        len1 = max(0, min(len1, lim - ho1 - p.seg[1].pos0));
        len2 = max(0, min(len2, lim - ho2 - p.seg[2].pos0));
        if (same0) F0 = min(max(first - p.seg[0].pos0, 0) >> 5, (len0 + 31) >> 5);
        if (same1) F1 = min(max(first - p.seg[1].pos0, 0) >> 5, (len1 + 31) >> 5);
        if (same2) F2 = min(max(first - p.seg[2].pos0, 0) >> 5, (len2 + 31) >> 5);
    }
    const int T0 = ((len0 + 31) >> 5) - F0, T1 = ((len1 + 31) >> 5) - F1, T2 = ((len2 + 31) >> 5) - F2;
    const int T = T0 + T1 + T2;

    const uint16_t* kb0 = p.seg[0].k + b * p.seg[0].sb + kvh * p.seg[0].sh;
    const uint16_t* vb0 = p.seg[0].v + b * p.seg[0].sb + kvh * p.seg[0].sh;
    const uint16_t* kb1 = p.seg[1].k + kv1_off + kvh * p.seg[1].sh;
    const uint16_t* vb1 = p.seg[1].v + kv1_off + kvh * p.seg[1].sh;
    const uint16_t* kb2 = p.seg[2].k + b * p.seg[2].sb + kvh * p.seg[2].sh;
    const uint16_t* vb2 = p.seg[2].v + b * p.seg[2].sb + kvh * p.seg[2].sh;
    const int64_t st0 = p.seg[0].st, st1 = p.seg[1].st, st2 = p.seg[2].st;
    const int sp0 = __builtin_amdgcn_readfirstlane(p.seg[0].pos0), sp1 = __builtin_amdgcn_readfirstlane(p.seg[1].pos0),
              sp2 = __builtin_amdgcn_readfirstlane(p.seg[2].pos0);

    // ---- this lane's query row: Q and dO fragments (B operands), LSE and delta ----------------------------
    const int r = r0 + w * 32 + n;
    const bool valid = r < R;
    const int qi = valid ? r / p.g : 0;
    const int hg = valid ? r - qi * p.g : 0;
    const int h = kvh * p.g + hg;
    bf16x8 qf[D / 16], dof[D / 16];
    {
        const uint16_t* qp = p.q + q_off + qi * p.q_st + (int64_t)h * p.q_sh;
        const uint16_t* dp = p.dout + do_off + qi * p.do_st + (int64_t)h * p.do_sh;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            u32x4 a = {0, 0, 0, 0}, d = {0, 0, 0, 0};
            if (valid) {
                a = *reinterpret_cast<const u32x4*>(qp + 16 * c + 8 * hi);
                d = *reinterpret_cast<const u32x4*>(dp + 16 * c + 8 * hi);
            }
            qf[c] = bw_as_bf16x8(a);
            dof[c] = bw_as_bf16x8(d);
        }
    }
    float lse2 = INFINITY, delta = 0.f;   // +inf: every probability of an absent row (or one that saw no key) is 0
    if (valid) {
        const int64_t si = stat_index(p, b, h, qi, s0);
        const float l = p.lse[si];
        if (l > -INFINITY) lse2 = l * 1.4426950408889634f;
        delta = p.delta[si];
    }
    const int qlim = BC ? ((p.q_pos0 + qi) / p.bs + 1) * p.bs : 0;
    int qlim_min = 0x7fffffff, qlim_max = 0;
    if (BC) {
        qlim_min = qlim_max = qlim;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            qlim_min = min(qlim_min, shfl_xor(qlim_min, off));
            qlim_max = max(qlim_max, shfl_xor(qlim_max, off));
        }
        qlim_min = __builtin_amdgcn_readfirstlane(qlim_min);
        qlim_max = __builtin_amdgcn_readfirstlane(qlim_max);
    }

    f32x16 dq[D / 32];
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[dt][i] = 0.f;

    u32x4 kreg[NLD], vreg[NLD];
#define BW_TILE(t, sg, lt, slen)                                                                         \
    const int sg = ((t) < T0) ? 0 : (((t) < T0 + T1) ? 1 : 2);                                           \
    const int lt = ((t) < T0) ? (t) + F0 : (((t) < T0 + T1) ? (t) - T0 + F1 : (t) - T0 - T1 + F2);      \
    const int slen = (sg == 0) ? len0 : ((sg == 1) ? len1 : len2);
#define BW_FETCH(t)                                                                                      \
    {                                                                                                    \
        const int tc_ = min((t), T - 1);                                                                 \
        BW_TILE(tc_, sg_, lt_, slen_)                                                                    \
        const uint16_t* kb = (sg_ == 0) ? kb0 : ((sg_ == 1) ? kb1 : kb2);                                \
        const uint16_t* vb = (sg_ == 0) ? vb0 : ((sg_ == 1) ? vb1 : vb2);                                \
        const int64_t stt = (sg_ == 0) ? st0 : ((sg_ == 1) ? st1 : st2);                                 \
        _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                                \
            const int cidx = tid + q * 256;                                                              \
            const int row = cidx / C8, c = cidx - row * C8;                                              \
            const int loc = min(lt_ * 32 + row, slen_ - 1);                                              \
            const int64_t off = loc * stt + c * 8;                                                       \
            kreg[q] = *reinterpret_cast<const u32x4*>(kb + off);                                         \
            vreg[q] = *reinterpret_cast<const u32x4*>(vb + off);                                         \
        }                                                                                                \
    }
#define BW_STORE(t)                                                                                      \
    {                                                                                                    \
        BW_TILE((t), sg_, lt_, slen_)                                                                    \
        (void)sg_;                                                                                       \
        _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                                \
            const int cidx = tid + q * 256;                                                              \
            const int row = cidx / C8, c = cidx - row * C8;                                              \
            const bool live = lt_ * 32 + row < slen_;                                                    \
            const u32x4 z = {0, 0, 0, 0};                                                                \
            const u32x4 kk = live ? kreg[q] : z;                                                         \
            *reinterpret_cast<u32x4*>(Krow + row * KP + c * 16) = kk;                                    \
            *reinterpret_cast<u32x4*>(Ktr + row * TP + c * 16) = kk;                                     \
            *reinterpret_cast<u32x4*>(Vrow + row * KP + c * 16) = live ? vreg[q] : z;                    \
        }                                                                                                \
    }

    if (T > 0) BW_FETCH(0);
    for (int t = 0; t < T; ++t) {
        BW_STORE(t);
        __syncthreads();
        BW_FETCH(t + 1);   // clamped to the last tile: the load is unconditional, its result unused past the end
        f32x16 S, dP;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            S[i] = 0.f;
            dP[i] = 0.f;
        }
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Krow + n * KP + (16 * c + 8 * hi) * 2);
            const bf16x8 vf = *reinterpret_cast<const bf16x8*>(Vrow + n * KP + (16 * c + 8 * hi) * 2);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], S, 0, 0, 0);
            dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[c], dP, 0, 0, 0);
        }
        BW_TILE(t, sg, lt, slen)
        const int spos0 = ((sg == 0) ? sp0 : ((sg == 1) ? sp1 : sp2)) + lt * 32;
        const int hoff = (sg == 0) ? ho0 : ((sg == 1) ? ho1 : ho2);
        const bool same = (sg == 0) ? same0 : ((sg == 1) ? same1 : same2);
        const bool ragged = (lt * 32 + 32 > slen) ||
                            (BC && (spos0 + 31 >= qlim_min - hoff || (same && spos0 < qlim_max - p.bs)));
        if (ragged) {
            const int pbase = spos0 + 4 * hi;
            int hi_r = spos0 - lt * 32 + slen;
            int lo_r = -(1 << 30);
            if (BC) {
                hi_r = min(hi_r, qlim - hoff);
                if (same) lo_r = qlim - p.bs;
            }
            const unsigned span = (unsigned)max(hi_r - lo_r, 0);
            const unsigned off0 = (unsigned)(pbase - lo_r);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (off0 + (unsigned)(8 * (i >> 2) + (i & 3)) >= span) S[i] = -INFINITY;
        }
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float p0 = fast_exp2(fmaf(S[i], p.scale_log2, -lse2));
            const float p1 = fast_exp2(fmaf(S[i + 1], p.scale_log2, -lse2));
            pk[i >> 1] = pack_bf16x2(p0 * (dP[i] - delta), p1 * (dP[i + 1] - delta));
        }
        bf16x8 dsf[2];
        {
            u32x4 lo = {pk[0], pk[1], pk[2], pk[3]}, hi4 = {pk[4], pk[5], pk[6], pk[7]};
            dsf[0] = bw_as_bf16x8(lo);
            dsf[1] = bw_as_bf16x8(hi4);
        }
        const int s16 = lane & 15, blk = (lane >> 4) & 1;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) {
                union { s16x4 h[2]; bf16x8 v; } kt;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int krow = 16 * j2 + 8 * q + 4 * hi + (s16 >> 2);
                    const int dcol = 32 * dt + 16 * blk + 4 * (s16 & 3);
                    kt.h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Ktr + krow * TP + dcol * 2));
                }
                dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt.v, dsf[j2], dq[dt], 0, 0, 0);
            }
        }
        __syncthreads();
    }
#undef BW_TILE
#undef BW_FETCH
#undef BW_STORE

    // dQ^T sits in the accumulators with lane = row: each wavefront transposes its 32 rows through a private LDS
    // region (the tiles are dead: the loop ended with a barrier, or never ran) and stores whole rows, 16 bytes per
    // lane, instead of 64 stores that touch 32 rows with 16 bytes each.
    {
        unsigned char* ob = smem + w * (32 * OPB);
        int64_t* roff = reinterpret_cast<int64_t*>(smem + 4 * 32 * OPB) + w * 32;
        if (hi == 0) roff[n] = valid ? qi * p.dq_st + (int64_t)h * p.dq_sh : (int64_t)-1;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 v;
                v[0] = pack_bf16x2(dq[dt][4 * q4] * p.scale, dq[dt][4 * q4 + 1] * p.scale);
                v[1] = pack_bf16x2(dq[dt][4 * q4 + 2] * p.scale, dq[dt][4 * q4 + 3] * p.scale);
                *reinterpret_cast<u32x2*>(ob + n * OPB + (32 * dt + 8 * q4 + 4 * hi) * 2) = v;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // one wavefront's LDS operations complete in order
#pragma unroll
        for (int q = 0; q < (32 * C8) / 64; ++q) {
            const int id = q * 64 + lane;
            const int row = id / C8, c = id - row * C8;
            const int64_t ro = roff[row];
            const u32x4 v = *reinterpret_cast<const u32x4*>(ob + row * OPB + c * 16);
            if (ro >= 0) *reinterpret_cast<u32x4*>(p.dq + dq_off + ro + 8 * c) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// DK = false: dV of the workgroup's keys (S -> P, dV^T += dO^T P).  DK = true: dK (S, dP -> dS, dK^T += Q^T dS).
// Two passes instead of one: a pass that holds both accumulators (2 x 64 registers at d = 128) next to the K and
// V fragments leaves one wavefront per SIMD or spills, and either way every tile waits out the full memory
// latency; apart, the passes keep two to three workgroups per CU with nothing spilled.  Price: S is formed twice.
template <int D, bool BC, bool DK>
__global__ __launch_bounds__(256, DK ? 2 : 3) void attn_bwd_dkv_kernel(BwdParams p, int sidx, int n_slabs, int pair, GridRemap rm) {
    constexpr int KP = D * 2 + 16;
    constexpr int TP = D * 2 + 64;
    constexpr int C8 = D / 8;
    constexpr int NLD = (32 * C8) / 256;
    // images: Q rows (both passes); DK: Q transposing + dO rows; DV: dO transposing
    constexpr int IMG_BYTES = DK ? (2 * 32 * KP + 32 * TP) : (32 * KP + 32 * TP);
    __shared__ __attribute__((aligned(16))) unsigned char smem[IMG_BYTES + 3 * 32 * 4];
    unsigned char* Qrow = smem;
    unsigned char* Xtr = smem + 32 * KP;              // Q^T source (DK) or dO^T source (DV)
    unsigned char* Grow = smem + 32 * KP + 32 * TP;   // dO rows (DK only)
    float* s_lse2 = reinterpret_cast<float*>(smem + IMG_BYTES);
    float* s_delta = s_lse2 + 32;
    int* s_qlim = reinterpret_cast<int*>(s_delta + 32);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = lane & 31, hi = lane >> 5;
    int b = blockIdx.z, kvh = blockIdx.y, bx = blockIdx.x;
    if (rm.nx > 0) {
        int grp;
        if (!remap_decode(rm, p.B * p.Hkv, grp, bx)) return;
        kvh = grp % p.Hkv;
        b = grp / p.Hkv;
    }
    // plain locals per segment field (a dynamically indexed struct member would go through memory)
    const uint16_t* sk = (sidx == 0) ? p.seg[0].k : ((sidx == 1) ? p.seg[1].k : p.seg[2].k);
    const uint16_t* sv = (sidx == 0) ? p.seg[0].v : ((sidx == 1) ? p.seg[1].v : p.seg[2].v);
    uint16_t* sdk = (sidx == 0) ? p.seg[0].dk : ((sidx == 1) ? p.seg[1].dk : p.seg[2].dk);
    uint16_t* sdv = (sidx == 0) ? p.seg[0].dv : ((sidx == 1) ? p.seg[1].dv : p.seg[2].dv);
    int slen = (sidx == 0) ? p.seg[0].len : ((sidx == 1) ? p.seg[1].len : p.seg[2].len);
    const int spos = (sidx == 0) ? p.seg[0].pos0 : ((sidx == 1) ? p.seg[1].pos0 : p.seg[2].pos0);
    const int64_t ssb = (sidx == 0) ? p.seg[0].sb : ((sidx == 1) ? p.seg[1].sb : p.seg[2].sb);
    const int64_t ssh = (sidx == 0) ? p.seg[0].sh : ((sidx == 1) ? p.seg[1].sh : p.seg[2].sh);
    const int64_t sst = (sidx == 0) ? p.seg[0].st : ((sidx == 1) ? p.seg[1].st : p.seg[2].st);
    const int srule = (sidx == 0) ? p.seg[0].rule : ((sidx == 1) ? p.seg[1].rule : p.seg[2].rule);

    int R = p.R, s0 = 0, Lq = p.Lq;
    int64_t q_off = b * p.q_sb, do_off = b * p.do_sb, kv_off = b * ssb;
    if (p.cu) {
        s0 = min(max(p.cu[b], 0), p.total);
        const int sl = max(min(min(p.cu[b + 1], p.total) - s0, p.Lq), 0);
        R = p.g * sl;
        Lq = sl;
        slen = min(slen, sl);
        q_off = s0 * p.q_st;
        do_off = s0 * p.do_st;
        kv_off = s0 * sst;
    }
    // Under a block-causal mask the work of a key slab shrinks with its index (later keys are seen by fewer rows).
    // pair != 0: a workgroup takes slab x and then slab n_slabs - 1 - x, so every workgroup does the same amount
    // of work and the workgroups of one (sequence, KV head) stay in step on the same Q / dO tiles (L2 reuse).
    // pair == 0: one slab per workgroup; every second group of 8 slabs is taken in reverse so that the 8 XCDs,
    // which get workgroups round-robin, receive equal sums.
    for (int pass = 0; pass < (pair ? 2 : 1); ++pass) {
    int slab = bx;
    if (pair) {
        slab = pass ? n_slabs - 1 - bx : bx;
        if (pass && slab <= bx) break;
    } else {
        const int oct = bx >> 3;
        if ((oct & 1) && (oct * 8 + 7 < n_slabs)) slab = oct * 8 + 7 - (bx & 7);
    }
    const int j0 = slab * 128;                        // first key of this pass inside the segment
    if (j0 >= slen) continue;

    // ---- this lane's key: K (and V) fragments (B operands) ----------------------------------------------------
    const int j = j0 + w * 32 + n;
    const bool kvalid = j < slen;
    bf16x8 kf[D / 16], vf[DK ? D / 16 : 1];
    {
        const uint16_t* kp = sk + kv_off + kvh * ssh + (int64_t)min(j, slen - 1) * sst;
        const uint16_t* vp = sv + kv_off + kvh * ssh + (int64_t)min(j, slen - 1) * sst;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            u32x4 a = {0, 0, 0, 0}, d = {0, 0, 0, 0};
            if (kvalid) {
                a = *reinterpret_cast<const u32x4*>(kp + 16 * c + 8 * hi);
                if (DK) d = *reinterpret_cast<const u32x4*>(vp + 16 * c + 8 * hi);
            }
            kf[c] = bw_as_bf16x8(a);
            if (DK) vf[c] = bw_as_bf16x8(d);
        }
    }
    const int kpos = spos + j;
    const int hoff = (BC && srule == DLM_SEG_EARLIER_BLOCKS) ? p.bs : 0;
    const bool same = BC && srule == DLM_SEG_SAME_BLOCK;

    // ---- rows that can see some key of this workgroup: tiles [rt_begin, rt_end) -----------------------------
    int rt_begin = 0, rt_end = (R + 31) >> 5;
    if (BC) {
        const int kp_first = spos + j0, kp_last = spos + min(j0 + 127, slen - 1);
        const int i_begin = max(0, ((kp_first + hoff) / p.bs) * p.bs - p.q_pos0);
        rt_begin = min(rt_end, (i_begin * p.g) >> 5);
        if (same) {
            const int i_end = max(0, min(Lq, (kp_last / p.bs + 1) * p.bs - p.q_pos0));
            rt_end = min(rt_end, (i_end * p.g + 31) >> 5);
        }
    }

    f32x16 acc[D / 32];   // dK^T or dV^T: lane = key, registers = 16 of the 32 head-dim entries of tile dt
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;

    // staging: thread -> NLD chunks of the 32-row tile; rows are (query, head) pairs gathered from Q / dO
    u32x4 qreg[NLD], greg[NLD];
    float st_lse2 = INFINITY, st_delta = 0.f;
    int st_qlim = 0;
    // Fast path for a full tile when the group size divides 32 (so a tile holds whole queries) and Q and dO share
    // their strides: row r of tile rt is query rt * (32 / g) + r / g, head r % g, i.e. a wave-uniform tile base plus
    // an offset that is fixed per thread: no division and no 64-bit per-thread arithmetic per tile.
    const bool rows_fast = (32 % p.g == 0) && p.q_st == p.do_st && p.q_sh == p.do_sh && p.q_st >= 0 && p.q_sh >= 0 &&
                           p.q_st < (1 << 25) && p.q_sh < (1 << 25);
    const int qpt = 32 / max(p.g, 1);                 // queries per tile (fast path)
    const int bs_shift = (BC && (p.bs & (p.bs - 1)) == 0) ? __builtin_ctz(p.bs) : -1;
    uint32_t roff[NLD];
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int cidx = tid + q * 256;
        const int row = cidx / C8, c = cidx - row * C8;
        roff[q] = (uint32_t)((row / p.g) * (int)p.q_st + (row % p.g) * (int)p.q_sh + c * 8);
    }
    const int st_r = tid & 31;
    const int st_i = st_r / p.g, st_h = kvh * p.g + st_r % p.g;     // this thread's statistics row inside a tile
    const int64_t st_base = stat_index(p, b, st_h, st_i, s0);       // ... of tile 0; tile rt is qpt entries further
#define BW_FETCH_ROWS(rt)                                                                                \
    {                                                                                                    \
        if (rows_fast && (rt) * 32 + 32 <= R) {                                                          \
            const int64_t tb_ = (int64_t)((rt) * qpt) * p.q_st + (int64_t)(kvh * p.g) * p.q_sh;          \
            const uint16_t* qb_ = p.q + q_off + tb_;                                                     \
            const uint16_t* gb_ = p.dout + do_off + tb_;                                                 \
            _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                            \
                qreg[q] = *reinterpret_cast<const u32x4*>(qb_ + roff[q]);                                \
                greg[q] = *reinterpret_cast<const u32x4*>(gb_ + roff[q]);                                \
            }                                                                                            \
            const int64_t si = st_base + (rt) * qpt;                                                     \
            const float l = p.lse[si];                                                                   \
            const float dl_ = DK ? p.delta[si] : 0.f;                                                    \
            st_lse2 = (l > -INFINITY) ? l * 1.4426950408889634f : INFINITY;                              \
            st_delta = dl_;                                                                              \
            const int qp_ = p.q_pos0 + (rt) * qpt + st_i;                                                \
            st_qlim = BC ? (bs_shift >= 0 ? (((qp_ >> bs_shift) + 1) << bs_shift) : (qp_ / p.bs + 1) * p.bs) : 0; \
        } else {                                                                                         \
        _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                                \
            const int cidx = tid + q * 256;                                                              \
            const int row = cidx / C8, c = cidx - row * C8;                                              \
            const int rr = min((rt) * 32 + row, R - 1);                                                  \
            const int ii = rr / p.g, hh = kvh * p.g + (rr - ii * p.g);                                   \
            qreg[q] = *reinterpret_cast<const u32x4*>(p.q + q_off + ii * p.q_st + (int64_t)hh * p.q_sh + c * 8);      \
            greg[q] = *reinterpret_cast<const u32x4*>(p.dout + do_off + ii * p.do_st + (int64_t)hh * p.do_sh + c * 8); \
        }                                                                                                \
        /* per-row statistics: every thread loads (row = tid mod 32, clamped) so that no load sits under a   */ \
        /* condition (the load counter stays exact and the prefetch really overlaps the tile's arithmetic)  */ \
        {                                                                                                \
            const int rr = (rt) * 32 + (tid & 31);                                                       \
            const int rc_ = min(rr, R - 1);                                                              \
            const int ii = rc_ / p.g, hh = kvh * p.g + (rc_ - ii * p.g);                                 \
            const int64_t si = stat_index(p, b, hh, ii, s0);                                             \
            const float l = p.lse[si];                                                                   \
            const float dl_ = DK ? p.delta[si] : 0.f;                                                    \
            const bool ok_ = rr < R;                                                                     \
            st_lse2 = (ok_ && l > -INFINITY) ? l * 1.4426950408889634f : INFINITY;                       \
            st_delta = ok_ ? dl_ : 0.f;                                                                  \
            /* an absent row: its probabilities are 0 through lse2; INT_MAX forces the masked path */    \
            st_qlim = ok_ ? (BC ? ((p.q_pos0 + ii) / p.bs + 1) * p.bs : 0) : 0x7fffffff;                 \
        }                                                                                                \
        }                                                                                                \
    }
#define BW_STORE_ROWS(rt)                                                                                \
    {                                                                                                    \
        const bool full_ = (rt) * 32 + 32 <= R;                                                          \
        _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                                \
            const int cidx = tid + q * 256;                                                              \
            const int row = cidx / C8, c = cidx - row * C8;                                              \
            const bool live = full_ || ((rt) * 32 + row < R);                                            \
            const u32x4 z = {0, 0, 0, 0};                                                                \
            const u32x4 qq = live ? qreg[q] : z, gg = live ? greg[q] : z;                                \
            *reinterpret_cast<u32x4*>(Qrow + row * KP + c * 16) = qq;                                    \
            if (DK) {                                                                                    \
                *reinterpret_cast<u32x4*>(Xtr + row * TP + c * 16) = qq;                                 \
                *reinterpret_cast<u32x4*>(Grow + row * KP + c * 16) = gg;                                \
            } else {                                                                                     \
                *reinterpret_cast<u32x4*>(Xtr + row * TP + c * 16) = gg;                                 \
            }                                                                                            \
        }                                                                                                \
        if (tid < 32) {                                                                                  \
            s_lse2[tid] = st_lse2;                                                                       \
            if (DK) s_delta[tid] = st_delta;                                                             \
            s_qlim[tid] = st_qlim;                                                                       \
        }                                                                                                \
    }

    // Row tiles are walked from the last one down: under a block-causal mask the workgroups of one (sequence,
    // KV head) differ in where their range BEGINS, so this way they all start on the same tile and stay in step.
    // The second slab of a pair is walked upwards: its range begins where the first slab's walk ended (slab x ends
    // after n - x steps, slab n - 1 - x begins at tile n - 1 - x), so at any time all the workgroups of the group
    // that are in their second pass are on one tile again, whatever their x.
    const bool up = pair && pass;
    if (rt_begin < rt_end) BW_FETCH_ROWS(up ? rt_begin : rt_end - 1);
    for (int it = 0; it < rt_end - rt_begin; ++it) {
        const int rt = up ? rt_begin + it : rt_end - 1 - it;
        BW_STORE_ROWS(rt);
        __syncthreads();
        BW_FETCH_ROWS(up ? min(rt + 1, rt_end - 1) : max(rt - 1, rt_begin));     // unconditional (clamped) prefetch of the next tile
        f32x16 S, dP;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            S[i] = 0.f;
            dP[i] = 0.f;
        }
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            const bf16x8 qa = *reinterpret_cast<const bf16x8*>(Qrow + n * KP + (16 * c + 8 * hi) * 2);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[c], S, 0, 0, 0);      // S[row, key]: lane = key
            if (DK) {
                const bf16x8 ga = *reinterpret_cast<const bf16x8*>(Grow + n * KP + (16 * c + 8 * hi) * 2);
                dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vf[c], dP, 0, 0, 0);
            }
        }
        // Masking is needed only where some (row, key) pair of this tile is hidden: rows' block ends are monotone,
        // so the first and the last row bound them (an absent last row carries INT_MAX: masked path for "own block").
        bool masked = !(j0 + w * 32 + 31 < slen);
        if (BC) {
            const int ql_first = s_qlim[0], ql_last = s_qlim[31];
            const int kp0 = spos + j0 + w * 32;
            masked = masked || !(kp0 + 31 + hoff < ql_first) || (same && !(ql_last <= kp0 + p.bs));
        }
        uint32_t pk[8];   // P (DV pass) or dS (DK pass) as bf16 pairs: the B operand of the second product
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            // registers 4 g4 .. 4 g4 + 3 hold rows 8 g4 + 4 hi + 0..3 of the tile
            const f32x4 l2 = *reinterpret_cast<const f32x4*>(s_lse2 + 8 * g4 + 4 * hi);
            float pe[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) pe[e] = fast_exp2(fmaf(S[4 * g4 + e], p.scale_log2, -l2[e]));
            if (masked) {
                i32x4 ql = {0, 0, 0, 0};
                if (BC) ql = *reinterpret_cast<const i32x4*>(s_qlim + 8 * g4 + 4 * hi);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bool vis = kvalid;
                    if (BC) vis = vis && (ql[e] > kpos + hoff) && (!same || ql[e] <= kpos + p.bs);
                    pe[e] = vis ? pe[e] : 0.f;
                }
            }
            if (DK) {
                const f32x4 dl = *reinterpret_cast<const f32x4*>(s_delta + 8 * g4 + 4 * hi);
#pragma unroll
                for (int e = 0; e < 4; ++e) pe[e] = pe[e] * (dP[4 * g4 + e] - dl[e]);
            }
            pk[2 * g4] = pack_bf16x2(pe[0], pe[1]);
            pk[2 * g4 + 1] = pack_bf16x2(pe[2], pe[3]);
        }
        bf16x8 bf[2];
        {
            u32x4 a = {pk[0], pk[1], pk[2], pk[3]}, c4 = {pk[4], pk[5], pk[6], pk[7]};
            bf[0] = bw_as_bf16x8(a);
            bf[1] = bw_as_bf16x8(c4);
        }
        const int s16 = lane & 15, blk = (lane >> 4) & 1;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) {
                union { s16x4 h[2]; bf16x8 v; } xt;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int rrow = 16 * j2 + 8 * q + 4 * hi + (s16 >> 2);
                    const int dcol = 32 * dt + 16 * blk + 4 * (s16 & 3);
                    xt.h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Xtr + rrow * TP + dcol * 2));
                }
                // DV: dV^T += dO^T P;  DK: dK^T += Q^T dS
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xt.v, bf[j2], acc[dt], 0, 0, 0);
            }
        }
        __syncthreads();
    }
#undef BW_FETCH_ROWS
#undef BW_STORE_ROWS

    if (kvalid) {
        uint16_t* op = (DK ? sdk : sdv) + kv_off + kvh * ssh + (int64_t)j * sst;
        const float f = DK ? p.scale : 1.0f;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 a;
                a[0] = pack_bf16x2(acc[dt][4 * q4] * f, acc[dt][4 * q4 + 1] * f);
                a[1] = pack_bf16x2(acc[dt][4 * q4 + 2] * f, acc[dt][4 * q4 + 3] * f);
                *reinterpret_cast<u32x2*>(op + 32 * dt + 8 * q4 + 4 * hi) = a;
            }
    }
    __syncthreads();   // the LDS images are reused by the next pass
    }
}

template <int D, bool BC>
static int launch_bwd(const BwdParams& p, hipStream_t st) {
    constexpr int RPB = 256 / (D / 8);
    const int rows = p.Lq * p.Hq;
    hipLaunchKernelGGL((attn_bwd_delta_kernel<D>), dim3((rows + RPB - 1) / RPB, 1, p.B), dim3(256), 0, st, p);
    int rc = check_hip(hipGetLastError(), "attn_bwd_delta_kernel launch");
    if (rc != DLM_OK) return rc;
    if (p.dq) {
        dim3 grid((p.R + 127) / 128, p.Hkv, p.B);
        GridRemap rm = no_remap();
        if ((g_attn_remap & 1) && grid.x >= 2) {
            const int64_t n_wg = set_remap(rm, (int64_t)p.B * p.Hkv, (int)grid.x, BC && (g_attn_remap & 2));
            if (n_wg > 0) grid = dim3((unsigned)n_wg);
            else rm = no_remap();
        }
        hipLaunchKernelGGL((attn_bwd_dq_kernel<D, BC>), grid, dim3(256), 0, st, p, rm);
        rc = check_hip(hipGetLastError(), "attn_bwd_dq_kernel launch");
        if (rc != DLM_OK) return rc;
    }
    for (int s = 0; s < 3; ++s) {
        if (!p.seg[s].dk || p.seg[s].len == 0) continue;
        const int n_slabs = (p.seg[s].len + 127) / 128;
        // equal-work pairing where the mask makes slabs unequal (not for "own block only": every slab sees one block's rows)
        const int pair = (BC && p.seg[s].rule != DLM_SEG_SAME_BLOCK && n_slabs >= 4) ? 1 : 0;
        dim3 grid(pair ? (n_slabs + 1) / 2 : n_slabs, p.Hkv, p.B);
        GridRemap rm = no_remap();
        if ((g_attn_remap & 4) && grid.x >= 2) {
            const int64_t n_wg = set_remap(rm, (int64_t)p.B * p.Hkv, (int)grid.x, false);
            if (n_wg > 0) grid = dim3((unsigned)n_wg);
            else rm = no_remap();
        }
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, BC, false>), grid, dim3(256), 0, st, p, s, n_slabs, pair, rm);
        rc = check_hip(hipGetLastError(), "attn_bwd_dkv_kernel (dV pass) launch");
        if (rc != DLM_OK) return rc;
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, BC, true>), grid, dim3(256), 0, st, p, s, n_slabs, pair, rm);
        rc = check_hip(hipGetLastError(), "attn_bwd_dkv_kernel (dK pass) launch");
        if (rc != DLM_OK) return rc;
    }
    return DLM_OK;
}

static int validate_bwd_seg(const dlm_kv_seg& s, const void* dk, const void* dv, const char* name, int d) {
    if (s.len < 0) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: %s.len < 0", name);
    if (s.rule < DLM_SEG_CAUSAL || s.rule > DLM_SEG_SAME_BLOCK) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: %s.rule %d unknown", name, s.rule);
    if ((dk == nullptr) != (dv == nullptr)) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: d%s k and v gradients go together", name);
    if (s.len == 0) return DLM_OK;
    if (!s.k || !s.v) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: %s has null k/v", name);
    if (!aligned16(s.k) || !aligned16(s.v) || !aligned16(dk) || !aligned16(dv))
        return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: %s pointers not 16-byte aligned", name);
    if ((s.stride_b | s.stride_h | s.stride_t) % 8) return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: %s strides must be multiples of 8", name);
    if (s.stride_t < d) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: %s.stride_t < d", name);
    if (s.pos0 < 0 || (int64_t)s.pos0 + s.len > (1 << 30)) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: %s positions outside [0, 2^30]", name);
    return DLM_OK;
}

static int validate_bwd(const dlm_attn_bwd_args* a) {
    if (!a) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: null args");
    if (a->struct_size != sizeof(dlm_attn_bwd_args))
        return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: struct_size %u != %zu", a->struct_size, sizeof(dlm_attn_bwd_args));
    if (a->B < 0 || a->Lq < 0 || a->Hq <= 0 || a->Hkv <= 0 || a->d <= 0)
        return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: bad sizes B=%d Lq=%d Hq=%d Hkv=%d d=%d", a->B, a->Lq, a->Hq, a->Hkv, a->d);
    if (a->Hq % a->Hkv) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: Hq=%d is not a multiple of Hkv=%d", a->Hq, a->Hkv);
    if (a->d != 64 && a->d != 128) return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: head_dim %d (supported: 64, 128)", a->d);
    if (a->mask_mode != DLM_MASK_FULL && a->mask_mode != DLM_MASK_BLOCK_CAUSAL)
        return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: unknown mask_mode %d", a->mask_mode);
    if (a->mask_mode == DLM_MASK_FULL && (a->prefix.rule | a->block.rule | a->suffix.rule))
        return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: segment rules need the block-causal mask mode");
    if (a->mask_mode == DLM_MASK_BLOCK_CAUSAL) {
        if (a->block_size < 1) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: block-causal needs block_size >= 1");
        if (a->q_pos0 < 0 || (int64_t)a->q_pos0 + a->Lq + a->block_size > (1 << 30))
            return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: query positions outside [0, 2^30]");
    }
    if (a->B > 65535 || a->Hkv > 65535) return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: B or Hkv above 65535");
    if ((int64_t)a->Lq * (a->Hq / a->Hkv) > (1 << 30)) return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: too many rows per KV head");
    if (a->cu_seqlens) {
        if (a->prefix.len || a->suffix.len) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: packed mode takes the block segment only");
        if (a->block.len != a->Lq) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: packed mode needs block.len == Lq");
        if (a->total_tokens < 0 || (int64_t)a->total_tokens > (int64_t)a->B * a->Lq)
            return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: total_tokens outside [0, B * Lq]");
        if (a->total_tokens == 0) return DLM_OK;
    }
    int rc;
    if ((rc = validate_bwd_seg(a->prefix, a->d_prefix_k, a->d_prefix_v, "prefix", a->d)) != DLM_OK) return rc;
    if ((rc = validate_bwd_seg(a->block, a->d_block_k, a->d_block_v, "block", a->d)) != DLM_OK) return rc;
    if ((rc = validate_bwd_seg(a->suffix, a->d_suffix_k, a->d_suffix_v, "suffix", a->d)) != DLM_OK) return rc;
    if ((int64_t)a->prefix.len + a->block.len + a->suffix.len > (1 << 30))
        return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: more than 2^30 keys");
    if (a->B == 0 || a->Lq == 0) return DLM_OK;
    if (!a->q || !a->out || !a->d_out || !a->lse) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: null q/out/d_out/lse");
    if (!aligned16(a->q) || !aligned16(a->out) || !aligned16(a->d_out) || !aligned16(a->d_q))
        return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: q/out/d_out/d_q not 16-byte aligned");
    if ((a->q_stride_b | a->q_stride_t | a->q_stride_h | a->o_stride_b | a->o_stride_t | a->o_stride_h |
         a->do_stride_b | a->do_stride_t | a->do_stride_h | a->dq_stride_b | a->dq_stride_t | a->dq_stride_h) % 8)
        return fail(DLM_ERR_UNSUPPORTED, "block_attn_bwd: strides must be multiples of 8");
    if (a->q_stride_h < a->d || a->o_stride_h < a->d || a->do_stride_h < a->d || (a->d_q && a->dq_stride_h < a->d))
        return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: head stride < d");
    if (!(a->scale == a->scale)) return fail(DLM_ERR_INVALID_ARG, "block_attn_bwd: scale is NaN");
    return DLM_OK;
}

}  // namespace dlm

using namespace dlm;

extern "C" size_t dlm_block_attn_bwd_workspace_bytes(const dlm_attn_bwd_args* a) {
    if (!a || a->B <= 0 || a->Lq <= 0 || a->Hq <= 0) return 0;
    const size_t rows = a->cu_seqlens ? (size_t)(a->total_tokens > 0 ? a->total_tokens : 0) : (size_t)a->B * a->Lq;
    return rows * (size_t)a->Hq * sizeof(float);
}

extern "C" int dlm_block_attn_bwd(const dlm_attn_bwd_args* a, void* stream) {
    int rc = validate_bwd(a);
    if (rc != DLM_OK) return rc;
    if (a->B == 0 || a->Lq == 0 || (a->cu_seqlens && a->total_tokens == 0)) return DLM_OK;
    const size_t need = dlm_block_attn_bwd_workspace_bytes(a);
    if (!a->workspace || a->workspace_bytes < need)
        return fail(DLM_ERR_WORKSPACE, "block_attn_bwd: workspace of %zu bytes needed, %zu given", need, a->workspace ? a->workspace_bytes : (size_t)0);
    if (!aligned16(a->workspace)) return fail(DLM_ERR_WORKSPACE, "block_attn_bwd: workspace not 16-byte aligned");
    BwdParams p;
    p.B = a->B; p.Lq = a->Lq; p.Hq = a->Hq; p.Hkv = a->Hkv; p.g = a->Hq / a->Hkv; p.R = p.g * a->Lq;
    p.q = (const uint16_t*)a->q; p.o = (const uint16_t*)a->out; p.dout = (const uint16_t*)a->d_out;
    p.q_sb = a->q_stride_b; p.q_st = a->q_stride_t; p.q_sh = a->q_stride_h;
    p.o_sb = a->o_stride_b; p.o_st = a->o_stride_t; p.o_sh = a->o_stride_h;
    p.do_sb = a->do_stride_b; p.do_st = a->do_stride_t; p.do_sh = a->do_stride_h;
    p.dq = (uint16_t*)a->d_q; p.dq_sb = a->dq_stride_b; p.dq_st = a->dq_stride_t; p.dq_sh = a->dq_stride_h;
    const dlm_kv_seg* segs[3] = {&a->prefix, &a->block, &a->suffix};
    void* dks[3] = {a->d_prefix_k, a->d_block_k, a->d_suffix_k};
    void* dvs[3] = {a->d_prefix_v, a->d_block_v, a->d_suffix_v};
    for (int s = 0; s < 3; ++s) {
        p.seg[s].k = (const uint16_t*)segs[s]->k; p.seg[s].v = (const uint16_t*)segs[s]->v;
        p.seg[s].dk = (uint16_t*)dks[s]; p.seg[s].dv = (uint16_t*)dvs[s];
        p.seg[s].len = segs[s]->len; p.seg[s].pos0 = segs[s]->pos0;
        p.seg[s].sb = segs[s]->stride_b; p.seg[s].sh = segs[s]->stride_h; p.seg[s].st = segs[s]->stride_t;
        p.seg[s].rule = segs[s]->rule;
    }
    p.lse = a->lse; p.delta = (float*)a->workspace;
    p.bs = a->block_size; p.q_pos0 = a->q_pos0;
    p.scale = a->scale > 0.f ? a->scale : 1.0f / sqrtf((float)a->d);
    p.scale_log2 = p.scale * 1.4426950408889634f;
    p.cu = a->cu_seqlens; p.total = a->total_tokens;
    hipStream_t st = (hipStream_t)stream;
    const bool bc = a->mask_mode == DLM_MASK_BLOCK_CAUSAL;
    if (a->d == 128) return bc ? launch_bwd<128, true>(p, st) : launch_bwd<128, false>(p, st);
    return bc ? launch_bwd<64, true>(p, st) : launch_bwd<64, false>(p, st);
}
