// dlm_block_attn: attention of a query block against [prefix | block | suffix] KV.
//
// Work decomposition (gfx950, 64-wide wavefronts, MFMA 32x32x16 bf16):
//   * The g = Hq/Hkv query heads that share a KV head are packed, together with the
//     Lq query rows, into R = g*Lq "rows" (row = i*g + head_in_group), so K/V of a
//     KV head are streamed once for all of them.
//   * A workgroup owns 32*NWR*RTW rows of one (sequence, KV head).  Its NWR*NWK
//     wavefronts either split the rows (NWK == 1: K/V tiles are shared through LDS)
//     or split the keys (NWR == 1: each wavefront streams every NWK-th 32-key tile
//     and the partial (max, sum, O) are merged through LDS at the end).
//   * Per 32-key tile: S^T = K Q^T with K as the MFMA A operand, so a lane ends up
//     holding 16 keys of ONE query column: the row max / row sum are in-register
//     reductions plus one exchange with lane^32.  P is rounded to bf16 in place and
//     is already in B-operand layout for O^T += V^T P^T; V^T fragments come from LDS
//     with the transposing 64-bit LDS read.
//   * fp32 scores, max, sum and accumulators; the row sum uses the unrounded p.
#include "common.hpp"
#include <string.h>

namespace dlm {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

struct SegDev {
    const uint16_t *k, *v;
    int len, pos0;
    int64_t sb, sh, st;
    int rule;   // block-causal visibility of this segment's keys: DLM_SEG_CAUSAL / _EARLIER_BLOCKS / _SAME_BLOCK
};

struct AttnParams {
    int B, Lq, Hq, Hkv, g, R;
    const uint16_t* q;
    int64_t q_sb, q_st, q_sh;
    SegDev seg[3];
    const int32_t* prefix_len_b;
    int bs, q_pos0;
    float scale_log2;  // scale * log2(e): softmax is evaluated with exp2
    uint16_t* out;
    int64_t o_sb, o_st, o_sh;
    float* lse;
    const int32_t* cu;  // packed variable-length mode: sequence b owns tokens [cu[b], cu[b+1])
    int total;          // cu[B]
    GridRemap remap;
    const int32_t* seq_active;   // optional [B]: 0 = skip the sequence
    // Key split across workgroups (nsplit > 1): workgroup `split` of a row tile walks the key tiles
    // [T * split / nsplit, T * (split + 1) / nsplit) and stores its unnormalised accumulators and its (running
    // maximum, sum) instead of the output; attn_merge_kernel combines the nsplit partials of every row.
    int nsplit;
    float* part_o;    // [nsplit][B * Hkv * R][d]
    float* part_ml;   // [nsplit][B * Hkv * R][2]  (maximum in log2 units, sum of exponentials relative to it)
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } x;
    x.u = v;
    return x.b;
}

// NTKV: K/V are fetched with non-temporal loads, for launches in which one workgroup is the only reader of its
// (sequence, KV head): the rollout step streams 70 - 1000 MB of cache that nothing reads twice.
// SWP: software-pipelined form of the 128-row shapes.  MFMA and vector-ALU instructions of DIFFERENT wavefronts of a
// SIMD do not run side by side on this chip (a wavefront of MFMAs beside a wavefront of exponentials takes the sum of
// their times: measured), those of ONE wavefront do; so each wavefront weaves the softmax of tile t between the score
// MFMAs of tile t + 1 and between the first P V MFMAs of tile t, instead of running the three phases one after another.
template <int D, int NWR, int NWK, int RTW, bool BC, int PF = 1, int OCC = 1, bool NTKV = false, bool SWP = false>
__global__ __launch_bounds__(64 * NWR * NWK, OCC) void attn_kernel(AttnParams p) {
    static_assert(!SWP || (RTW == 1 && NWK == 1 && NWR > 1 && D == 128 && PF == 1), "the pipelined form exists for 128-row workgroups, d = 128");
    static_assert(NWR == 1 || NWK <= 2, "row-split workgroups have at most two key groups");
    constexpr int NT = 64 * NWR * NWK;
    constexpr int FD = (SWP || OCC >= 3 || (NWR == 1 && OCC == 2)) ? 2 : 4;  // operand fragments in flight from LDS ahead of the MFMA that uses them (registers permitting)
    static_assert(D / 16 >= FD && 2 * (D / 32) >= FD, "fragment ring deeper than the step count");
    constexpr int KP = D * 2 + 16;          // K tile row pitch (bytes): 16-byte reads of 16 rows hit distinct banks
    constexpr int VP = D * 2 + 64;          // V tile row pitch: 4 rows x 64 B of a transposing read tile the 64 banks
    constexpr int TILE_BYTES = 32 * KP + 32 * VP;
    constexpr int C8 = D / 8;               // 16-byte chunks per row
    constexpr int NLD = (32 * C8) / (64 * NWR);
    constexpr int MP = D + 4;               // merge buffer row pitch (floats)
    // merge buffer: key-split wavefronts (NWR == 1) leave all NWK partials there; a row-split workgroup with two key
    // groups (NWR > 1, NWK == 2) passes the second group's partial through it
    constexpr int MERGE_BYTES = (NWK > 1) ? (NWR > 1 ? NWR : NWK) * 32 * MP * 4 : 0;
    constexpr bool DB = (NWR > 1) || (NWK == 1);   // row-split shapes double-buffer the K/V tile their NWR wavefronts share: one barrier per tile
    constexpr int NBUF = SWP ? 3 : (DB ? 2 : 1);   // the pipelined form reads K of tile t + 1 and V of tile t while tile t + 2 is stored
    constexpr int SMEM = (NBUF * NWK * TILE_BYTES > MERGE_BYTES) ? NBUF * NWK * TILE_BYTES : MERGE_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];

    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform by construction: kept in scalar registers so that the per-tile bookkeeping derived from the key
    // group index stays scalar too
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = w % NWR, wk = (NWK == 1) ? 0 : w / NWR;
    const int n = lane & 31, hi = lane >> 5;
    int b = blockIdx.z, kvh = blockIdx.y, bx = blockIdx.x;
    if (p.remap.nx > 0) {
        int grp;
        if (!remap_decode(p.remap, p.B * p.Hkv, grp, bx)) return;
        kvh = grp % p.Hkv;
        b = grp / p.Hkv;
    }
    if (p.seq_active && p.seq_active[b] == 0) return;   // nobody reads this sequence's output in this step
    int split = 0;
    if (p.nsplit > 1) {
        split = bx % p.nsplit;
        bx /= p.nsplit;
    }
    const int r0 = bx * (32 * NWR * RTW);

    // ---- visible extent of each segment for this workgroup -----------------
    int len0 = p.seg[0].len, len1 = p.seg[1].len, len2 = p.seg[2].len;
    if (p.prefix_len_b) len0 = min(len0, max(p.prefix_len_b[b], 0));
    // Packed mode: this sequence's tokens start at row s0 of q / out / the block segment and there are
    // sl of them; a workgroup whose rows all lie past the sequence's end has nothing to do.
    int R = p.R, s0 = 0;
    int64_t q_off = b * p.q_sb, o_off = b * p.o_sb, kv1_off = b * p.seg[1].sb;
    if (p.cu) {
        s0 = min(max(p.cu[b], 0), p.total);   // offsets are clamped to the buffer whatever the array holds
        const int sl = max(min(min(p.cu[b + 1], p.total) - s0, p.Lq), 0);
        R = p.g * sl;
        if (r0 >= R) return;
        len1 = min(len1, sl);
        q_off = s0 * p.q_st;
        o_off = s0 * p.o_st;
        kv1_off = s0 * p.seg[1].st;
    }
    // Block-causal visibility, per segment: a key at position pos is visible to a query whose block ends at
    // qlim (exclusive) iff  lo <= pos < hi  with  hi = qlim - hoff_s  (hoff_s = block size for "earlier blocks
    // only", else 0)  and  lo = qlim - block size for "own block only" (else no lower bound).
    int F0 = 0, F1 = 0, F2 = 0;                    // first 32-key tile of each segment that some row here can see
    int ho0 = 0, ho1 = 0, ho2 = 0;
    bool same0 = false, same1 = false, same2 = false;
    if (BC) {
        const int rows_end = min(r0 + 32 * NWR * RTW, R);
        const int lim = ((p.q_pos0 + (rows_end - 1) / p.g) / p.bs + 1) * p.bs;  // positions >= lim are invisible to every row here
        const int first = ((p.q_pos0 + r0 / p.g) / p.bs) * p.bs;               // start of the first row's block
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
    // Key tiles never straddle two segments: each segment is cut into its own 32-key tiles (its last one may
    // be ragged), so a tile's rows share one base pointer, stride and position origin (all wave-uniform).
    const int T0 = ((len0 + 31) >> 5) - F0, T1 = ((len1 + 31) >> 5) - F1, T2 = ((len2 + 31) >> 5) - F2;
    const int T = T0 + T1 + T2;
    // this workgroup's share of the key tiles: tiles t_lo .. t_lo + Tn - 1 (all of them without a key split)
    int t_lo = 0, Tn = T;
    if (p.nsplit > 1) {
        t_lo = (int)((int64_t)T * split / p.nsplit);
        Tn = (int)((int64_t)T * (split + 1) / p.nsplit) - t_lo;
    }
    const int n_it = (Tn + NWK - 1) / NWK;

    const uint16_t* kb0 = p.seg[0].k + b * p.seg[0].sb + kvh * p.seg[0].sh;
    const uint16_t* vb0 = p.seg[0].v + b * p.seg[0].sb + kvh * p.seg[0].sh;
    const uint16_t* kb1 = p.seg[1].k + kv1_off + kvh * p.seg[1].sh;
    const uint16_t* vb1 = p.seg[1].v + kv1_off + kvh * p.seg[1].sh;
    const uint16_t* kb2 = p.seg[2].k + b * p.seg[2].sb + kvh * p.seg[2].sh;
    const uint16_t* vb2 = p.seg[2].v + b * p.seg[2].sb + kvh * p.seg[2].sh;
    const int64_t st0 = p.seg[0].st, st1 = p.seg[1].st, st2 = p.seg[2].st;
    // plain locals, so that selecting among them stays a register select (never an indexed reload of `p`)
    const int sp0 = __builtin_amdgcn_readfirstlane(p.seg[0].pos0), sp1 = __builtin_amdgcn_readfirstlane(p.seg[1].pos0),
              sp2 = __builtin_amdgcn_readfirstlane(p.seg[2].pos0);

    // ---- Q fragments (B operand: lane = query column, 8 consecutive d) ------
    bf16x8 qf[RTW][D / 16];
    int qlim[RTW];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
        const int r = r0 + (wr * RTW + rt) * 32 + n;
        const bool valid = r < R;
        const int i = valid ? r / p.g : 0;
        const int hg = valid ? r - i * p.g : 0;
        const uint16_t* qp = p.q + q_off + i * p.q_st + (int64_t)(kvh * p.g + hg) * p.q_sh;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            u32x4 v = {0, 0, 0, 0};
            if (valid) v = *reinterpret_cast<const u32x4*>(qp + 16 * c + 8 * hi);
            qf[rt][c] = as_bf16x8(v);
        }
        qlim[rt] = BC ? ((p.q_pos0 + i) / p.bs + 1) * p.bs : 0;
    }
    int qlim_min = 0x7fffffff;   // smallest and largest block end over the rows of this wavefront
    int qlim_max = 0;
    if (BC) {
#pragma unroll
        for (int rt = 0; rt < RTW; ++rt) {
            qlim_min = min(qlim_min, qlim[rt]);
            qlim_max = max(qlim_max, qlim[rt]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            qlim_min = min(qlim_min, shfl_xor(qlim_min, off));
            qlim_max = max(qlim_max, shfl_xor(qlim_max, off));
        }
        qlim_min = __builtin_amdgcn_readfirstlane(qlim_min);   // wave-uniform now: keep them in scalar registers
        qlim_max = __builtin_amdgcn_readfirstlane(qlim_max);
    }

    f32x16 O[RTW][D / 32];
    float m_run[RTW], l_run[RTW];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
        m_run[rt] = -INFINITY;
        l_run[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[rt][dt][i] = 0.f;
    }

    unsigned char* Kl = smem + wk * NBUF * TILE_BYTES;   // re-pointed per tile when double-buffering
    unsigned char* Vl = Kl + 32 * KP;
    const int tl = wr * 64 + lane;  // thread index inside the wave group that shares a tile

    // PF tiles of K/V are in flight in registers per wave group; addresses are clamped so that the loads
    // are unconditional (the load-counter waits stay exact) and rows past the end are zeroed when staged.
    u32x4 kreg[PF][NLD], vreg[PF][NLD];
    // Full tiles are addressed as (wave-uniform tile base) + (this thread's element offset inside a tile): no
    // 64-bit per-thread arithmetic per tile.  Needs every segment that is present to have the same row stride
    // (views of one cache tensor, the usual case) and 32 rows of it to fit 32 bits.
    const int64_t st_c = p.seg[0].len ? st0 : (p.seg[1].len ? st1 : st2);
    const bool fast_addr = st_c >= 0 && st_c < (1 << 25) && (!p.seg[0].len || st0 == st_c) &&
                           (!p.seg[1].len || st1 == st_c) && (!p.seg[2].len || st2 == st_c);
    uint32_t toff[NLD];
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int cidx = tl + q * (64 * NWR);
        const int row = cidx / C8, c = cidx - row * C8;
        toff[q] = (uint32_t)(row * (int)st_c + c * 8);
    }
    // segment of this workgroup's tile t (t < Tn), its index inside the segment, and the segment's extent
#define ATTN_TILE(t, sg, lt, slen)                                                                       \
    const int gt_##sg = (t) + t_lo;                                                                      \
    const int sg = (gt_##sg < T0) ? 0 : ((gt_##sg < T0 + T1) ? 1 : 2);                                   \
    const int lt = (gt_##sg < T0) ? gt_##sg + F0 : ((gt_##sg < T0 + T1) ? gt_##sg - T0 + F1 : gt_##sg - T0 - T1 + F2); \
    const int slen = (sg == 0) ? len0 : ((sg == 1) ? len1 : len2);
#define ATTN_LD(ptr) (NTKV ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ptr)) : *reinterpret_cast<const u32x4*>(ptr))
#define ATTN_PREFETCH(slot, t)                                                                           \
    {                                                                                                    \
        const int tc_ = min((t), Tn - 1);                                                                 \
        ATTN_TILE(tc_, sg_, lt_, slen_)                                                                  \
        const uint16_t* kb = (sg_ == 0) ? kb0 : ((sg_ == 1) ? kb1 : kb2);                                \
        const uint16_t* vb = (sg_ == 0) ? vb0 : ((sg_ == 1) ? vb1 : vb2);                                \
        const int64_t stt = (sg_ == 0) ? st0 : ((sg_ == 1) ? st1 : st2);                                 \
        if (fast_addr && lt_ * 32 + 32 <= slen_) {                                                       \
            /* a full tile: wave-uniform tile base + this thread's fixed 32-bit offset */                \
            const uint16_t* kt = kb + (int64_t)(lt_ * 32) * stt;                                         \
            const uint16_t* vt = vb + (int64_t)(lt_ * 32) * stt;                                         \
            _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                            \
                kreg[slot][q] = ATTN_LD(kt + toff[q]);                                                   \
                vreg[slot][q] = ATTN_LD(vt + toff[q]);                                                   \
            }                                                                                            \
        } else {                                                                                         \
            _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                            \
                const int cidx = tl + q * (64 * NWR);                                                    \
                const int row = cidx / C8, c = cidx - row * C8;                                          \
                const int loc = min(lt_ * 32 + row, slen_ - 1);                                          \
                const int64_t off = loc * stt + c * 8;                                                   \
                kreg[slot][q] = ATTN_LD(kb + off);                                                       \
                vreg[slot][q] = ATTN_LD(vb + off);                                                       \
            }                                                                                            \
        }                                                                                                \
    }
// Key-split wave groups are single wavefronts with private LDS tiles: LDS operations of one wavefront are
    // processed in order, so only the compiler has to be kept from reordering them; no workgroup barrier.
#define ATTN_TILE_SYNC()                                                                                 \
    {                                                                                                    \
        if (NWR == 1) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                 \
        else __syncthreads();                                                                            \
    }
#define ATTN_STAGE(slot, t)                                                                              \
    {                                                                                                    \
        ATTN_TILE(min((t), Tn - 1), sg_, lt_, slen_)                                                      \
        (void)sg_;                                                                                       \
        ATTN_TILE_SYNC(); /* the previous tile has been read */                                          \
        _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                                \
            const int cidx = tl + q * (64 * NWR);                                                        \
            const int row = cidx / C8, c = cidx - row * C8;                                              \
            const bool live = ((t) < Tn) && (lt_ * 32 + row < slen_);                                     \
            const u32x4 z = {0, 0, 0, 0};                                                                \
            *reinterpret_cast<u32x4*>(Kl + row * KP + c * 16) = live ? kreg[slot][q] : z;                \
            *reinterpret_cast<u32x4*>(Vl + row * VP + c * 16) = live ? vreg[slot][q] : z;                \
        }                                                                                                \
        ATTN_TILE_SYNC();                                                                                \
    }

#define ATTN_STORE(slot, t, buf)                                                                         \
    {                                                                                                    \
        ATTN_TILE(min((t), Tn - 1), sg_, lt_, slen_)                                                      \
        (void)sg_;                                                                                       \
        unsigned char* Kd = smem + (wk * NBUF + (buf)) * TILE_BYTES;                                     \
        unsigned char* Vd = Kd + 32 * KP;                                                                \
        if ((t) < Tn && lt_ * 32 + 32 <= slen_) {   /* a full tile: every row is live */                  \
            _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                            \
                const int cidx = tl + q * (64 * NWR);                                                    \
                const int row = cidx / C8, c = cidx - row * C8;                                          \
                *reinterpret_cast<u32x4*>(Kd + row * KP + c * 16) = kreg[slot][q];                       \
                *reinterpret_cast<u32x4*>(Vd + row * VP + c * 16) = vreg[slot][q];                       \
            }                                                                                            \
        } else {                                                                                         \
            _Pragma("unroll") for (int q = 0; q < NLD; ++q) {                                            \
                const int cidx = tl + q * (64 * NWR);                                                    \
                const int row = cidx / C8, c = cidx - row * C8;                                          \
                const bool live = ((t) < Tn) && (lt_ * 32 + row < slen_);                                 \
                const u32x4 z = {0, 0, 0, 0};                                                            \
                *reinterpret_cast<u32x4*>(Kd + row * KP + c * 16) = live ? kreg[slot][q] : z;            \
                *reinterpret_cast<u32x4*>(Vd + row * VP + c * 16) = live ? vreg[slot][q] : z;            \
            }                                                                                            \
        }                                                                                                \
    }

    // One K/V tile: scores, (lazy) online softmax, P V.  A macro rather than a lambda: every array it
    // touches must stay in registers.
#define ATTN_COMPUTE() /* uses the tile index `t` of the enclosing scope */                              \
    if (t < Tn) {                                                                                        \
        f32x16 S[RTW]; \
_Pragma("unroll") \
        for (int rt = 0; rt < RTW; ++rt) \
_Pragma("unroll") \
            for (int i = 0; i < 16; ++i) S[rt][i] = 0.f; \
        /* K fragments are requested FD MFMA steps ahead of their use, so that the LDS round trip of one fragment \
           is covered by the MFMAs of the steps before it instead of sitting between two dependent MFMAs */ \
        { \
            bf16x8 kfr[FD]; \
_Pragma("unroll") \
            for (int c = 0; c < FD; ++c) kfr[c] = *reinterpret_cast<const bf16x8*>(Kl + n * KP + (16 * c + 8 * hi) * 2); \
_Pragma("unroll") \
            for (int c = 0; c < D / 16; ++c) { \
_Pragma("unroll") \
                for (int rt = 0; rt < RTW; ++rt) S[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[c % FD], qf[rt][c], S[rt], 0, 0, 0); \
                if (c + FD < D / 16) kfr[c % FD] = *reinterpret_cast<const bf16x8*>(Kl + n * KP + (16 * (c + FD) + 8 * hi) * 2); \
                __builtin_amdgcn_sched_barrier(0); \
            } \
        } \
        ATTN_TILE(t, sg, lt, slen) \
        const int spos0 = ((sg == 0) ? sp0 : ((sg == 1) ? sp1 : sp2)) + lt * 32; \
        const int hoff = (sg == 0) ? ho0 : ((sg == 1) ? ho1 : ho2); \
        const bool same = (sg == 0) ? same0 : ((sg == 1) ? same1 : same2); \
        const bool ragged = (lt * 32 + 32 > slen) || \
                            (BC && (spos0 + 31 >= qlim_min - hoff || (same && spos0 < qlim_max - p.bs))); \
        bf16x8 pf[RTW][2]; \
_Pragma("unroll") \
        for (int rt = 0; rt < RTW; ++rt) { \
            float mx = -INFINITY; \
            if (ragged) { \
                /* element i sits at position pbase + 8 * (i / 4) + i % 4; visible iff lo_r <= position < hi_r */ \
                const int pbase = spos0 + 4 * hi; \
                int hi_r = spos0 - lt * 32 + slen;   /* end of the segment */ \
                int lo_r = -(1 << 30); \
                if (BC) { \
                    hi_r = min(hi_r, qlim[rt] - hoff); \
                    if (same) lo_r = qlim[rt] - p.bs; \
                } \
                const unsigned span = (unsigned)max(hi_r - lo_r, 0); \
                const unsigned off0 = (unsigned)(pbase - lo_r); \
_Pragma("unroll") \
                for (int i = 0; i < 16; ++i) \
                    if (off0 + (unsigned)(8 * (i >> 2) + (i & 3)) >= span) S[rt][i] = -INFINITY; \
            } \
_Pragma("unroll") \
            for (int i = 0; i < 16; i += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, S[rt][i]), S[rt][i + 1]); /* v_max3 */ \
            { /* other half of the wavefront: one lane-half swap instead of a permute through LDS */ \
                const auto sw_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false); \
                mx = __builtin_fmaxf(__uint_as_float(sw_[0]), __uint_as_float(sw_[1])) * p.scale_log2; \
            } \
            constexpr float LAZY = 8.0f; \
            const bool grow = mx > m_run[rt] + LAZY; \
            const float m_new = grow ? mx : m_run[rt]; \
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new; \
            const float alpha = grow ? fast_exp2(m_run[rt] - m_use) : 1.0f; \
            float rs = 0.f; \
            uint32_t pk[8]; \
_Pragma("unroll") \
            for (int i = 0; i < 16; i += 2) { \
                const float p0 = fast_exp2(fmaf(S[rt][i], p.scale_log2, -m_use)); \
                const float p1 = fast_exp2(fmaf(S[rt][i + 1], p.scale_log2, -m_use)); \
                rs += p0 + p1; \
                pk[i >> 1] = pack_bf16x2(p0, p1); \
            } \
            l_run[rt] = l_run[rt] * alpha + rs; \
            if (__any(grow && m_run[rt] != -INFINITY)) { \
_Pragma("unroll") \
                for (int dt = 0; dt < D / 32; ++dt) \
_Pragma("unroll") \
                    for (int i = 0; i < 16; ++i) O[rt][dt][i] *= alpha; \
            } \
            m_run[rt] = m_new; \
            u32x4 lo = {pk[0], pk[1], pk[2], pk[3]}, hi4 = {pk[4], pk[5], pk[6], pk[7]}; \
            pf[rt][0] = as_bf16x8(lo); \
            pf[rt][1] = as_bf16x8(hi4); \
        } \
        const int s16 = lane & 15, blk = (lane >> 4) & 1; \
        /* step e = 2 * dt + j2 of the second product; its V^T fragment (two transposing reads) is requested FD steps ahead */ \
        { \
            union VFrag { s16x4 h[2]; bf16x8 v; }; \
            VFrag vfr[FD]; \
            const unsigned char* vbase = Vl + (4 * hi + (s16 >> 2)) * VP + (16 * blk + 4 * (s16 & 3)) * 2; \
_Pragma("unroll") \
            for (int e = 0; e < FD; ++e) \
_Pragma("unroll") \
                for (int q = 0; q < 2; ++q) \
                    vfr[e].h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbase + (16 * (e & 1) + 8 * q) * VP + 32 * (e >> 1) * 2)); \
_Pragma("unroll") \
            for (int e = 0; e < 2 * (D / 32); ++e) { \
_Pragma("unroll") \
                for (int rt = 0; rt < RTW; ++rt) \
                    O[rt][e >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[e % FD].v, pf[rt][e & 1], O[rt][e >> 1], 0, 0, 0); \
                if (e + FD < 2 * (D / 32)) { \
_Pragma("unroll") \
                    for (int q = 0; q < 2; ++q) \
                        vfr[e % FD].h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbase + (16 * ((e + FD) & 1) + 8 * q) * VP + 32 * ((e + FD) >> 1) * 2)); \
                } \
                __builtin_amdgcn_sched_barrier(0); \
            } \
        } \
    }

    // tile of iteration `it` for this wave group: it * NWK + wk; it sits in register slot it % PF
    if (n_it > 0) {
        const int rot0 = DB ? 0 : (int)(((unsigned)b * (unsigned)p.Hkv + (unsigned)kvh) * 5u % (unsigned)n_it);
#pragma unroll
        for (int s = 0; s < PF; ++s)
            if (s < n_it) ATTN_PREFETCH(s, ((s + rot0 >= n_it) ? s + rot0 - n_it : s + rot0) * NWK + wk);
    }
    if constexpr (SWP) {
        // Tile i lives in LDS buffer i % 3.  Iteration t first stores tile t + 2 (requested an iteration ago) into the third
        // buffer and requests tile t + 3; it holds the raw scores of tile t in registers (SC), computes those of tile t + 1
        // (SN) from buffer (t + 1) % 3 while turning SC into probabilities, and multiplies them with V of tile t from
        // buffer t % 3.  One barrier per iteration.
#define ATTN_SWP_MASK(SC, tt)                                                                            \
    {                                                                                                    \
        ATTN_TILE(tt, sg, lt, slen)                                                                      \
        const int spos0 = ((sg == 0) ? sp0 : ((sg == 1) ? sp1 : sp2)) + lt * 32;                         \
        const int hoff = (sg == 0) ? ho0 : ((sg == 1) ? ho1 : ho2);                                      \
        const bool same = (sg == 0) ? same0 : ((sg == 1) ? same1 : same2);                               \
        const bool ragged = (lt * 32 + 32 > slen) ||                                                     \
                            (BC && (spos0 + 31 >= qlim_min - hoff || (same && spos0 < qlim_max - p.bs))); \
        if (ragged) {                                                                                    \
            const int pbase = spos0 + 4 * hi;                                                            \
            int hi_r = spos0 - lt * 32 + slen;                                                           \
            int lo_r = -(1 << 30);                                                                       \
            if (BC) {                                                                                    \
                hi_r = min(hi_r, qlim[0] - hoff);                                                        \
                if (same) lo_r = qlim[0] - p.bs;                                                         \
            }                                                                                            \
            const unsigned span = (unsigned)max(hi_r - lo_r, 0);                                         \
            const unsigned off0 = (unsigned)(pbase - lo_r);                                              \
            _Pragma("unroll") for (int i = 0; i < 16; ++i)                                               \
                if (off0 + (unsigned)(8 * (i >> 2) + (i & 3)) >= span) SC[i] = -INFINITY;                \
        }                                                                                                \
    }
#define ATTN_SWP_PAIR(SC, j)                                                                             \
    {                                                                                                    \
        const float p0_ = fast_exp2(fmaf(SC[2 * (j)], p.scale_log2, -m_use));                            \
        const float p1_ = fast_exp2(fmaf(SC[2 * (j) + 1], p.scale_log2, -m_use));                        \
        rs += p0_ + p1_;                                                                                 \
        pk[j] = pack_bf16x2(p0_, p1_);                                                                   \
    }
#define ATTN_SWP_ITER(SC, SN, tt)                                                                        \
    {                                                                                                    \
        const int t = (tt);                                                                              \
        /* tile t + 2, requested an iteration ago, goes into the buffer that tile t - 1 has left; tile t + 3 is requested \
           right away, so that it has this whole iteration to arrive */                                  \
        ATTN_STORE(0, t + 2, (t + 2) % 3);                                                               \
        ATTN_PREFETCH(0, t + 3);                                                                         \
        ATTN_SWP_MASK(SC, t)                                                                             \
        const unsigned char* Kn = smem + ((t + 1) % 3) * TILE_BYTES + n * KP + 16 * hi;                  \
        const unsigned char* Vc = smem + (t % 3) * TILE_BYTES + 32 * KP + (4 * hi + ((lane & 15) >> 2)) * VP + \
                                  (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;                         \
        float mx = -INFINITY, m_new = 0.f, m_use = 0.f, alpha = 1.f, rs = 0.f;                           \
        bool grow = false;                                                                               \
        uint32_t pk[8];                                                                                  \
        /* ---- scores of tile t + 1 between the softmax pieces of tile t ---- */                        \
        /* The (rare) rescaling of the accumulators is a branch; it sits right behind the two steps that decide it, so  \
           that everything after it, the exponentials and both MFMA chains, is one straight block the scheduler keeps   \
           in the written order (code before a branch whose results are only used after it would be sunk past it). */   \
        bf16x8 kfr[FD];                                                                                  \
        _Pragma("unroll") for (int c = 0; c < FD; ++c) kfr[c] = *reinterpret_cast<const bf16x8*>(Kn + 32 * c); \
        _Pragma("unroll") for (int c = 0; c < 2; ++c) {                                                  \
            if (c == 0) { const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
                          SN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[0], qf[0][0], z_, 0, 0, 0); } \
            else SN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[c % FD], qf[0][c], SN, 0, 0, 0);       \
            kfr[c % FD] = *reinterpret_cast<const bf16x8*>(Kn + 32 * (c + FD));                          \
            if (c == 0) {                                                                                \
                _Pragma("unroll") for (int i = 0; i < 16; i += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, SC[i]), SC[i + 1]); \
            } else {                                                                                     \
                const auto sw_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false); \
                mx = __builtin_fmaxf(__uint_as_float(sw_[0]), __uint_as_float(sw_[1])) * p.scale_log2;   \
                grow = mx > m_run[0] + 8.0f;                                                             \
                m_new = grow ? mx : m_run[0];                                                            \
                m_use = (m_new == -INFINITY) ? 0.f : m_new;                                              \
                alpha = grow ? fast_exp2(m_run[0] - m_use) : 1.0f;                                       \
            }                                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                                           \
        }                                                                                                \
        if (__any(grow && m_run[0] != -INFINITY)) {                                                      \
            _Pragma("unroll") for (int dt = 0; dt < 4; ++dt)                                             \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) O[0][dt][i] *= alpha;                     \
        }                                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                               \
        _Pragma("unroll") for (int c = 2; c < 8; ++c) {                                                  \
            SN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[c % FD], qf[0][c], SN, 0, 0, 0);            \
            if (c + FD < 8) kfr[c % FD] = *reinterpret_cast<const bf16x8*>(Kn + 32 * (c + FD));          \
            ATTN_SWP_PAIR(SC, c - 2)                                                                     \
            __builtin_amdgcn_sched_barrier(0);                                                           \
        }                                                                                                \
        /* ---- P V of tile t: the keys 0..15 half first, while the last probabilities of the other half are formed ---- */ \
        {                                                                                                \
            union VFrag { s16x4 h[2]; bf16x8 v; };                                                       \
            VFrag vfr[FD];                                                                               \
            _Pragma("unroll") for (int e = 0; e < FD; ++e)                                               \
                _Pragma("unroll") for (int q = 0; q < 2; ++q)                                            \
                    vfr[e].h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Vc + (16 * (e >> 2) + 8 * q) * VP + 32 * (e & 3) * 2)); \
            bf16x8 pf0, pf1;                                                                             \
            { const u32x4 lo_ = {pk[0], pk[1], pk[2], pk[3]}; pf0 = as_bf16x8(lo_); }                    \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                              \
                if (e == 4) { const u32x4 hi_ = {pk[4], pk[5], pk[6], pk[7]}; pf1 = as_bf16x8(hi_); }    \
                O[0][e & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[e % FD].v, (e < 4) ? pf0 : pf1, O[0][e & 3], 0, 0, 0); \
                if (e + FD < 8) {                                                                        \
                    _Pragma("unroll") for (int q = 0; q < 2; ++q)                                        \
                        vfr[e % FD].h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Vc + (16 * ((e + FD) >> 2) + 8 * q) * VP + 32 * ((e + FD) & 3) * 2)); \
                }                                                                                        \
                if (e == 0) { ATTN_SWP_PAIR(SC, 6) }                                                     \
                else if (e == 1) { ATTN_SWP_PAIR(SC, 7) }                                                \
                else if (e == 2) { l_run[0] = l_run[0] * alpha + rs; m_run[0] = m_new; }                 \
                __builtin_amdgcn_sched_barrier(0);                                                       \
            }                                                                                            \
        }                                                                                                \
        __syncthreads();                                                                                 \
    }
        f32x16 SA, SB;
        if (n_it > 0) {
            // Everything requested so far (Q, tile 0) is needed now; an explicit full wait leaves the compiler's
            // load-counter bookkeeping with nothing pending from before the loop, so that its waits inside the loop
            // count only the loop's own requests.
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            ATTN_STORE(0, 0, 0);
            ATTN_PREFETCH(0, 1);
            __syncthreads();
            {   // scores of tile 0, not overlapped with anything
                const unsigned char* K0 = smem + n * KP + 16 * hi;
                const f32x16 z_ = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                SA = z_;
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    SA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(K0 + 32 * c), qf[0][c], SA, 0, 0, 0);
            }
            ATTN_STORE(0, 1, 1);
            ATTN_PREFETCH(0, 2);
            __syncthreads();
        }
        int it = 0;
        for (; it + 1 < n_it; it += 2) {
            ATTN_SWP_ITER(SA, SB, it);
            ATTN_SWP_ITER(SB, SA, it + 1);
        }
        if (it < n_it) ATTN_SWP_ITER(SA, SB, it);
#undef ATTN_SWP_ITER
#undef ATTN_SWP_PAIR
#undef ATTN_SWP_MASK
    } else
    if (DB) {
        // iteration `i` multiplies this key group's tile i * NWK + wk from LDS buffer i & 1 while the tile of iteration
        // i + 1 is stored into the other buffer and the one of iteration i + 1 + PF is requested into the register slot
        // that store frees
#define ATTN_DB_TILE(i) ((i) * NWK + wk)
        if (n_it > 0) {
            ATTN_STORE(0, ATTN_DB_TILE(0), 0);
            if (PF < n_it) ATTN_PREFETCH(0, ATTN_DB_TILE(PF));
        }
        __syncthreads();
        int it = 0;
        const int n_steady = (n_it - PF - 1 > 0) ? ((n_it - PF - 1) / PF) * PF : 0;
        for (; it < n_steady; it += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int i = it + u;
                const int t = ATTN_DB_TILE(i);
                ATTN_STORE((u + 1) % PF, ATTN_DB_TILE(i + 1), (i + 1) & 1);
                ATTN_PREFETCH((u + 1) % PF, ATTN_DB_TILE(i + 1 + PF));
                Kl = smem + (wk * NBUF + (i & 1)) * TILE_BYTES;
                Vl = Kl + 32 * KP;
                ATTN_COMPUTE();
                __syncthreads();
            }
        }
#pragma unroll
        for (int u = 0; u < 2 * PF + 1; ++u) {
            const int i = it + u;
            if (i < n_it) {
                const int t = ATTN_DB_TILE(i);
                if (i + 1 < n_it) {
                    ATTN_STORE((u + 1) % PF, ATTN_DB_TILE(i + 1), (i + 1) & 1);
                    if (i + 1 + PF < n_it) ATTN_PREFETCH((u + 1) % PF, ATTN_DB_TILE(i + 1 + PF));
                }
                Kl = smem + (wk * NBUF + (i & 1)) * TILE_BYTES;
                Vl = Kl + 32 * KP;
                ATTN_COMPUTE();
                __syncthreads();
            }
        }
#undef ATTN_DB_TILE
    } else {
        // Each (sequence, KV head) starts its walk over the key tiles at a different tile and wraps: the K/V
        // blocks of different heads are a large power-of-two-ish stride apart, so workgroups that all begin at
        // tile 0 hit the same few HBM channels together.  Softmax is order-independent up to rounding.
        const int rot = (n_it > 0) ? (int)(((unsigned)b * (unsigned)p.Hkv + (unsigned)kvh) * 5u % (unsigned)n_it) : 0;
#define ATTN_KS_TILE(i) ((((i) + rot) >= n_it ? (i) + rot - n_it : (i) + rot) * NWK + wk)
        int it = 0;
        const int n_steady = (n_it - PF > 0) ? ((n_it - PF) / PF) * PF : 0;
        for (; it < n_steady; it += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int t = ATTN_KS_TILE(it + u);
                ATTN_STAGE(u, t);
                ATTN_PREFETCH(u, ATTN_KS_TILE(it + u + PF));
                ATTN_COMPUTE();
            }
        }
#pragma unroll
        for (int u = 0; u < 2 * PF; ++u) {
            const int i = it + u;
            if (i < n_it) {
                const int t = ATTN_KS_TILE(i);
                ATTN_STAGE(u % PF, t);
                if (i + PF < n_it) ATTN_PREFETCH(u % PF, ATTN_KS_TILE(i + PF));
                ATTN_COMPUTE();
            }
        }
#undef ATTN_KS_TILE
    }
#undef ATTN_STORE
#undef ATTN_TILE_SYNC
#undef ATTN_COMPUTE
#undef ATTN_PREFETCH
#undef ATTN_LD
#undef ATTN_TILE
#undef ATTN_STAGE

    // ---- finish -----------------------------------------------------------------
    constexpr float LN2 = 0.6931471805599453f;
    if (NWR > 1 && NWK > 1) {
        // Two key groups of NWR wavefronts each: group 1 hands its accumulators, running maximum and (per half-wave)
        // sum to group 0 through LDS (the tiles are dead: the loop ended with a barrier); group 0 folds them into its own
        // registers, lane for lane, and finishes alone.
        float* mb = reinterpret_cast<float*>(smem);
#pragma unroll
        for (int rt = 0; rt < RTW; ++rt) {
            float* row = mb + (wr * 32 + n) * MP;
            if (rt > 0) __syncthreads();
            if (wk == 1) {
#pragma unroll
                for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x4 v = {O[rt][dt][4 * q4], O[rt][dt][4 * q4 + 1], O[rt][dt][4 * q4 + 2], O[rt][dt][4 * q4 + 3]};
                        *reinterpret_cast<f32x4*>(row + 32 * dt + 8 * q4 + 4 * hi) = v;
                    }
                if (hi == 0) row[D] = m_run[rt];
                row[D + 1 + hi] = l_run[rt];
            }
            __syncthreads();
            if (wk == 0) {
                const float m1 = row[D], l1 = row[D + 1 + hi];
                const float M = fmaxf(m_run[rt], m1);
                const float a0 = (m_run[rt] == -INFINITY) ? 0.f : fast_exp2(m_run[rt] - M);
                const float a1 = (m1 == -INFINITY) ? 0.f : fast_exp2(m1 - M);
#pragma unroll
                for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const f32x4 v = *reinterpret_cast<const f32x4*>(row + 32 * dt + 8 * q4 + 4 * hi);
#pragma unroll
                        for (int e = 0; e < 4; ++e) O[rt][dt][4 * q4 + e] = a0 * O[rt][dt][4 * q4 + e] + a1 * v[e];
                    }
                l_run[rt] = a0 * l_run[rt] + a1 * l1;
                m_run[rt] = M;
            }
        }
        __syncthreads();     // group 0 re-uses the buffer for its output staging
        if (wk != 0) return;
    }
    if (NWR > 1 || NWK == 1) {
        // The accumulators hold O^T (lane = row, registers = head-dim entries): stored straight from registers a
        // wavefront's store touches 32 rows with 16 bytes each, 64 such stores per row tile.  Each wavefront instead
        // transposes its 32 rows through a private LDS region (the K/V tiles are dead: the loop ended with a
        // barrier) and writes whole rows, 16 bytes per lane: 4 (d = 64) or 8 stores that cover full cache lines.
        constexpr int OPB = D * 2 + 16;                    // staging row pitch in bytes (16-byte aligned)
        static_assert(NWR * 32 * OPB + NWR * 32 * 8 <= 2 * TILE_BYTES, "output staging must fit in the tile buffers");
        unsigned char* ob = smem + wr * (32 * OPB);
        int64_t* roff = reinterpret_cast<int64_t*>(smem + NWR * 32 * OPB) + wr * 32;
        if (p.nsplit > 1) {
            // a partial result: accumulators as they are (relative to the running maximum), 16 bytes per store
            const int64_t rows_total = (int64_t)p.B * p.Hkv * p.R;
#pragma unroll
            for (int rt = 0; rt < RTW; ++rt) {
                const float l = l_run[rt] + shfl_xor(l_run[rt], 32);
                const int r = r0 + (wr * RTW + rt) * 32 + n;
                if (r < R) {
                    const int64_t row = (int64_t)split * rows_total + ((int64_t)b * p.Hkv + kvh) * p.R + r;
                    float* po = p.part_o + row * D;
#pragma unroll
                    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const f32x4 v = {O[rt][dt][4 * q4], O[rt][dt][4 * q4 + 1], O[rt][dt][4 * q4 + 2], O[rt][dt][4 * q4 + 3]};
                            *reinterpret_cast<f32x4*>(po + 32 * dt + 8 * q4 + 4 * hi) = v;
                        }
                    if (hi == 0) {
                        p.part_ml[row * 2] = m_run[rt];
                        p.part_ml[row * 2 + 1] = l;
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int rt = 0; rt < RTW; ++rt) {
            const float l = l_run[rt] + shfl_xor(l_run[rt], 32);
            const float inv = l > 0.f ? 1.f / l : 0.f;
            const int r = r0 + (wr * RTW + rt) * 32 + n;
            int64_t off = -1;
            if (r < R) {
                const int i = r / p.g, hg = r - i * p.g;
                const int h = kvh * p.g + hg;
                off = i * p.o_st + (int64_t)h * p.o_sh;
                if (p.lse && hi == 0)
                    p.lse[p.cu ? (int64_t)h * p.total + s0 + i : ((int64_t)b * p.Hq + h) * p.Lq + i] = l > 0.f ? (m_run[rt] + log2f(l)) * LN2 : -INFINITY;
            }
            if (hi == 0) roff[n] = off;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 v;
                    v[0] = pack_bf16x2(O[rt][dt][4 * q4] * inv, O[rt][dt][4 * q4 + 1] * inv);
                    v[1] = pack_bf16x2(O[rt][dt][4 * q4 + 2] * inv, O[rt][dt][4 * q4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(ob + n * OPB + (32 * dt + 8 * q4 + 4 * hi) * 2) = v;
                }
            // one wavefront's LDS operations complete in order: only the compiler must not move the reads up
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int q = 0; q < (32 * C8) / 64; ++q) {
                const int id = q * 64 + lane;
                const int row = id / C8, c = id - row * C8;
                const int64_t ro = roff[row];
                const u32x4 v = *reinterpret_cast<const u32x4*>(ob + row * OPB + c * 16);
                if (ro >= 0) *reinterpret_cast<u32x4*>(p.out + o_off + ro + 8 * c) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // before the next row tile overwrites the region
        }
    } else {
        float* mb = reinterpret_cast<float*>(smem);
#pragma unroll
        for (int rt = 0; rt < RTW; ++rt) {
            __syncthreads();  // tiles (or the previous row tile's merge data) are no longer needed
            const float l = l_run[rt] + shfl_xor(l_run[rt], 32);
            float* row = mb + (wk * 32 + n) * MP;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 v = {O[rt][dt][4 * q4], O[rt][dt][4 * q4 + 1], O[rt][dt][4 * q4 + 2], O[rt][dt][4 * q4 + 3]};
                    *reinterpret_cast<f32x4*>(row + 32 * dt + 8 * q4 + 4 * hi) = v;
                }
            if (hi == 0) {
                row[D] = m_run[rt];
                row[D + 1] = l;
            }
            __syncthreads();
            for (int task = tid; task < 32 * C8; task += NT) {
                const int rr = task / C8, c8 = task - rr * C8;
                const int r = r0 + rt * 32 + rr;
                if (r >= R) continue;
                float M = -INFINITY;
#pragma unroll
                for (int k = 0; k < NWK; ++k) M = fmaxf(M, mb[(k * 32 + rr) * MP + D]);
                float wgt[NWK], den = 0.f;
#pragma unroll
                for (int k = 0; k < NWK; ++k) {
                    const float mk = mb[(k * 32 + rr) * MP + D];
                    wgt[k] = (mk == -INFINITY) ? 0.f : fast_exp2(mk - M);
                    den += wgt[k] * mb[(k * 32 + rr) * MP + D + 1];
                }
                const float inv = den > 0.f ? 1.f / den : 0.f;
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
                for (int k = 0; k < NWK; ++k) {
                    const f32x4 a = *reinterpret_cast<const f32x4*>(mb + (k * 32 + rr) * MP + 8 * c8);
                    const f32x4 c = *reinterpret_cast<const f32x4*>(mb + (k * 32 + rr) * MP + 8 * c8 + 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        o[e] += wgt[k] * a[e];
                        o[4 + e] += wgt[k] * c[e];
                    }
                }
                if (p.nsplit > 1) {   // a partial result: the merged accumulators of the four wavefronts, unnormalised
                    const int64_t row = (int64_t)split * ((int64_t)p.B * p.Hkv * p.R) + ((int64_t)b * p.Hkv + kvh) * p.R + r;
                    float* po = p.part_o + row * D + 8 * c8;
                    *reinterpret_cast<f32x4*>(po) = f32x4{o[0], o[1], o[2], o[3]};
                    *reinterpret_cast<f32x4*>(po + 4) = f32x4{o[4], o[5], o[6], o[7]};
                    if (c8 == 0) {
                        p.part_ml[row * 2] = M;
                        p.part_ml[row * 2 + 1] = den;
                    }
                    continue;
                }
                const int i = r / p.g, hg = r - i * p.g;
                const int h = kvh * p.g + hg;
                u32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = pack_bf16x2(o[2 * e] * inv, o[2 * e + 1] * inv);
                *reinterpret_cast<u32x4*>(p.out + o_off + i * p.o_st + (int64_t)h * p.o_sh + 8 * c8) = v;
                if (p.lse && c8 == 0)
                    p.lse[p.cu ? (int64_t)h * p.total + s0 + i : ((int64_t)b * p.Hq + h) * p.Lq + i] = den > 0.f ? (M + log2f(den)) * LN2 : -INFINITY;
            }
        }
    }
}

// Combines the nsplit partial results of every (sequence, head, query row) in a fixed order (split 0, 1, ...): with
// M = max_s m_s and w_s = 2^(m_s - M), out = sum_s w_s o_s / sum_s w_s l_s and lse = (M + log2 sum_s w_s l_s) ln 2.
// D / 4 threads per row (16 bytes of fp32 in, 8 bytes of bf16 out each), 256 / (D / 4) rows per workgroup.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnParams p) {
    constexpr int TPR = D / 4, RPW = 256 / TPR;
    const int64_t rows_total = (int64_t)p.B * p.Hkv * p.R;
    const int64_t row = (int64_t)blockIdx.x * RPW + threadIdx.x / TPR;
    const int c4 = threadIdx.x % TPR;
    if (row >= rows_total) return;
    const int grp = (int)(row / p.R), r = (int)(row - (int64_t)grp * p.R);
    const int b = grp / p.Hkv, kvh = grp - b * p.Hkv;
    if (p.seq_active && p.seq_active[b] == 0) return;
    float M = -INFINITY;
    for (int s = 0; s < p.nsplit; ++s) M = fmaxf(M, p.part_ml[(s * rows_total + row) * 2]);
    float den = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < p.nsplit; ++s) {
        const float ms = p.part_ml[(s * rows_total + row) * 2];
        const float ls = p.part_ml[(s * rows_total + row) * 2 + 1];
        const float wgt = (ms == -INFINITY) ? 0.f : fast_exp2(ms - M);
        const f32x4 o = *reinterpret_cast<const f32x4*>(p.part_o + (s * rows_total + row) * D + 4 * c4);
        den += wgt * ls;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += wgt * o[e];
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    const int i = r / p.g, hg = r - i * p.g;
    const int h = kvh * p.g + hg;
    u32x2 v;
    v[0] = pack_bf16x2(acc[0] * inv, acc[1] * inv);
    v[1] = pack_bf16x2(acc[2] * inv, acc[3] * inv);
    *reinterpret_cast<u32x2*>(p.out + b * p.o_sb + i * p.o_st + (int64_t)h * p.o_sh + 4 * c4) = v;
    if (p.lse && c4 == 0)
        p.lse[((int64_t)b * p.Hq + h) * p.Lq + i] = den > 0.f ? (M + log2f(den)) * 0.6931471805599453f : -INFINITY;
}

int g_attn_split = 0;    // 0 = choose the key split across workgroups from the shape; 1 = never; 2..16 = force (dlm_set_option "attn_split")
int g_attn_nt = 1;       // 1 = non-temporal K/V loads in the one-workgroup-per-KV-head shape (default); 0 = never (tuning)
int g_attn_variant = 0;  // 0 = choose by shape; 1..3 force a kernel shape (dlm_set_option "attn_variant")
int g_attn_remap = 7;    // XCD-grouped grids: bit 0 forward and dQ, bit 1 longest key range first, bit 2 dK / dV (dlm_set_option "attn_remap")

// The kernel shape the planner picks for a problem (0 = "automatic" resolved).  Measured on MI355X (us, GPU time):
//   g * Lq <= 32 (every rollout step): one key-split workgroup per (sequence, KV head); sized for two per CU it is
//     8 - 10 % faster than sized for one even when only one is resident (c2 22.4 -> 19.7, c3 72 -> 66, c5a 173 -> 162);
//   more rows: 128-row workgroups; with at most one of them per CU, eight wavefronts in two key groups (two wavefronts
//     per SIMD from one workgroup: c4 39.1 -> 32.2), otherwise two or three four-wavefront workgroups per CU.
static int plan_variant(const AttnParams& p) {
    const int64_t BH = (int64_t)p.B * p.Hkv;
    int variant = g_attn_variant;
    if (variant == 0) {
        const int64_t wgs128 = BH * ((p.R + 127) / 128) * (p.nsplit > 1 ? p.nsplit : 1);
        if (p.R <= 32) variant = 12;          // waves split the keys, merge on chip
        // far too few 128-row workgroups for 256 CUs (and no workspace to split the keys across workgroups with):
        // 32-row key-split tiles (K/V re-read per row tile, through one L2)
        else if (wgs128 <= 64 || (wgs128 <= 128 && p.R <= 64)) variant = 11;
        else if (wgs128 <= 256) variant = 13; // one 128-row workgroup per CU at most: eight wavefronts, two key groups
        else if (wgs128 >= 768) variant = 6;  // 128-row workgroups, three resident per CU (softmax of one overlaps MFMA of another)
        else variant = 4;                     // 128-row workgroups, two resident per CU, deeper prefetch
    }
    return variant;
}

// How many workgroups share the keys of one row tile.  A split costs a second launch (the merge) and (d + 2) * 4 bytes
// written and read again per row and split, so it pays only where the unsplit launch leaves most of the chip idle: at
// most 128 workgroups (half the CUs) and at least 32 key tiles.  Then the count brings the launch to about one
// workgroup per CU with at least four key tiles each.  Measured (us): 1 x 32 heads x 8192 keys 114 -> 33 (8 splits);
// 1 x 32/8 heads x 16384 keys 318 -> 43 (16); 8 x 28/4 heads x 4096 keys 88 -> 40 (4); 4 x 32 heads x 2048 keys 33 -> 30 (2).
// With 256 or more workgroups every split measured slower (c2 19.7 -> 28.4, c3 66 -> 81, c4 32 -> 50, c5a 162 -> 180):
// those launches already keep the memory system busy and the partials and the second launch are pure cost.
// Never in packed mode (each sequence has its own key range) and only when the caller provides the workspace.
static int plan_nsplit(const dlm_attn_args* a) {
    if (a->cu_seqlens || g_attn_split == 1) return 1;
    const int g = a->Hq / a->Hkv;
    const int64_t R = (int64_t)g * a->Lq, BH = (int64_t)a->B * a->Hkv;
    const int64_t tiles = ((int64_t)a->prefix.len + 31) / 32 + ((int64_t)a->block.len + 31) / 32 + ((int64_t)a->suffix.len + 31) / 32;
    int64_t n = 1;
    if (g_attn_split >= 2) n = g_attn_split;
    else if (g_attn_variant == 0) {
        const int64_t wgs = R <= 32 ? BH : BH * ((R + 127) / 128);
        if (wgs <= 128 && tiles >= 32) n = 256 / wgs;
    }
    if (n > 16) n = 16;
    if (n > tiles / 4) n = tiles / 4;         // at least four key tiles per workgroup
    return n < 1 ? 1 : (int)n;
}

template <int D, bool BC>
static int launch_attn(const AttnParams& p, hipStream_t st) {
    const int64_t BH = (int64_t)p.B * p.Hkv;
    const int ns = p.nsplit > 1 ? p.nsplit : 1;
    int variant = plan_variant(p);
    if (variant == 0 + 11 || (variant == 1 && p.R > 32)) {
        // 32-row workgroups whose wavefronts split the keys, several row tiles per (sequence, KV head), XCD-grouped
        AttnParams q = p;
        const int64_t n_wg = set_remap(q.remap, BH, (p.R + 31) / 32 * ns, BC && (g_attn_remap & 2));
        if (n_wg > 0) {
            hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 1>), dim3((unsigned)n_wg), dim3(256), 0, st, q);
            return check_hip(hipGetLastError(), "attn_kernel launch");
        }
        variant = 2;
    }
    if (variant >= 8 && p.R <= 32) {   // key-split alternatives (tuning)
        const dim3 grid(ns, p.Hkv, p.B);
        if (variant == 12) hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 1, 2, true>), grid, dim3(256), 0, st, p);
        else if (variant == 8) hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 2, 1, true>), grid, dim3(256), 0, st, p);
        else if (variant == 9) hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 3, 1, true>), grid, dim3(256), 0, st, p);
        else hipLaunchKernelGGL((attn_kernel<D, 1, 8, 1, BC, 1, 1, true>), grid, dim3(512), 0, st, p);
        return check_hip(hipGetLastError(), "attn_kernel launch");
    }
    if (variant == 13 || variant == 14) {
        // 128-row workgroups of 8 wavefronts: two key groups of 4 (two wavefronts per SIMD from ONE workgroup per CU),
        // combined through LDS at the end.  For row counts that give at most one 128-row workgroup per CU.
        dim3 grid((p.R + 127) / 128 * ns, p.Hkv, p.B);
        AttnParams q = p;
        if ((g_attn_remap & 1) && grid.x >= 2) {
            const int64_t n_wg = set_remap(q.remap, BH, (int)grid.x, BC && (g_attn_remap & 2));
            if (n_wg > 0) grid = dim3((unsigned)n_wg);
            else q = p;
        }
        if (variant == 13) hipLaunchKernelGGL((attn_kernel<D, 4, 2, 1, BC, 1, 1>), grid, dim3(512), 0, st, q);
        else hipLaunchKernelGGL((attn_kernel<D, 4, 2, 1, BC, 2, 1>), grid, dim3(512), 0, st, q);
        return check_hip(hipGetLastError(), "attn_kernel launch");
    }
    if (variant == 15) {
        // the software-pipelined 128-row shape (d = 128 only), two workgroups per CU
        if constexpr (D == 128) {
            dim3 grid((p.R + 127) / 128 * ns, p.Hkv, p.B);
            AttnParams q = p;
            if ((g_attn_remap & 1) && grid.x >= 2) {
                const int64_t n_wg = set_remap(q.remap, BH, (int)grid.x, BC && (g_attn_remap & 2));
                if (n_wg > 0) grid = dim3((unsigned)n_wg);
                else q = p;
            }
            hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 1, 2, false, true>), grid, dim3(256), 0, st, q);
            return check_hip(hipGetLastError(), "attn_kernel launch");
        } else {
            variant = 4;
        }
    }
    if (variant >= 8) variant = 0 + 4;
    if (variant >= 4) {   // 128-row workgroups, several resident per CU
        dim3 grid((p.R + 127) / 128 * ns, p.Hkv, p.B);
        AttnParams q = p;
        if ((g_attn_remap & 1) && grid.x >= 2) {
            const int64_t n_wg = set_remap(q.remap, BH, (int)grid.x, BC && (g_attn_remap & 2));
            if (n_wg > 0) grid = dim3((unsigned)n_wg);
            else q = p;
        }
        if (variant == 4) hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 2, 2>), grid, dim3(256), 0, st, q);
        else if (variant == 5) hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 2, 3>), grid, dim3(256), 0, st, q);
        else if (variant == 6) hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 1, 3>), grid, dim3(256), 0, st, q);
        else hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 1, 4>), grid, dim3(256), 0, st, q);
        return check_hip(hipGetLastError(), "attn_kernel launch");
    }
    if (variant == 1) {
        if (g_attn_nt) hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 1, 1, true>), dim3(ns, p.Hkv, p.B), dim3(256), 0, st, p);
        else hipLaunchKernelGGL((attn_kernel<D, 1, 4, 1, BC, 1>), dim3(ns, p.Hkv, p.B), dim3(256), 0, st, p);
    } else if (variant == 2) {
        hipLaunchKernelGGL((attn_kernel<D, 4, 1, 1, BC, 3>), dim3((p.R + 127) / 128 * ns, p.Hkv, p.B), dim3(256), 0, st, p);
    } else {
        hipLaunchKernelGGL((attn_kernel<D, 4, 1, 2, BC, 3>), dim3((p.R + 255) / 256 * ns, p.Hkv, p.B), dim3(256), 0, st, p);
    }
    return check_hip(hipGetLastError(), "attn_kernel launch");
}

static int validate_seg(const dlm_kv_seg& s, const char* name, int d) {
    if (s.len < 0) return fail(DLM_ERR_INVALID_ARG, "block_attn: %s.len < 0", name);
    if (s.rule < DLM_SEG_CAUSAL || s.rule > DLM_SEG_SAME_BLOCK) return fail(DLM_ERR_INVALID_ARG, "block_attn: %s.rule %d unknown", name, s.rule);
    if (s.len == 0) return DLM_OK;
    if (!s.k || !s.v) return fail(DLM_ERR_INVALID_ARG, "block_attn: %s has null k/v", name);
    if (!aligned16(s.k) || !aligned16(s.v)) return fail(DLM_ERR_UNSUPPORTED, "block_attn: %s k/v not 16-byte aligned", name);
    if ((s.stride_b | s.stride_h | s.stride_t) % 8) return fail(DLM_ERR_UNSUPPORTED, "block_attn: %s strides must be multiples of 8", name);
    if (s.stride_t < d) return fail(DLM_ERR_INVALID_ARG, "block_attn: %s.stride_t < d", name);
    if (s.pos0 < 0 || (int64_t)s.pos0 + s.len > (1 << 30)) return fail(DLM_ERR_INVALID_ARG, "block_attn: %s positions outside [0, 2^30]", name);
    return DLM_OK;
}

static int validate_attn(const dlm_attn_args* a) {
    if (!a) return fail(DLM_ERR_INVALID_ARG, "block_attn: null args");
    if (a->struct_size != sizeof(dlm_attn_args))
        return fail(DLM_ERR_INVALID_ARG, "block_attn: struct_size %u != %zu", a->struct_size, sizeof(dlm_attn_args));
    if (a->B < 0 || a->Lq < 0 || a->Hq <= 0 || a->Hkv <= 0 || a->d <= 0)
        return fail(DLM_ERR_INVALID_ARG, "block_attn: bad sizes B=%d Lq=%d Hq=%d Hkv=%d d=%d", a->B, a->Lq, a->Hq, a->Hkv, a->d);
    if (a->Hq % a->Hkv) return fail(DLM_ERR_INVALID_ARG, "block_attn: Hq=%d is not a multiple of Hkv=%d", a->Hq, a->Hkv);
    if (a->d != 64 && a->d != 128) return fail(DLM_ERR_UNSUPPORTED, "block_attn: head_dim %d (supported: 64, 128)", a->d);
    if (a->mask_mode != DLM_MASK_FULL && a->mask_mode != DLM_MASK_BLOCK_CAUSAL)
        return fail(DLM_ERR_INVALID_ARG, "block_attn: unknown mask_mode %d", a->mask_mode);
    if (a->mask_mode == DLM_MASK_FULL && (a->prefix.rule | a->block.rule | a->suffix.rule))
        return fail(DLM_ERR_INVALID_ARG, "block_attn: segment rules need the block-causal mask mode");
    if (a->mask_mode == DLM_MASK_BLOCK_CAUSAL) {
        if (a->block_size < 1) return fail(DLM_ERR_INVALID_ARG, "block_attn: block-causal needs block_size >= 1");
        if (a->q_pos0 < 0 || (int64_t)a->q_pos0 + a->Lq + a->block_size > (1 << 30))
            return fail(DLM_ERR_INVALID_ARG, "block_attn: query positions outside [0, 2^30]");
    }
    if (a->B > 65535 || a->Hkv > 65535) return fail(DLM_ERR_UNSUPPORTED, "block_attn: B or Hkv above 65535");
    if ((int64_t)a->Lq * (a->Hq / a->Hkv) > (1 << 30)) return fail(DLM_ERR_UNSUPPORTED, "block_attn: too many rows per KV head");
    if (a->cu_seqlens) {
        if (a->prefix.len || a->suffix.len || a->prefix_len_b)
            return fail(DLM_ERR_INVALID_ARG, "block_attn: packed mode takes the block segment only");
        if (a->block.len != a->Lq) return fail(DLM_ERR_INVALID_ARG, "block_attn: packed mode needs block.len == Lq (the longest sequence)");
        if (a->total_tokens < 0) return fail(DLM_ERR_INVALID_ARG, "block_attn: total_tokens < 0");
        if ((int64_t)a->total_tokens > (int64_t)a->B * a->Lq) return fail(DLM_ERR_INVALID_ARG, "block_attn: total_tokens > B * Lq");
        if (a->total_tokens == 0) return DLM_OK;   // an empty packed batch: nothing is read
    }
    int rc;
    if ((rc = validate_seg(a->prefix, "prefix", a->d)) != DLM_OK) return rc;
    if ((rc = validate_seg(a->block, "block", a->d)) != DLM_OK) return rc;
    if ((rc = validate_seg(a->suffix, "suffix", a->d)) != DLM_OK) return rc;
    if ((int64_t)a->prefix.len + a->block.len + a->suffix.len > (1 << 30))
        return fail(DLM_ERR_UNSUPPORTED, "block_attn: more than 2^30 keys");
    if (a->B == 0 || a->Lq == 0 || (a->cu_seqlens && a->total_tokens == 0)) return DLM_OK;
    if (!a->q || !a->out) return fail(DLM_ERR_INVALID_ARG, "block_attn: null q/out");
    if (!aligned16(a->q) || !aligned16(a->out)) return fail(DLM_ERR_UNSUPPORTED, "block_attn: q/out not 16-byte aligned");
    if ((a->q_stride_b | a->q_stride_t | a->q_stride_h | a->o_stride_b | a->o_stride_t | a->o_stride_h) % 8)
        return fail(DLM_ERR_UNSUPPORTED, "block_attn: q/out strides must be multiples of 8");
    if (a->q_stride_h < a->d || a->o_stride_h < a->d) return fail(DLM_ERR_INVALID_ARG, "block_attn: head stride < d");
    if (!(a->scale == a->scale)) return fail(DLM_ERR_INVALID_ARG, "block_attn: scale is NaN");
    return DLM_OK;
}

}  // namespace dlm

using namespace dlm;

extern "C" int dlm_set_option(const char* name, int value) {
    if (!name) return fail(DLM_ERR_INVALID_ARG, "set_option: null name");
    if (!strcmp(name, "attn_variant")) {
        if (value < 0 || value > 15) return fail(DLM_ERR_INVALID_ARG, "set_option: attn_variant must be 0..15");
        g_attn_variant = value;
        return DLM_OK;
    }
    if (!strcmp(name, "lmhead_variant")) return lm_set_variant(value);
    if (!strcmp(name, "lmhead_block")) return lm_set_block(value);
    if (!strcmp(name, "lmhead_nt")) return lm_set_nt(value);
    if (!strcmp(name, "lmhead_cus")) return lm_set_cus(value);
    if (!strcmp(name, "kv_copy_unroll")) return copy_set_unroll(value);
    if (!strcmp(name, "attn_remap")) {
        if (value < 0 || value > 7) return fail(DLM_ERR_INVALID_ARG, "set_option: attn_remap must be 0..7");
        g_attn_remap = value;
        return DLM_OK;
    }
    if (!strcmp(name, "attn_split")) {
        if (value < 0 || value > 16) return fail(DLM_ERR_INVALID_ARG, "set_option: attn_split must be 0..16");
        g_attn_split = value;
        return DLM_OK;
    }
    if (!strcmp(name, "attn_nt")) {
        if (value < 0 || value > 1) return fail(DLM_ERR_INVALID_ARG, "set_option: attn_nt must be 0 or 1");
        g_attn_nt = value;
        return DLM_OK;
    }
    return fail(DLM_ERR_INVALID_ARG, "set_option: unknown option '%s'", name);
}

static size_t split_workspace_bytes(const dlm_attn_args* a, int nsplit) {
    if (nsplit <= 1) return 0;
    return (size_t)nsplit * (size_t)a->B * (size_t)a->Hq * (size_t)a->Lq * (size_t)(a->d + 2) * sizeof(float);
}

extern "C" size_t dlm_block_attn_workspace_bytes(const dlm_attn_args* a) {
    if (!a || a->struct_size != sizeof(dlm_attn_args) || a->B <= 0 || a->Lq <= 0 || a->Hq <= 0 || a->Hkv <= 0 ||
        a->Hq % a->Hkv || a->d <= 0)
        return 0;
    return split_workspace_bytes(a, plan_nsplit(a));
}

extern "C" int dlm_block_attn(const dlm_attn_args* a, void* stream) {
    int rc = validate_attn(a);
    if (rc != DLM_OK) return rc;
    if (a->B == 0 || a->Lq == 0 || (a->cu_seqlens && a->total_tokens == 0)) return DLM_OK;
    AttnParams p;
    p.B = a->B; p.Lq = a->Lq; p.Hq = a->Hq; p.Hkv = a->Hkv; p.g = a->Hq / a->Hkv; p.R = p.g * a->Lq;
    p.q = (const uint16_t*)a->q; p.q_sb = a->q_stride_b; p.q_st = a->q_stride_t; p.q_sh = a->q_stride_h;
    const dlm_kv_seg* segs[3] = {&a->prefix, &a->block, &a->suffix};
    for (int s = 0; s < 3; ++s) {
        p.seg[s].k = (const uint16_t*)segs[s]->k; p.seg[s].v = (const uint16_t*)segs[s]->v;
        p.seg[s].len = segs[s]->len; p.seg[s].pos0 = segs[s]->pos0;
        p.seg[s].sb = segs[s]->stride_b; p.seg[s].sh = segs[s]->stride_h; p.seg[s].st = segs[s]->stride_t;
        p.seg[s].rule = segs[s]->rule;
    }
    p.prefix_len_b = a->prefix_len_b;
    p.bs = a->block_size; p.q_pos0 = a->q_pos0;
    const float scale = a->scale > 0.f ? a->scale : 1.0f / sqrtf((float)a->d);
    p.scale_log2 = scale * 1.4426950408889634f;
    p.out = (uint16_t*)a->out; p.o_sb = a->o_stride_b; p.o_st = a->o_stride_t; p.o_sh = a->o_stride_h;
    p.lse = a->lse;
    p.cu = a->cu_seqlens; p.total = a->total_tokens;
    p.seq_active = a->seq_active;
    p.remap = no_remap();
    // The key split across workgroups is taken only when the caller brought the workspace it needs.
    p.nsplit = 1; p.part_o = nullptr; p.part_ml = nullptr;
    const int ns = plan_nsplit(a);
    const size_t need = split_workspace_bytes(a, ns);
    if (ns > 1 && a->workspace && a->workspace_bytes >= need && aligned16(a->workspace)) {
        const size_t rows_total = (size_t)a->B * a->Hq * a->Lq;
        p.nsplit = ns;
        p.part_o = (float*)a->workspace;
        p.part_ml = p.part_o + (size_t)ns * rows_total * a->d;
    }
    hipStream_t st = (hipStream_t)stream;
    const bool bc = a->mask_mode == DLM_MASK_BLOCK_CAUSAL;
    if (a->d == 128) rc = bc ? launch_attn<128, true>(p, st) : launch_attn<128, false>(p, st);
    else rc = bc ? launch_attn<64, true>(p, st) : launch_attn<64, false>(p, st);
    if (rc != DLM_OK || p.nsplit <= 1) return rc;
    const int64_t rows_total = (int64_t)a->B * a->Hq * a->Lq;
    if (a->d == 128) hipLaunchKernelGGL(attn_merge_kernel<128>, dim3((unsigned)((rows_total + 7) / 8)), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(attn_merge_kernel<64>, dim3((unsigned)((rows_total + 15) / 16)), dim3(256), 0, st, p);
    return check_hip(hipGetLastError(), "attn_merge_kernel launch");
}
