// dlm_unmask_commit, dlm_mask_compact, dlm_kv_refresh: selection of the positions
// to fix in this denoising step, token / mask update, compaction of the rows that
// stay masked, and the K/V copies into the cache.
//
// Selection is integer work decided by fp32 compares: one wavefront owns one
// commit group (a block of the rollout, or one block of a block-diffusion
// sequence), keeps the group's confidences in registers and finds arg-maxima
// with xor-shuffles, so the result is independent of scheduling.
#include "common.hpp"

namespace dlm {

struct Cand {
    float v;
    int i;
};
__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
    return av > bv || (av == bv && ai < bi);
}
__device__ __forceinline__ Cand wave_argmax(Cand c) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = shfl_xor(c.v, off);
        int oi = shfl_xor(c.i, off);
        if (better(ov, oi, c.v, c.i)) { c.v = ov; c.i = oi; }
    }
    return c;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += shfl_xor(v, off);
    return v;
}

struct CommitParams {
    int B, n_pos, group_len, n_groups;
    int rule;
    float threshold;
    int force_top1, k;
    const float* conf;
    const int32_t* tok;
    int32_t* x;
    int64_t x_stride_b;
    int x_pos0;
    uint8_t* mask;
    int64_t mask_stride_b;
    uint8_t* commit_now;
    int32_t *n_commit, *remaining;
    int16_t* commit_step;
    int step;
};

// CH = ceil(group_len / 64): positions per lane.
template <int CH>
__global__ __launch_bounds__(256) void commit_wave_kernel(CommitParams p) {
    const int lane = lane_id();
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (gw >= p.B * p.n_groups) return;
    const int b = gw / p.n_groups, gi = gw - b * p.n_groups;
    const int g0 = gi * p.group_len;
    const int64_t base = (int64_t)b * p.n_pos + g0;
    uint8_t* mrow = p.mask + b * p.mask_stride_b + g0;

    float cf[CH];
    bool masked[CH], chosen[CH];
    int cnt = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int i = lane + 64 * c;
        masked[c] = (i < p.group_len) && (mrow[i] != 0);
        chosen[c] = false;
        float v = -INFINITY;
        if (masked[c]) {
            v = p.conf[base + i];
            if (!(v == v)) v = -INFINITY;
            ++cnt;
        }
        cf[c] = v;
    }
    cnt = wave_sum(cnt);
    int ncom = 0;
    if (cnt > 0) {
        if (p.rule == DLM_RULE_THRESHOLD) {
#pragma unroll
            for (int c = 0; c < CH; ++c) chosen[c] = masked[c] && (cf[c] >= p.threshold);
            if (p.force_top1) {
                Cand best{-INFINITY, 0x7fffffff};
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (masked[c] && better(cf[c], lane + 64 * c, best.v, best.i)) best = Cand{cf[c], lane + 64 * c};
                best = wave_argmax(best);
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (masked[c] && best.i == lane + 64 * c) chosen[c] = true;
            }
        } else {
            const int kk = min(p.k, cnt);
            for (int it = 0; it < kk; ++it) {
                Cand best{-INFINITY, 0x7fffffff};
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (masked[c] && !chosen[c] && better(cf[c], lane + 64 * c, best.v, best.i))
                        best = Cand{cf[c], lane + 64 * c};
                best = wave_argmax(best);
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (masked[c] && best.i == lane + 64 * c) chosen[c] = true;
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = lane + 64 * c;
            if (chosen[c]) {
                p.x[b * p.x_stride_b + p.x_pos0 + g0 + i] = p.tok[base + i];
                mrow[i] = 0;
                if (p.commit_step) p.commit_step[base + i] = (int16_t)p.step;
                ++ncom;
            }
        }
        ncom = wave_sum(ncom);
    }
    if (p.commit_now) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = lane + 64 * c;
            if (i < p.group_len) p.commit_now[base + i] = chosen[c] ? 1 : 0;
        }
    }
    if (lane == 0) {
        if (p.n_groups == 1) {
            p.n_commit[b] = ncom;
            p.remaining[b] = cnt - ncom;
        } else if (cnt > 0) {
            atomicAdd(&p.n_commit[b], ncom);           // integer sums: order-independent
            atomicAdd(&p.remaining[b], cnt - ncom);
        }
    }
}

struct CopyParams {
    const uint16_t *sk, *sv;
    int64_t s_sb, s_sh, s_st;
    uint16_t *ck, *cv;
    int64_t c_sb, c_sh, c_st;
    int len, d8;  // rows, 16-byte chunks per row
    int cache_pos0;
    // conditional write-back
    int mode;  // 0 unconditional, DLM_WB_BLOCK_WHEN_DONE, DLM_WB_COMMITTED_ROWS, DLM_WB_WHILE_ACTIVE
    const int32_t *n_commit, *remaining;
    const uint8_t* commit_now;
    int n_pos;
    const int32_t* active_in;  // DLM_WB_WHILE_ACTIVE: copy sequence b iff active_in[b] != 0
    int Hkv;
    int split;                 // kv_copy_kernel: K and V by different workgroups
    int nt;                    // bit 0: non-temporal loads, bit 1: non-temporal stores (split form only)
};

// Rollout-sized problems (one commit group per sequence, at most 16384 positions in all): ONE workgroup
// selects for every sequence (a wavefront per sequence, 16 at a time), then compacts the still-masked rows
// in order and publishes the total, so a denoising step needs a single small launch here.
constexpr int FUSED_MAX_POS = 16384;
template <int CH>
__global__ __launch_bounds__(1024) void commit_fused_kernel(CommitParams p, int32_t* row_idx, int32_t* next_m,
                                                            int32_t* host_total, int32_t* host_max, CopyParams cp) {
    __shared__ uint8_t newmask[FUSED_MAX_POS];
    __shared__ int wave_tot[16], wave_max[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (blockIdx.x > 0) {
        // DLM_WB_WHILE_ACTIVE: workgroups 1.. copy the block's K/V of one (sequence, KV head) each.  They read
        // nothing that workgroup 0 writes (active_in is the caller's copy of the previous step's counts), so the
        // write-back shares the selection's launch instead of following it.
        const int g = blockIdx.x - 1, b = g / cp.Hkv, h = g - b * cp.Hkv;
        if (cp.active_in[b] == 0) return;
        const uint16_t* sk = cp.sk + b * cp.s_sb + h * cp.s_sh;
        const uint16_t* sv = cp.sv + b * cp.s_sb + h * cp.s_sh;
        uint16_t* ck = cp.ck + b * cp.c_sb + h * cp.c_sh + (int64_t)cp.cache_pos0 * cp.c_st;
        uint16_t* cv = cp.cv + b * cp.c_sb + h * cp.c_sh + (int64_t)cp.cache_pos0 * cp.c_st;
        const int total = cp.len * cp.d8;
        for (int e = tid; e < total; e += 1024) {
            const int t = e / cp.d8, c = e - t * cp.d8;
            const u32x4 kk = *reinterpret_cast<const u32x4*>(sk + t * cp.s_st + c * 8);
            const u32x4 vv = *reinterpret_cast<const u32x4*>(sv + t * cp.s_st + c * 8);
            *reinterpret_cast<u32x4*>(ck + t * cp.c_st + c * 8) = kk;
            *reinterpret_cast<u32x4*>(cv + t * cp.c_st + c * 8) = vv;
        }
        return;
    }
    int left_max = 0;                 // most positions any of this wavefront's sequences still has masked
    for (int b = w; b < p.B; b += 16) {
        const int64_t base = (int64_t)b * p.n_pos;
        uint8_t* mrow = p.mask + b * p.mask_stride_b;
        float cf[CH];
        bool masked[CH], chosen[CH];
        int cnt = 0;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = lane + 64 * c;
            masked[c] = (i < p.group_len) && (mrow[i] != 0);
            chosen[c] = false;
            float v = -INFINITY;
            if (masked[c]) {
                v = p.conf[base + i];
                if (!(v == v)) v = -INFINITY;
                ++cnt;
            }
            cf[c] = v;
        }
        cnt = wave_sum(cnt);
        int ncom = 0;
        if (cnt > 0) {
            if (p.rule == DLM_RULE_THRESHOLD) {
#pragma unroll
                for (int c = 0; c < CH; ++c) chosen[c] = masked[c] && (cf[c] >= p.threshold);
                if (p.force_top1) {
                    Cand best{-INFINITY, 0x7fffffff};
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        if (masked[c] && better(cf[c], lane + 64 * c, best.v, best.i)) best = Cand{cf[c], lane + 64 * c};
                    best = wave_argmax(best);
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        if (masked[c] && best.i == lane + 64 * c) chosen[c] = true;
                }
            } else {
                const int kk = min(p.k, cnt);
                for (int it = 0; it < kk; ++it) {
                    Cand best{-INFINITY, 0x7fffffff};
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        if (masked[c] && !chosen[c] && better(cf[c], lane + 64 * c, best.v, best.i))
                            best = Cand{cf[c], lane + 64 * c};
                    best = wave_argmax(best);
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        if (masked[c] && best.i == lane + 64 * c) chosen[c] = true;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = lane + 64 * c;
            if (i < p.group_len) {
                if (chosen[c]) {
                    p.x[b * p.x_stride_b + p.x_pos0 + i] = p.tok[base + i];
                    mrow[i] = 0;
                    if (p.commit_step) p.commit_step[base + i] = (int16_t)p.step;
                    ++ncom;
                }
                if (p.commit_now) p.commit_now[base + i] = chosen[c] ? 1 : 0;
                newmask[base + i] = (masked[c] && !chosen[c]) ? 1 : 0;
            }
        }
        ncom = wave_sum(ncom);
        left_max = max(left_max, cnt - ncom);
        if (lane == 0) {
            p.n_commit[b] = ncom;
            p.remaining[b] = cnt - ncom;
        }
    }
    if (lane == 0) wave_max[w] = left_max;
    __syncthreads();
    // ordered compaction of the still-masked positions (from LDS)
    const int N = p.B * p.n_pos;
    int running = 0;
    for (int start = 0; start < N; start += 1024) {
        const int idx = start + tid;
        const bool flag = (idx < N) && newmask[idx] != 0;
        const unsigned long long bal = __ballot(flag);
        const int prefix = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[w] = __popcll(bal);
        __syncthreads();
        int off = running, all = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = wave_tot[j];
            if (j < w) off += t;
            all += t;
        }
        if (flag && row_idx) row_idx[off + prefix] = idx;
        running += all;
        __syncthreads();
    }
    if (tid == 0) {
        if (next_m) *next_m = running;
        if (host_total) {
            if (host_max) {
                int mx = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j) mx = max(mx, wave_max[j]);
                __hip_atomic_store(host_max, mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __hip_atomic_store(host_total, running, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);   // orders the maximum before it
        }
    }
}

// Many small commit groups (block-diffusion full-sequence pass: 65536 groups of 4): one LANE per group, the
// group's confidences in registers, so the whole call is a single pass over ~15 bytes per position.
template <int GL>
__global__ __launch_bounds__(256) void commit_lane_kernel(CommitParams p) {
    const int64_t total = (int64_t)p.B * p.n_groups;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = gid < total;
    const int b = active ? (int)(gid / p.n_groups) : -1;
    const int gi = active ? (int)(gid - (int64_t)b * p.n_groups) : 0;
    int ncom = 0, cnt = 0;
    if (active) {
        const int g0 = gi * GL;
        const int64_t base = (int64_t)b * p.n_pos + g0;
        uint8_t* mrow = p.mask + b * p.mask_stride_b + g0;
        float cf[GL];
        bool masked[GL], chosen[GL];
#pragma unroll
        for (int i = 0; i < GL; ++i) {
            masked[i] = mrow[i] != 0;
            chosen[i] = false;
            float v = -INFINITY;
            if (masked[i]) {
                v = p.conf[base + i];
                if (!(v == v)) v = -INFINITY;
                ++cnt;
            }
            cf[i] = v;
        }
        if (cnt > 0) {
            if (p.rule == DLM_RULE_THRESHOLD) {
#pragma unroll
                for (int i = 0; i < GL; ++i) chosen[i] = masked[i] && (cf[i] >= p.threshold);
                if (p.force_top1) {
                    float bv = -INFINITY;
                    int bi = 0x7fffffff;
#pragma unroll
                    for (int i = 0; i < GL; ++i)
                        if (masked[i] && better(cf[i], i, bv, bi)) { bv = cf[i]; bi = i; }
#pragma unroll
                    for (int i = 0; i < GL; ++i)
                        if (i == bi) chosen[i] = true;
                }
            } else {
                const int kk = min(p.k, cnt);
                for (int it = 0; it < kk; ++it) {
                    float bv = -INFINITY;
                    int bi = 0x7fffffff;
#pragma unroll
                    for (int i = 0; i < GL; ++i)
                        if (masked[i] && !chosen[i] && better(cf[i], i, bv, bi)) { bv = cf[i]; bi = i; }
#pragma unroll
                    for (int i = 0; i < GL; ++i)
                        if (i == bi) chosen[i] = true;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < GL; ++i) {
            if (chosen[i]) {
                p.x[b * p.x_stride_b + p.x_pos0 + g0 + i] = p.tok[base + i];
                mrow[i] = 0;
                if (p.commit_step) p.commit_step[base + i] = (int16_t)p.step;
                ++ncom;
            }
            if (p.commit_now) p.commit_now[base + i] = chosen[i] ? 1 : 0;
        }
    }
    // per-sequence totals: one atomic per wavefront when all its lanes belong to one sequence
    const int b0 = __builtin_amdgcn_readfirstlane(b);
    const bool uniform = __all(b == b0 || !active) && b0 >= 0;
    if (uniform) {
        const int wn = wave_sum(ncom), wr = wave_sum(cnt - ncom);
        if (lane_id() == 0 && (wn | wr)) {
            atomicAdd(&p.n_commit[b0], wn);
            atomicAdd(&p.remaining[b0], wr);
        }
    } else if (active && cnt > 0) {
        atomicAdd(&p.n_commit[b], ncom);
        atomicAdd(&p.remaining[b], cnt - ncom);
    }
}

__global__ void zero2_i32_kernel(int32_t* a, int32_t* b, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { a[i] = 0; b[i] = 0; }
}

// Ordered stream compaction of mask != 0 by a single 1024-thread workgroup.
__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t* mask, int64_t mask_stride_b, int B, int n_pos,
                                                        int32_t* row_idx, int32_t* m_out) {
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t N = (int64_t)B * n_pos;
    int running = 0;
    for (int64_t start = 0; start < N; start += 1024) {
        const int64_t idx = start + tid;
        bool flag = false;
        if (idx < N) {
            const int b = (int)(idx / n_pos), i = (int)(idx - (int64_t)b * n_pos);
            flag = mask[b * mask_stride_b + i] != 0;
        }
        const unsigned long long bal = __ballot(flag);
        const int prefix = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[w] = __popcll(bal);
        __syncthreads();
        int off = running, all = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = wave_tot[j];
            if (j < w) off += t;
            all += t;
        }
        if (flag) row_idx[off + prefix] = (int32_t)idx;
        running += all;
        __syncthreads();
    }
    if (tid == 0) *m_out = running;
}


template <int U>
__global__ __launch_bounds__(256) void kv_copy_kernel(CopyParams p) {
    const int b = blockIdx.z;
    // split != 0: grid.y = 2 * Hkv, the first Hkv rows of workgroups copy K, the others V (one read and one write
    // stream per workgroup instead of two of each)
    const int h = p.split ? (int)blockIdx.y % p.Hkv : (int)blockIdx.y;
    const bool do_k = !p.split || (int)blockIdx.y < p.Hkv, do_v = !p.split || (int)blockIdx.y >= p.Hkv;
    if (p.mode == DLM_WB_BLOCK_WHEN_DONE) {
        if (!(p.remaining[b] == 0 && p.n_commit[b] > 0)) return;
    }
    if (p.mode == DLM_WB_WHILE_ACTIVE && p.active_in[b] == 0) return;
    const uint32_t total = (uint32_t)p.len * (uint32_t)p.d8;      // < 2^31 (checked by the host)
    const uint16_t* sk = p.sk + b * p.s_sb + h * p.s_sh;
    const uint16_t* sv = p.sv + b * p.s_sb + h * p.s_sh;
    uint16_t* ck = p.ck + b * p.c_sb + h * p.c_sh + (int64_t)p.cache_pos0 * p.c_st;
    uint16_t* cv = p.cv + b * p.c_sb + h * p.c_sh + (int64_t)p.cache_pos0 * p.c_st;
    u32x4 kreg[U], vreg[U];
    int64_t so[U], co[U];
    bool ok[U];
    // 16-byte pieces per row: a power of two for the usual head sizes (a shift instead of a division per piece)
    const int sh = ((p.d8 & (p.d8 - 1)) == 0) ? __builtin_ctz(p.d8) : -1;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t e = (blockIdx.x * U + u) * 256u + threadIdx.x;
        ok[u] = e < total;
        const uint32_t ec = ok[u] ? e : 0u;
        const int t = (int)(sh >= 0 ? ec >> sh : ec / (uint32_t)p.d8);
        const int c = (int)(ec - (uint32_t)t * (uint32_t)p.d8);
        if (p.mode == DLM_WB_COMMITTED_ROWS && ok[u]) ok[u] = p.commit_now[(int64_t)b * p.n_pos + t] != 0;
        so[u] = (int64_t)t * p.s_st + c * 8;
        co[u] = (int64_t)t * p.c_st + c * 8;
    }
    // a workgroup that lies wholly inside the segment (all but the last of a slab): no per-piece conditions
    if ((blockIdx.x * U + U) * 256u <= total && p.mode != DLM_WB_COMMITTED_ROWS) {
        const uint16_t* src = do_k ? sk : sv;
        uint16_t* dst = do_k ? ck : cv;
#pragma unroll
        for (int u = 0; u < U; ++u) kreg[u] = (p.nt & 1) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + so[u])) : *reinterpret_cast<const u32x4*>(src + so[u]);
        if (do_k && do_v) {
#pragma unroll
            for (int u = 0; u < U; ++u) vreg[u] = *reinterpret_cast<const u32x4*>(sv + so[u]);
        }
        if (p.nt & 2) {
#pragma unroll
            for (int u = 0; u < U; ++u) __builtin_nontemporal_store(kreg[u], reinterpret_cast<u32x4*>(dst + co[u]));
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) *reinterpret_cast<u32x4*>(dst + co[u]) = kreg[u];
        }
        if (do_k && do_v) {
#pragma unroll
            for (int u = 0; u < U; ++u) *reinterpret_cast<u32x4*>(cv + co[u]) = vreg[u];
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (ok[u]) {
            if (do_k) kreg[u] = *reinterpret_cast<const u32x4*>(sk + so[u]);
            if (do_v) vreg[u] = *reinterpret_cast<const u32x4*>(sv + so[u]);
        }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (ok[u]) {
            if (do_k) *reinterpret_cast<u32x4*>(ck + co[u]) = kreg[u];
            if (do_v) *reinterpret_cast<u32x4*>(cv + co[u]) = vreg[u];
        }
}

// One workgroup per sequence; every thread sums a strided slice in a fixed order, then a fixed tree.
__global__ __launch_bounds__(256) void seq_logprob_kernel(const float* zt, const float* lse, const uint8_t* mask,
                                                         int64_t mask_stride_b, const float* weight, int n_pos,
                                                         float* out, int32_t* n_terms) {
    __shared__ float ssum[4];
    __shared__ int scnt[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* z = zt + (int64_t)b * n_pos;
    const float* l = lse + (int64_t)b * n_pos;
    const uint8_t* m = mask + b * mask_stride_b;
    float acc = 0.f;
    int cnt = 0;
    for (int i = tid; i < n_pos; i += 256)
        if (m[i]) {
            acc += z[i] - l[i];
            ++cnt;
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        acc += shfl_xor(acc, off);
        cnt += shfl_xor(cnt, off);
    }
    if ((tid & 63) == 0) {
        ssum[tid >> 6] = acc;
        scnt[tid >> 6] = cnt;
    }
    __syncthreads();
    if (tid == 0) {
        const float tot = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
        out[b] = (weight ? weight[b] : 1.0f) * tot;
        if (n_terms) n_terms[b] = scnt[0] + scnt[1] + scnt[2] + scnt[3];
    }
}

static int validate_seg_copy(const dlm_kv_seg* s, int B, int Hkv, int d, const void* ck, const void* cv,
                             int64_t c_sb, int64_t c_sh, int64_t c_st, int cache_pos0) {
    if (!s) return fail(DLM_ERR_INVALID_ARG, "kv copy: null source segment");
    if (B < 0 || Hkv <= 0 || d <= 0 || s->len < 0 || cache_pos0 < 0)
        return fail(DLM_ERR_INVALID_ARG, "kv copy: negative size (B=%d Hkv=%d d=%d len=%d pos0=%d)", B, Hkv, d, s->len, cache_pos0);
    if (d % 8) return fail(DLM_ERR_UNSUPPORTED, "kv copy: d=%d is not a multiple of 8", d);
    if (s->len == 0 || B == 0) return DLM_OK;
    if (!s->k || !s->v || !ck || !cv) return fail(DLM_ERR_INVALID_ARG, "kv copy: null K/V pointer");
    if (!aligned16(s->k) || !aligned16(s->v) || !aligned16(ck) || !aligned16(cv))
        return fail(DLM_ERR_UNSUPPORTED, "kv copy: pointers must be 16-byte aligned");
    if ((s->stride_b | s->stride_h | s->stride_t | c_sb | c_sh | c_st) % 8)
        return fail(DLM_ERR_UNSUPPORTED, "kv copy: strides must be multiples of 8 elements");
    if (s->stride_t < d || c_st < d) return fail(DLM_ERR_INVALID_ARG, "kv copy: row stride smaller than d");
    return DLM_OK;
}

static int g_copy_nt = 0;       // tuning: non-temporal loads (1) / stores (2) in the copy kernel
static int g_copy_split = 1;    // 1: K and V copied by different workgroups (tuning)
static int g_copy_unroll = 1;   // 16-byte pieces per thread of kv_copy_kernel (tuning: 1, 2, 4, 8): small workgroups interleave reads and writes best

static CopyParams copy_params(const dlm_kv_seg* s, int Hkv, int d, void* ck, void* cv, int64_t c_sb, int64_t c_sh,
                              int64_t c_st, int cache_pos0, int mode, const int32_t* n_commit, const int32_t* remaining,
                              const uint8_t* commit_now, int n_pos, const int32_t* active_in) {
    CopyParams p;
    p.sk = (const uint16_t*)s->k; p.sv = (const uint16_t*)s->v;
    p.s_sb = s->stride_b; p.s_sh = s->stride_h; p.s_st = s->stride_t;
    p.ck = (uint16_t*)ck; p.cv = (uint16_t*)cv;
    p.c_sb = c_sb; p.c_sh = c_sh; p.c_st = c_st;
    p.len = s->len; p.d8 = d / 8; p.cache_pos0 = cache_pos0;
    p.mode = mode; p.n_commit = n_commit; p.remaining = remaining; p.commit_now = commit_now; p.n_pos = n_pos;
    p.active_in = active_in; p.Hkv = Hkv; p.split = 0; p.nt = 0;
    return p;
}

static int launch_kv_copy(const dlm_kv_seg* s, int B, int Hkv, int d, void* ck, void* cv, int64_t c_sb, int64_t c_sh,
                          int64_t c_st, int cache_pos0, int mode, const int32_t* n_commit, const int32_t* remaining,
                          const uint8_t* commit_now, int n_pos, hipStream_t st, const int32_t* active_in = nullptr) {
    if (s->len == 0 || B == 0) return DLM_OK;
    CopyParams p = copy_params(s, Hkv, d, ck, cv, c_sb, c_sh, c_st, cache_pos0, mode, n_commit, remaining, commit_now,
                               n_pos, active_in);
    p.split = (g_copy_split && 2 * Hkv <= 65535) ? 1 : 0;
    p.nt = p.split ? g_copy_nt : 0;
    const int64_t total = (int64_t)s->len * p.d8;
    if (total > 0x7fffffff) return fail(DLM_ERR_UNSUPPORTED, "kv copy: segment too long");
    if (Hkv > 65535 || B > 65535) return fail(DLM_ERR_UNSUPPORTED, "kv copy: B or Hkv above 65535");
    const int U = g_copy_unroll;
    const int64_t gx = (total + 256 * U - 1) / (256 * U);
    if (gx > 0x7fffffff) return fail(DLM_ERR_UNSUPPORTED, "kv copy: segment too long");
    const dim3 grid((unsigned)gx, p.split ? 2 * Hkv : Hkv, B);
    if (U == 1) hipLaunchKernelGGL(kv_copy_kernel<1>, grid, dim3(256), 0, st, p);
    else if (U == 2) hipLaunchKernelGGL(kv_copy_kernel<2>, grid, dim3(256), 0, st, p);
    else if (U == 8) hipLaunchKernelGGL(kv_copy_kernel<8>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(kv_copy_kernel<4>, grid, dim3(256), 0, st, p);
    return check_hip(hipGetLastError(), "kv_copy_kernel launch");
}

}  // namespace dlm

using namespace dlm;

extern "C" int dlm_kv_refresh(const dlm_kv_seg* src, int32_t B, int32_t Hkv, int32_t d, void* cache_k, void* cache_v,
                              int64_t c_stride_b, int64_t c_stride_h, int64_t c_stride_t, int32_t cache_pos0,
                              void* stream) {
    int rc = validate_seg_copy(src, B, Hkv, d, cache_k, cache_v, c_stride_b, c_stride_h, c_stride_t, cache_pos0);
    if (rc != DLM_OK) return rc;
    return launch_kv_copy(src, B, Hkv, d, cache_k, cache_v, c_stride_b, c_stride_h, c_stride_t, cache_pos0, 0, nullptr,
                          nullptr, nullptr, 0, (hipStream_t)stream);
}

extern "C" int dlm_seq_logprob(const float* ztarget, const float* lse, const uint8_t* mask, int64_t mask_stride_b,
                               const float* weight, int32_t B, int32_t n_pos, float* out, int32_t* n_terms,
                               void* stream) {
    if (B < 0 || n_pos < 0) return fail(DLM_ERR_INVALID_ARG, "seq_logprob: negative size");
    if (B == 0) return DLM_OK;
    if (!out) return fail(DLM_ERR_INVALID_ARG, "seq_logprob: null out");
    if (n_pos > 0 && (!ztarget || !lse || !mask)) return fail(DLM_ERR_INVALID_ARG, "seq_logprob: null ztarget/lse/mask");
    if (n_pos > 0 && mask_stride_b < n_pos) return fail(DLM_ERR_INVALID_ARG, "seq_logprob: stride < n_pos");
    hipLaunchKernelGGL(seq_logprob_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, ztarget, lse, mask, mask_stride_b,
                       weight, n_pos, out, n_terms);
    return check_hip(hipGetLastError(), "seq_logprob_kernel launch");
}

extern "C" int dlm_mask_compact(const uint8_t* mask, int64_t mask_stride_b, int32_t B, int32_t n_pos, int32_t* row_idx,
                                int32_t* m_out, void* stream) {
    if (B < 0 || n_pos < 0) return fail(DLM_ERR_INVALID_ARG, "mask_compact: negative size");
    if (!m_out) return fail(DLM_ERR_INVALID_ARG, "mask_compact: null m_out");
    if ((int64_t)B * n_pos > 0 && (!mask || !row_idx)) return fail(DLM_ERR_INVALID_ARG, "mask_compact: null pointer");
    if ((int64_t)B * n_pos > 0x7fffffff) return fail(DLM_ERR_UNSUPPORTED, "mask_compact: more than 2^31 positions");
    if (B > 0 && n_pos > 0 && mask_stride_b < n_pos) return fail(DLM_ERR_INVALID_ARG, "mask_compact: stride < n_pos");
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, mask, mask_stride_b, B, n_pos,
                       row_idx, m_out);
    return check_hip(hipGetLastError(), "compact_kernel launch");
}

extern "C" int dlm_unmask_commit(const dlm_commit_args* a, void* stream) {
    if (!a) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: null args");
    if (a->struct_size != sizeof(dlm_commit_args))
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: struct_size %u != %zu", a->struct_size, sizeof(dlm_commit_args));
    if (a->B < 0 || a->n_pos < 0) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: negative B or n_pos");
    if (a->group_len < 1 || a->group_len > 1024)
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: group_len=%d outside [1, 1024]", a->group_len);
    if (a->n_pos % a->group_len) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: n_pos %% group_len != 0");
    if (a->rule != DLM_RULE_THRESHOLD && a->rule != DLM_RULE_TOPK)
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: unknown rule %d", a->rule);
    if (a->rule == DLM_RULE_TOPK && a->k < 1) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: top-k needs k >= 1");
    if (a->rule == DLM_RULE_THRESHOLD && !(a->threshold == a->threshold))
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: threshold is NaN");
    if (a->writeback < DLM_WB_NONE || a->writeback > DLM_WB_WHILE_ACTIVE)
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: unknown writeback mode %d", a->writeback);
    const int64_t N = (int64_t)a->B * a->n_pos;
    if (N > 0x7fffffff) return fail(DLM_ERR_UNSUPPORTED, "unmask_commit: more than 2^31 positions");
    if (a->B > 0 && (!a->n_commit || !a->remaining)) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: null n_commit/remaining");
    if (N > 0) {
        if (!a->conf || !a->tok || !a->x || !a->mask) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: null conf/tok/x/mask");
        if (a->mask_stride_b < a->n_pos || a->x_stride_b < (int64_t)a->x_pos0 + a->n_pos || a->x_pos0 < 0)
            return fail(DLM_ERR_INVALID_ARG, "unmask_commit: x/mask stride too small for n_pos (+x_pos0)");
    }
    if ((a->next_row_idx == nullptr) != (a->next_m == nullptr))
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: next_row_idx and next_m go together");
    if (a->writeback != DLM_WB_NONE) {
        if (a->src_block.len <= 0) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: write-back needs a non-empty src_block");
        int rc = validate_seg_copy(&a->src_block, a->B, a->Hkv, a->d, a->cache_k, a->cache_v, a->c_stride_b,
                                   a->c_stride_h, a->c_stride_t, a->cache_pos0);
        if (rc != DLM_OK) return rc;
        if (a->writeback == DLM_WB_COMMITTED_ROWS) {
            if (a->src_block.len != a->n_pos)
                return fail(DLM_ERR_INVALID_ARG, "unmask_commit: COMMITTED_ROWS needs src_block.len == n_pos");
            if (!a->commit_now && N > 0)
                return fail(DLM_ERR_INVALID_ARG, "unmask_commit: COMMITTED_ROWS needs commit_now");
        }
        if (a->writeback == DLM_WB_WHILE_ACTIVE) {
            if (!a->active_in && a->B > 0) return fail(DLM_ERR_INVALID_ARG, "unmask_commit: WHILE_ACTIVE needs active_in");
            if (a->active_in == a->remaining || a->active_in == a->n_commit)
                return fail(DLM_ERR_INVALID_ARG, "unmask_commit: active_in must not alias remaining / n_commit");
            if ((int64_t)a->B * a->Hkv >= 0x7fffffff || (int64_t)a->src_block.len * (a->d / 8) > 0x7fffffff)
                return fail(DLM_ERR_UNSUPPORTED, "unmask_commit: B * Hkv or src_block.len * d too large");
        }
    }
    hipStream_t st = (hipStream_t)stream;
    if (a->B == 0) return DLM_OK;
    const int n_groups = a->group_len > 0 ? a->n_pos / a->group_len : 0;
    const bool fused = N > 0 && n_groups == 1 && N <= FUSED_MAX_POS;
    if (a->host_remaining_max && !a->host_remaining_total)
        return fail(DLM_ERR_INVALID_ARG, "unmask_commit: host_remaining_max goes with host_remaining_total");
    if (a->host_remaining_total && !fused)
        return fail(DLM_ERR_UNSUPPORTED, "unmask_commit: host_remaining_total needs one group per sequence and B*n_pos <= %d", FUSED_MAX_POS);
    CommitParams p;
    p.B = a->B; p.n_pos = a->n_pos; p.group_len = a->group_len; p.n_groups = n_groups;
    p.rule = a->rule; p.threshold = a->threshold; p.force_top1 = a->force_top1; p.k = a->k;
    p.conf = a->conf; p.tok = a->tok; p.x = a->x; p.x_stride_b = a->x_stride_b; p.x_pos0 = a->x_pos0;
    p.mask = a->mask; p.mask_stride_b = a->mask_stride_b; p.commit_now = a->commit_now;
    p.n_commit = a->n_commit; p.remaining = a->remaining; p.commit_step = a->commit_step; p.step = a->step;
    const bool wb_inside = fused && a->writeback == DLM_WB_WHILE_ACTIVE;   // the copy rides in the selection's launch
    if (fused) {
        CopyParams cp = {};
        unsigned grid = 1;
        if (wb_inside) {
            cp = copy_params(&a->src_block, a->Hkv, a->d, a->cache_k, a->cache_v, a->c_stride_b, a->c_stride_h, a->c_stride_t,
                             a->cache_pos0, a->writeback, a->n_commit, a->remaining, a->commit_now, a->n_pos, a->active_in);
            grid += (unsigned)(a->B * a->Hkv);
        }
        if (a->group_len <= 64) hipLaunchKernelGGL(commit_fused_kernel<1>, dim3(grid), dim3(1024), 0, st, p, a->next_row_idx, a->next_m, a->host_remaining_total, a->host_remaining_max, cp);
        else if (a->group_len <= 256) hipLaunchKernelGGL(commit_fused_kernel<4>, dim3(grid), dim3(1024), 0, st, p, a->next_row_idx, a->next_m, a->host_remaining_total, a->host_remaining_max, cp);
        else hipLaunchKernelGGL(commit_fused_kernel<16>, dim3(grid), dim3(1024), 0, st, p, a->next_row_idx, a->next_m, a->host_remaining_total, a->host_remaining_max, cp);
        int rc = check_hip(hipGetLastError(), "commit_fused_kernel launch");
        if (rc != DLM_OK) return rc;
    } else {
        if (N > 0) {
            if (n_groups != 1) {
                hipLaunchKernelGGL(zero2_i32_kernel, dim3((a->B + 255) / 256), dim3(256), 0, st, a->n_commit, a->remaining, a->B);
            }
            const int64_t waves = (int64_t)a->B * n_groups;
            const unsigned grid = (unsigned)((waves + 3) / 4);
            const unsigned lgrid = (unsigned)((waves + 255) / 256);
            const int gl = a->group_len;
            if (n_groups > 1 && (gl == 1 || gl == 2 || gl == 4 || gl == 8)) {
                if (gl == 1) hipLaunchKernelGGL(commit_lane_kernel<1>, dim3(lgrid), dim3(256), 0, st, p);
                else if (gl == 2) hipLaunchKernelGGL(commit_lane_kernel<2>, dim3(lgrid), dim3(256), 0, st, p);
                else if (gl == 4) hipLaunchKernelGGL(commit_lane_kernel<4>, dim3(lgrid), dim3(256), 0, st, p);
                else hipLaunchKernelGGL(commit_lane_kernel<8>, dim3(lgrid), dim3(256), 0, st, p);
            } else if (a->group_len <= 64) hipLaunchKernelGGL(commit_wave_kernel<1>, dim3(grid), dim3(256), 0, st, p);
            else if (a->group_len <= 256) hipLaunchKernelGGL(commit_wave_kernel<4>, dim3(grid), dim3(256), 0, st, p);
            else hipLaunchKernelGGL(commit_wave_kernel<16>, dim3(grid), dim3(256), 0, st, p);
            int rc = check_hip(hipGetLastError(), "commit_wave_kernel launch");
            if (rc != DLM_OK) return rc;
        } else {
            hipLaunchKernelGGL(zero2_i32_kernel, dim3((a->B + 255) / 256), dim3(256), 0, st, a->n_commit, a->remaining, a->B);
        }
        if (a->next_row_idx) {
            hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, st, a->mask, a->mask_stride_b, a->B, a->n_pos,
                               a->next_row_idx, a->next_m);
            int rc = check_hip(hipGetLastError(), "compact_kernel launch");
            if (rc != DLM_OK) return rc;
        }
    }
    if (a->writeback != DLM_WB_NONE && N > 0 && !wb_inside) {
        return launch_kv_copy(&a->src_block, a->B, a->Hkv, a->d, a->cache_k, a->cache_v, a->c_stride_b, a->c_stride_h,
                              a->c_stride_t, a->cache_pos0, a->writeback, a->n_commit, a->remaining, a->commit_now,
                              a->n_pos, st, a->active_in);
    }
    return DLM_OK;
}

namespace dlm {
int copy_set_unroll(int v) {
    // low digit: pieces per thread (2, 4, 8); +16: K and V by different workgroups
    const int u = v & 15;
    if ((u != 1 && u != 2 && u != 4 && u != 8) || (v & ~127)) return fail(DLM_ERR_INVALID_ARG, "set_option: kv_copy_unroll must be 1, 2, 4 or 8 (+16, +32, +64)");
    g_copy_unroll = u;
    g_copy_split = (v >> 4) & 1;
    g_copy_nt = (v >> 5) & 3;
    return DLM_OK;
}
}  // namespace dlm
