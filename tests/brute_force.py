"""Pure-Python brute-force formulations used only to pin the oracle on tiny inputs.

Deliberately a different formulation from the oracle: K/V heads are first
repeated to one per query head, the full [Lq, Lk] visibility matrix is
materialised, every sum is an exactly rounded math.fsum, and the softmax is
normalised before it multiplies V.
"""
import math
import struct


def bf16_to_float(u):
    return struct.unpack("<f", struct.pack("<I", (int(u) & 0xFFFF) << 16))[0]


def attention_brute(q, k, v, key_pos, q_pos0, mode, bs, key_ok=None, scale=None):
    """q [B][Lq][Hq][d], k/v [B][Hkv][Lk][d] nested lists of floats.
    returns O [B][Lq][Hq][d], lse [B][Hq][Lq]"""
    B, Lq, Hq, d = len(q), len(q[0]), len(q[0][0]), len(q[0][0][0])
    Hkv, Lk = len(k[0]), len(k[0][0])
    g = Hq // Hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    # repeat kv heads
    kk = [[k[b][h // g] for h in range(Hq)] for b in range(B)]
    vv = [[v[b][h // g] for h in range(Hq)] for b in range(B)]
    vis = [[[(key_ok is None or key_ok[b][j]) and
             (mode == "full" or (key_pos[j] // bs) <= ((q_pos0 + i) // bs))
             for j in range(Lk)] for i in range(Lq)] for b in range(B)]
    O = [[[[0.0] * d for _ in range(Hq)] for _ in range(Lq)] for _ in range(B)]
    lse = [[[-math.inf] * Lq for _ in range(Hq)] for _ in range(B)]
    for b in range(B):
        for h in range(Hq):
            for i in range(Lq):
                js = [j for j in range(Lk) if vis[b][i][j]]
                if not js:
                    continue
                s = [scale * math.fsum(q[b][i][h][c] * kk[b][h][j][c] for c in range(d)) for j in js]
                m = max(s)
                e = [math.exp(x - m) for x in s]
                z = math.fsum(e)
                p = [x / z for x in e]
                for c in range(d):
                    O[b][i][h][c] = math.fsum(p[n] * vv[b][h][j][c] for n, j in enumerate(js))
                lse[b][h][i] = m + math.log(z)
    return O, lse


def lmhead_brute(h, w, inv_t=1.0, forbid=-1):
    """h [Dh], w [V][Dh] floats -> (conf, tok, lse, zmax, z2nd) by direct softmax."""
    V = len(w)
    z = [math.fsum(h[c] * w[v][c] for c in range(len(h))) * inv_t for v in range(V)]
    if forbid >= 0:
        z[forbid] = -math.inf
    zmax = max(z)
    tok = z.index(zmax)
    den = math.fsum(math.exp(x - zmax) for x in z)
    probs = [math.exp(x - zmax) / den for x in z]
    rest = [x for i, x in enumerate(z) if i != tok]
    return probs[tok], tok, zmax + math.log(den), zmax, (max(rest) if rest else -math.inf)


def select_brute(conf, mask, rule, tau, k, force_top1=True):
    """One commit group; enumeration over subsets is overkill, so: direct set definitions."""
    cand = [i for i, m in enumerate(mask) if m]
    if not cand:
        return set()
    if rule == "threshold":
        c = {i for i in cand if conf[i] >= tau}
        if force_top1:
            top = max(conf[i] for i in cand)
            c.add(min(i for i in cand if conf[i] == top))
        return c
    kk = min(k, len(cand))
    chosen = set()
    pool = list(cand)
    for _ in range(kk):
        top = max(conf[i] for i in pool)
        j = min(i for i in pool if conf[i] == top)
        chosen.add(j)
        pool.remove(j)
    return chosen
