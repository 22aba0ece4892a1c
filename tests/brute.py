"""A second, independent statement of the layer in pure Python loops, used to
pin the C oracle on tiny cases.  Written from the set equations of the paper's
re-routing section (primary set, most-similar primary, re-routing condition,
final set) and the MoE preliminaries of its appendix; it shares nothing with
the C oracle and is far too slow for anything but toy sizes."""
import math


def widen(bits_or_float, dtype):
    import struct
    if dtype == 0:
        return float(bits_or_float)
    return struct.unpack("<f", struct.pack("<I", int(bits_or_float) << 16))[0]


def top_k(logits_row, K):
    order = sorted(range(len(logits_row)), key=lambda e: (-logits_row[e], e))
    sel = order[:K]
    m = logits_row[sel[0]]
    ex = [math.exp(logits_row[e] - m) for e in sel]
    z = sum(ex)
    return sel, [v / z for v in ex]


def reroute(ids, sim, S, rho):
    """ids: list of K-lists.  Returns (ids', primary set, final set)."""
    primary = set()
    for row in ids:
        primary.update(row[:S])
    activated = set(e for row in ids for e in row)
    mapping = {}
    final = set(primary)
    for u in sorted(activated - primary):
        best_v, best_s = None, None
        for v in sorted(primary):
            if best_s is None or sim[u][v] > best_s:
                best_v, best_s = v, sim[u][v]
        if rho > 0 and best_s < rho:
            final.add(u)            # critical expert stays
        else:
            mapping[u] = best_v
    out = [[e if k < S else mapping.get(e, e) for k, e in enumerate(row)] for row in ids]
    return out, primary, final


def silu(z):
    return z / (1.0 + math.exp(-z))


def expert(x, gate_up, down, dm):
    dh = len(x)
    h = []
    for j in range(dm):
        g = sum(gate_up[j][i] * x[i] for i in range(dh))
        u = sum(gate_up[dm + j][i] * x[i] for i in range(dh))
        h.append(silu(g) * u)
    return [sum(down[r][j] * h[j] for j in range(dm)) for r in range(dh)]


def layer(x, router, gate_up, down, K, sim, S, rho, shared=None):
    """x [T][dh], router [M][dh], gate_up [M][2dm][dh], down [M][dh][dm], all
    Python floats.  Returns (ids, weights, ids', out_base, out_sere)."""
    T, dh = len(x), len(x[0])
    M = len(router)
    dm = len(down[0][0])
    ids, wts = [], []
    for t in range(T):
        logits = [sum(x[t][i] * router[e][i] for i in range(dh)) for e in range(M)]
        sel, w = top_k(logits, K)
        ids.append(sel)
        wts.append(w)
    new_ids, _, _ = reroute(ids, sim, S, rho)

    def run(mapping):
        out = []
        for t in range(T):
            acc = [0.0] * dh
            for k in range(K):
                y = expert(x[t], gate_up[mapping[t][k]], down[mapping[t][k]], dm)
                acc = [a + wts[t][k] * v for a, v in zip(acc, y)]
            for sh in shared or []:
                y = expert(x[t], sh[0], sh[1], dm)
                acc = [a + v for a, v in zip(acc, y)]
            out.append(acc)
        return out

    return ids, wts, new_ids, run(ids), run(new_ids)
