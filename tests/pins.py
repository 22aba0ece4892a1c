"""Pins for the CPU oracle: each check compares one oracle routine with
something fixed by the paper or by mathematics (a closed form, a library
routine on a special case, an invariant, a brute-force second implementation),
never with the oracle itself.  Every check takes the oracle object ``o`` so the
same checks can be pointed at deliberately broken builds of the oracle
(tests/test_oracle_mutants.py) to show that each plausible mistake is caught.
"""
import itertools
import json
import math
import os

import numpy as np

from paper_2602_07616_amd import workloads as wk
from . import brute

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rng_case(seed, dtype, T, dh, M, dm, n_sh=0):
    """Small random layer in storage format (values from the shared generator)."""
    def draw(tag, shape, scale):
        n = int(np.prod(shape))
        return wk.to_storage(np.float32(scale) * wk.std_normal(seed, tag, n), dtype).reshape(shape)
    case = dict(
        hidden=draw("x", (T, dh), 1.0), router_w=draw("r", (M, dh), 0.3),
        w_gate_up=draw("gu", (M, 2 * dm, dh), 0.3), w_down=draw("dn", (M, dh, dm), 0.3),
        shared_gate_up=None, shared_down=None)
    if n_sh:
        case["shared_gate_up"] = draw("sgu", (n_sh, 2 * dm, dh), 0.3)
        case["shared_down"] = draw("sdn", (n_sh, dh, dm), 0.3)
    return case


def rand_sim(seed, M, levels=0, symmetric=True):
    """Random similarity matrix in [0,1]; ``levels`` > 0 quantises it to force ties."""
    u = (wk.raw_bits(seed, "sim", 0, M * M) >> np.uint64(11)).astype(np.float64) / float(1 << 53)
    s = u.reshape(M, M)
    if symmetric:
        s = np.triu(s, 1)
        s = s + s.T
    if levels:
        s = np.floor(s * levels) / levels
    np.fill_diagonal(s, 1.0)
    return s.astype(np.float32)


def rand_ids(seed, T, K, M):
    """T rows of K distinct experts, in random order."""
    keys = (wk.raw_bits(seed, "ids", 0, T * M) >> np.uint64(11)).reshape(T, M)
    return np.argsort(keys, axis=1, kind="stable")[:, :K].astype(np.int32)


def f64(a, dtype):
    return wk.storage_to_f64(a, dtype)


def np_silu(z):
    return z / (1.0 + np.exp(-z))


def np_expert(x, gu, dn):
    """E(x) with library matmuls; x [n,dh], gu [2dm,dh], dn [dh,dm] (float64)."""
    dm = dn.shape[1]
    g = x @ gu[:dm].T
    u = x @ gu[dm:].T
    return (np_silu(g) * u) @ dn.T


# ---------------------------------------------------------------- router ---
def pin_router_logits_library(o):
    for dtype, seed in ((wk.F32, 11), (wk.BF16, 12)):
        c = rng_case(seed, dtype, 5, 96, 7, 4)
        got = o.router_logits(c["hidden"], c["router_w"], dtype)
        want = f64(c["hidden"], dtype) @ f64(c["router_w"], dtype).T
        assert got.shape == want.shape
        assert np.allclose(got, want, rtol=0, atol=1e-12), np.abs(got - want).max()
    # a non-square, hand-checkable case: logit[t][e] = <x_t, r_e>
    x = np.array([[1, 2, 3], [0, -1, 4]], dtype=np.float32)
    r = np.array([[1, 0, 0], [0, 1, 0], [1, 1, 1], [2, -1, 0.5]], dtype=np.float32)
    got = o.router_logits(x, r, wk.F32)
    assert np.array_equal(got, np.array([[1, 2, 6, 1.5], [0, -1, 3, 3]], dtype=np.float64))


def pin_topk_order_and_gate(o):
    # hand case with a tie: equal logits -> lower index first
    logits = np.array([[0.5, 2.0, 2.0, -1.0, 1.0],
                       [3.0, 3.0, 3.0, 3.0, 3.0]])
    ids, w, gap = o.topk_gate(logits, 3)
    assert ids.tolist() == [[1, 2, 4], [0, 1, 2]]
    e = math.exp(-1.0)
    assert np.allclose(w[0], [1 / (2 + e), 1 / (2 + e), e / (2 + e)], atol=1e-15)
    assert np.allclose(w[1], [1 / 3] * 3, atol=1e-15)
    assert gap == 0.0
    # random: against a stable library sort and scipy's softmax
    from scipy.special import softmax
    lg = wk.std_normal(21, "lg", 40 * 33).astype(np.float64).reshape(40, 33)
    lg[:, 5] = lg[:, 17]                      # planted exact ties
    for K in (1, 4, 33):
        ids, w, gap = o.topk_gate(lg, K)
        want = np.argsort(-lg, axis=1, kind="stable")[:, :K]
        assert np.array_equal(ids, want)
        assert np.allclose(w, softmax(np.take_along_axis(lg, want, 1), axis=1), atol=1e-15)
        assert np.allclose(w.sum(1), 1.0, atol=1e-14)
        assert np.all(np.diff(w, axis=1) <= 0)
        srt = -np.sort(-lg, axis=1)
        want_gap = np.min(srt[:, :min(K, 32)] - srt[:, 1:min(K, 32) + 1])
        assert gap == want_gap, (gap, want_gap)
    # K == M: min_gap covers only ranks inside the row
    _, _, gap = o.topk_gate(np.array([[1.0, 4.0, 2.0]]), 3)
    assert gap == 1.0


# --------------------------------------------------------------- re-route ---
def _fig2():
    with open(os.path.join(GOLDEN, "fig2_behaviour.json")) as f:
        return json.load(f)


def pin_fig2_behaviour(o):
    g = _fig2()
    ids = np.array(g["topk_ids"], dtype=np.int32)
    sim = np.array(g["sim"], dtype=np.float32)
    H = o.primary_mask(ids, g["S"], 4)
    assert np.flatnonzero(H).tolist() == g["expect_primary"]
    out, final, target, star = o.reroute_sets(ids, sim, g["S"], g["rho"])
    assert out.tolist() == g["expect_rerouted_ids"]
    assert np.flatnonzero(final).tolist() == g["expect_final_set"]
    assert target.tolist() == [-1, 0, 3, -1]
    assert np.allclose(star, [0, 0.9, 0.2, 0])
    assert o.reroute_per_slot(ids, sim, g["S"], g["rho"]).tolist() == g["expect_rerouted_ids"]


def pin_reroute_hand_cases(o):
    for fn in (o.reroute_per_slot, lambda *a: o.reroute_sets(*a)[0]):
        # one token, K=3, S=1, rho=0: both secondaries collapse onto the only primary
        ids = np.array([[2, 0, 3]], dtype=np.int32)
        sim = rand_sim(3, 4)
        assert fn(ids, sim, 1, 0.0).tolist() == [[2, 2, 2]]
        # S == K: identity
        assert fn(ids, sim, 3, 0.0).tolist() == ids.tolist()
        # rho above every off-diagonal similarity: identity (the original model)
        assert fn(ids, sim, 1, 1.5).tolist() == ids.tolist()
        # constant similarity: the lowest-index primary wins the tie
        ids = np.array([[3, 0], [1, 2], [4, 5]], dtype=np.int32)
        const = np.full((6, 6), 0.25, dtype=np.float32)
        assert fn(ids, const, 1, 0.0).tolist() == [[3, 1], [1, 1], [4, 1]]
        # boundary: sim* == rho re-routes, just below keeps
        assert fn(ids, const, 1, 0.25).tolist() == [[3, 1], [1, 1], [4, 1]]
        assert fn(ids, const, 1, np.nextafter(np.float32(0.25), np.float32(1))).tolist() == ids.tolist()
        # a secondary that is primary for another token is never re-routed
        ids = np.array([[0, 1], [1, 2]], dtype=np.int32)
        sim = np.array([[1, .1, .9], [.1, 1, .2], [.9, .2, 1]], dtype=np.float32)
        assert fn(ids, sim, 1, 0.0).tolist() == [[0, 1], [1, 0]]
        # ... and the diagonal is never consulted (here it is the row minimum)
        np.fill_diagonal(sim, 0.0)
        assert fn(ids, sim, 1, 0.0).tolist() == [[0, 1], [1, 0]]
        # asymmetric matrix: the ROW is the secondary expert
        ids = np.array([[0, 2], [1, 2]], dtype=np.int32)
        sim = np.array([[1, 0, 0], [0, 1, 0], [0.2, 0.7, 1]], dtype=np.float32)
        assert fn(ids, sim, 1, 0.0).tolist() == [[0, 1], [1, 1]]
        sim = np.array([[1, 0, 0.2], [0, 1, 0.7], [0.6, 0.1, 1]], dtype=np.float32)
        assert fn(ids, sim, 1, 0.0).tolist() == [[0, 0], [1, 0]]
        # negative rho behaves like rho = 0 (threshold test disabled)
        assert fn(ids, sim, 1, -1.0).tolist() == [[0, 0], [1, 0]]
        # M == K: every expert active in every token; with S=1 and rho=0 all
        # secondaries move onto primaries
        ids = np.array([[0, 1, 2], [0, 2, 1]], dtype=np.int32)
        sim = np.array([[1, .3, .4], [.3, 1, .5], [.4, .5, 1]], dtype=np.float32)
        assert fn(ids, sim, 1, 0.0).tolist() == [[0, 0, 0], [0, 0, 0]]
        assert fn(ids, sim, 2, 0.0).tolist() == ids.tolist()
        # all tokens identical: primary set = the shared top-S
        ids = np.array([[5, 1, 7, 2]] * 3, dtype=np.int32)
        sim = rand_sim(9, 8)
        out = fn(ids, sim, 2, 0.0)
        assert set(out.ravel().tolist()) == {5, 1}
        assert out[:, :2].tolist() == [[5, 1]] * 3


def pin_reroute_against_brute(o, cases=1200):
    for c in range(cases):
        M = 2 + c % 7
        K = 1 + (c // 7) % min(3, M)
        T = 1 + (c // 21) % 6
        S = 1 + (c // 5) % K
        rho = [0.0, 0.3, 0.5, 0.75, 1.0, -0.5][c % 6]
        ids = rand_ids(1000 + c, T, K, M)
        sim = rand_sim(2000 + c, M, levels=4 if c % 2 else 0, symmetric=bool(c % 3))
        want, primary, final = brute.reroute(ids.tolist(), sim.tolist(), S, rho)
        got_slot = o.reroute_per_slot(ids, sim, S, rho)
        got_set, final_set, _, _ = o.reroute_sets(ids, sim, S, rho)
        assert got_slot.tolist() == want, (c, ids, sim, S, rho)
        assert got_set.tolist() == want, (c, ids, sim, S, rho)
        assert np.flatnonzero(final_set).tolist() == sorted(final), c
        assert np.flatnonzero(o.primary_mask(ids, S, M)).tolist() == sorted(primary), c
        # the final set is exactly the set of experts the new map uses
        assert sorted(set(got_set.ravel().tolist())) == sorted(final), c


def check_reroute_invariants(ids, new_ids, sim, S, rho, H, final_set, cnt_b, cnt_a):
    """Properties of Sec. 3.2.2 that hold for any input (also used on GPU output)."""
    T, K = ids.shape
    M = sim.shape[0]
    assert np.array_equal(new_ids[:, :S], ids[:, :S])          # primaries untouched
    assert cnt_a.sum() == cnt_b.sum() == T * K
    active_b, active_a = cnt_b > 0, cnt_a > 0
    assert np.all(active_b[active_a])                           # no new expert appears
    assert active_a.sum() <= active_b.sum()
    assert np.all(active_a[H.astype(bool)])                     # primaries stay active
    assert np.array_equal(active_a.astype(np.int32), final_set)
    prim = np.flatnonzero(H)
    for t in range(T):
        for k in range(S, K):
            u, v = int(ids[t, k]), int(new_ids[t, k])
            if v != u:
                assert H[v] == 1 and not H[u]
                row = sim[u, prim]
                assert sim[u, v] == row.max()
                assert v == prim[np.argmax(row)]                # first maximum
                assert rho <= 0 or sim[u, v] >= np.float32(rho)
            elif not H[u]:
                assert rho > 0 and sim[u, prim].max() < np.float32(rho)   # critical expert
    for u in range(M):
        if active_b[u] and not H[u] and rho > 0 and sim[u, prim].max() < np.float32(rho):
            assert cnt_a[u] == cnt_b[u]
        if H[u]:
            assert cnt_a[u] >= cnt_b[u]
    if rho <= 0:
        assert np.array_equal(final_set, H)
        assert np.all(H[new_ids.ravel()] == 1)


def pin_reroute_invariants(o):
    for c in range(200):
        M, K, T = 6 + c % 20, 2 + c % 4, 1 + c % 17
        ids = rand_ids(300 + c, T, K, M)
        sim = rand_sim(400 + c, M, levels=8 if c % 2 else 0, symmetric=bool(c % 3))
        prev_after = None
        for S in range(1, K + 1):
            last = None
            for rho in (0.0, 0.2, 0.5, 0.8, 1.1):
                new_ids, final_set, _, _ = o.reroute_sets(ids, sim, S, rho)
                H = o.primary_mask(ids, S, M)
                cnt_b = o.compact(ids, M)[0]
                cnt_a = o.compact(new_ids, M)[0]
                check_reroute_invariants(ids, new_ids, sim, S, rho, H, final_set, cnt_b, cnt_a)
                n_after = int((cnt_a > 0).sum())
                assert last is None or n_after >= last          # non-decreasing in rho
                last = n_after
            H_S = o.primary_mask(ids, S, M)
            if prev_after is not None:
                assert np.all(H_S[prev_after.astype(bool)] == 1)   # E_p(S-1) within E_p(S)
            prev_after = H_S


# ------------------------------------------------------------- compaction ---
def pin_compact(o):
    ids = np.array([[2, 0], [0, 2], [3, 0]], dtype=np.int32)
    cnt, offs, tok, slot, n = o.compact(ids, 5)
    assert cnt.tolist() == [3, 0, 2, 1, 0] and offs.tolist() == [0, 3, 3, 5, 6, 6] and n == 3
    assert tok.tolist() == [0, 1, 2, 0, 1, 2] and slot.tolist() == [1, 0, 1, 0, 1, 0]
    # duplicates inside a token (possible after re-routing) are separate slots
    cnt, offs, tok, slot, n = o.compact(np.array([[1, 1, 0]], dtype=np.int32), 2)
    assert cnt.tolist() == [1, 2] and tok.tolist() == [0, 0, 0] and slot.tolist() == [2, 0, 1]
    for c in range(50):
        T, K, M = 1 + c % 9, 1 + c % 5, 5 + c % 11
        ids = rand_ids(700 + c, T, K, M)
        if c % 2:
            ids[:, -1] = ids[:, 0]
        cnt, offs, tok, slot, n = o.compact(ids, M)
        flat = ids.ravel()
        order = np.argsort(flat, kind="stable")
        assert np.array_equal(tok, order // K) and np.array_equal(slot, order % K)
        assert np.array_equal(cnt, np.bincount(flat, minlength=M))
        assert np.array_equal(offs, np.concatenate([[0], np.cumsum(cnt)]))
        assert n == len(set(flat.tolist()))


# ------------------------------------------------------------ expert / layer ---
def pin_expert_closed_form(o):
    # x=[1,2]; gate=I, up=[[1,1],[1,-1]], down=I  ->  y = [3*silu(1), -silu(2)]
    x = np.array([1, 2], dtype=np.float32)
    gu = np.array([[1, 0], [0, 1], [1, 1], [1, -1]], dtype=np.float32)
    dn = np.array([[1, 0], [0, 1]], dtype=np.float32)
    y = o.expert_ffn(x, gu, dn, wk.F32)
    s1, s2 = 1 / (1 + math.exp(-1)), 2 / (1 + math.exp(-2))
    assert np.allclose(y, [3 * s1, -s2], atol=1e-15)
    # rectangular (dm != dh), asymmetric down: y = down @ h
    gu = np.array([[1, 0], [0, 0], [2, 0], [5, 5]], dtype=np.float32)     # g=[1,0], u=[2,15]
    dn = np.array([[1, 10], [-2, 4]], dtype=np.float32)
    y = o.expert_ffn(x, gu, dn, wk.F32)
    assert np.allclose(y, [2 * s1, -4 * s1], atol=1e-15)                 # silu(0)*15 = 0
    dn3 = np.array([[1, 0, 2], [0, 1, 0]], dtype=np.float32)             # dh=2, dm=3
    gu3 = np.array([[1, 0], [0, 1], [1, 1], [1, 0], [0, 1], [1, 1]], dtype=np.float32)
    y = o.expert_ffn(x, gu3, dn3, wk.F32)
    s3 = 3 / (1 + math.exp(-3))
    assert np.allclose(y, [1 * s1 + 2 * (3 * s3), 2 * s2], atol=1e-14)
    # bf16 storage widens exactly: 1.0078125 = 0x3F81
    xb = np.array([0x3F81, 0x4000], dtype=np.uint16)
    gub = wk.f32_to_bf16_bits(np.array([[1, 0], [0, 1], [1, 0], [0, 1]], dtype=np.float32))
    dnb = wk.f32_to_bf16_bits(np.array([[1, 0], [0, 1]], dtype=np.float32))
    y = o.expert_ffn(xb, gub, dnb, wk.BF16)
    a = 1.0078125
    assert np.allclose(y, [a * a / (1 + math.exp(-a)), 4 / (1 + math.exp(-2))], atol=1e-15)
    # random, against library matmuls
    for dtype, seed in ((wk.F32, 31), (wk.BF16, 32)):
        c = rng_case(seed, dtype, 1, 40, 2, 24)
        y = o.expert_ffn(c["hidden"][0], c["w_gate_up"][1], c["w_down"][1], dtype)
        want = np_expert(f64(c["hidden"], dtype), f64(c["w_gate_up"][1], dtype),
                         f64(c["w_down"][1], dtype))[0]
        assert np.allclose(y, want, rtol=1e-12, atol=1e-13)


def dense_layer(c, dtype, ids, w):
    """Layer output as the dense sum over ALL experts with P zero off the
    selected slots, by library matmuls (the textbook top-k MoE)."""
    x = f64(c["hidden"], dtype)
    T = x.shape[0]
    M = c["w_gate_up"].shape[0]
    P = np.zeros((T, M))
    for t in range(T):
        for k in range(ids.shape[1]):
            P[t, ids[t, k]] += w[t, k]
    out = np.zeros_like(x)
    for e in range(M):
        out += P[:, e:e + 1] * np_expert(x, f64(c["w_gate_up"][e], dtype), f64(c["w_down"][e], dtype))
    if c["shared_gate_up"] is not None:
        for s in range(c["shared_gate_up"].shape[0]):
            out += np_expert(x, f64(c["shared_gate_up"][s], dtype), f64(c["shared_down"][s], dtype))
    return out


def pin_layer_dense_formulation(o):
    for dtype, seed, n_sh in ((wk.F32, 41, 0), (wk.BF16, 42, 2)):
        c = rng_case(seed, dtype, 6, 48, 9, 20, n_sh)
        sim = rand_sim(seed, 9)
        r = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], c["shared_gate_up"],
                    c["shared_down"], dtype, 3, sim, 1, 0.3)
        lg = f64(c["hidden"], dtype) @ f64(c["router_w"], dtype).T
        want_ids = np.argsort(-lg, axis=1, kind="stable")[:, :3]
        assert np.array_equal(r.topk_ids, want_ids)
        assert np.allclose(r.out_base, dense_layer(c, dtype, r.topk_ids, r.topk_weights),
                           rtol=1e-11, atol=1e-12)
        assert not np.array_equal(r.rerouted_ids, r.topk_ids)
        assert np.allclose(r.out_sere, dense_layer(c, dtype, r.rerouted_ids, r.topk_weights),
                           rtol=1e-11, atol=1e-12)


def pin_shared_experts_closed_form(o):
    """Two shared experts of width dm equal ONE expert of width 2*dm whose
    gate/up rows and down columns are the concatenation (SwiGLU separates over
    intermediate columns)."""
    dtype = wk.BF16
    c = rng_case(51, dtype, 4, 32, 5, 8, 2)
    sim = rand_sim(51, 5)
    r = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], c["shared_gate_up"],
                c["shared_down"], dtype, 2, sim, 1, 0.0)
    no_sh = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], None, None,
                    dtype, 2, sim, 1, 0.0)
    sg, sd = c["shared_gate_up"], c["shared_down"]
    wide_gu = np.concatenate([sg[0][:8], sg[1][:8], sg[0][8:], sg[1][8:]], axis=0)
    wide_dn = np.concatenate([sd[0], sd[1]], axis=1)
    for t in range(4):
        wide = o.expert_ffn(c["hidden"][t], np.ascontiguousarray(wide_gu),
                            np.ascontiguousarray(wide_dn), dtype)
        assert np.allclose(r.out_base[t] - no_sh.out_base[t], wide, rtol=1e-10, atol=1e-12)
        assert np.allclose(r.out_sere[t] - no_sh.out_sere[t], wide, rtol=1e-10, atol=1e-12)


def pin_layer_against_brute(o):
    for dtype, seed in ((wk.F32, 61), (wk.BF16, 62)):
        c = rng_case(seed, dtype, 3, 6, 5, 4, 1)
        sim = rand_sim(seed, 5, levels=4)
        r = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], c["shared_gate_up"],
                    c["shared_down"], dtype, 3, sim, 1, 0.25)
        tl = lambda a: f64(a, dtype).tolist()
        shared = [(tl(c["shared_gate_up"][0]), tl(c["shared_down"][0]))]
        ids, wts, new_ids, base, sere = brute.layer(
            tl(c["hidden"]), tl(c["router_w"]), tl(c["w_gate_up"]), tl(c["w_down"]), 3,
            sim.tolist(), 1, 0.25, shared)
        assert r.topk_ids.tolist() == ids and r.rerouted_ids.tolist() == new_ids
        assert np.allclose(r.topk_weights, wts, atol=1e-15)
        assert np.allclose(r.out_base, base, rtol=1e-12, atol=1e-13)
        assert np.allclose(r.out_sere, sere, rtol=1e-12, atol=1e-13)


def pin_disabled_reroute_is_standard_moe(o):
    c = rng_case(71, wk.BF16, 7, 32, 8, 8)
    sim = rand_sim(71, 8) * np.float32(0.99)
    np.fill_diagonal(sim, 1.0)
    kw = dict(hidden=c["hidden"], router_w=c["router_w"], w_gate_up=c["w_gate_up"],
              w_down=c["w_down"], shared_gate_up=None, shared_down=None, dtype=wk.BF16, K=3, sim=sim)
    a = o.layer(S=3, rho=0.0, **kw)          # S == K
    b = o.layer(S=1, rho=1.0, **kw)          # rho = 1: the original model
    for r in (a, b):
        assert np.array_equal(r.rerouted_ids, r.topk_ids)
        assert np.array_equal(r.out_sere, r.out_base)
        assert r.n_active_after == r.n_active_before


def pin_substitution_identity(o):
    """Layer-output difference of one substituted expert = w_a (E_a(z) - E~_a(z))
    (first equation of the substitution-error proof), summed over changed slots."""
    dtype = wk.BF16
    c = rng_case(81, dtype, 6, 40, 10, 12)
    sim = rand_sim(81, 10)
    r = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], None, None, dtype,
                4, sim, 1, 0.0)
    changed = 0
    for t in range(6):
        d = np.zeros(40)
        for k in range(4):
            a, b = r.topk_ids[t, k], r.rerouted_ids[t, k]
            if a != b:
                changed += 1
                ea = o.expert_ffn(c["hidden"][t], c["w_gate_up"][a], c["w_down"][a], dtype)
                eb = o.expert_ffn(c["hidden"][t], c["w_gate_up"][b], c["w_down"][b], dtype)
                d += r.topk_weights[t, k] * (eb - ea)
        assert np.allclose(r.out_sere[t] - r.out_base[t], d, rtol=1e-9, atol=1e-13)
    assert changed > 0
    # gate weights are the router's, untouched by re-routing: they sum to 1
    assert np.allclose(r.topk_weights.sum(1), 1.0, atol=1e-14)


def pin_exact_twins(o):
    """Experts 4-7 are bit-exact copies of 0-3 and only twin pairs are similar:
    every re-route lands on an identical function, so the output cannot move."""
    dtype = wk.F32
    c = rng_case(91, dtype, 8, 24, 8, 6)
    c["w_gate_up"][4:] = c["w_gate_up"][:4]
    c["w_down"][4:] = c["w_down"][:4]
    sim = np.zeros((8, 8), dtype=np.float32)
    np.fill_diagonal(sim, 1.0)
    for i in range(4):
        sim[i, i + 4] = sim[i + 4, i] = 1.0
    r = o.layer(c["hidden"], c["router_w"], c["w_gate_up"], c["w_down"], None, None, dtype,
                3, sim, 1, 0.5)
    assert not np.array_equal(r.rerouted_ids, r.topk_ids)
    assert np.allclose(r.out_sere, r.out_base, rtol=0, atol=1e-15)
    assert r.n_active_after < r.n_active_before


# --------------------------------------------------------------- similarity ---
def np_similarity(calib, gu, dn, dtype):
    N = calib.shape[0]
    M = gu.shape[0]
    S = np.zeros((M, M))
    for b in range(N):
        acts = [np_expert(f64(calib[b], dtype), f64(gu[e], dtype), f64(dn[e], dtype))
                for e in range(M)]
        D = np.array([[np.linalg.norm(acts[p] - acts[q]) for q in range(M)] for p in range(M)])
        S += 1.0 - D / D.max()
    return S / N


def pin_similarity(o):
    # two experts: the only pair is the farthest pair -> off-diagonal 0, diagonal 1
    c = rng_case(101, wk.F32, 1, 16, 2, 4)
    cal = wk.std_normal(101, "cal", 2 * 3 * 16).reshape(2, 3, 16)
    s = o.similarity_frobenius(cal, c["w_gate_up"], c["w_down"], wk.F32)
    assert np.allclose(s, np.eye(2), atol=1e-15)
    for dtype, seed in ((wk.F32, 102), (wk.BF16, 103)):
        c = rng_case(seed, dtype, 1, 24, 6, 10)
        c["w_gate_up"][5] = c["w_gate_up"][2]
        c["w_down"][5] = c["w_down"][2]                       # exact twin of expert 2
        cal = wk.to_storage(wk.std_normal(seed, "cal", 3 * 5 * 24), dtype).reshape(3, 5, 24)
        s = o.similarity_frobenius(cal, c["w_gate_up"], c["w_down"], dtype)
        want = np_similarity(cal, c["w_gate_up"], c["w_down"], dtype)
        assert np.allclose(s, want, rtol=1e-11, atol=1e-13)
        assert np.array_equal(s, s.T)
        assert np.allclose(np.diag(s), 1.0, atol=1e-15)
        assert s.min() >= 0.0 and s.max() <= 1.0 + 1e-15
        assert abs(s[2, 5] - 1.0) < 1e-15
    # single batch: the farthest pair scores exactly 0
    c = rng_case(104, wk.F32, 1, 16, 4, 4)
    cal = wk.std_normal(104, "cal", 4 * 16).reshape(1, 4, 16)
    s = o.similarity_frobenius(cal, c["w_gate_up"], c["w_down"], wk.F32)
    assert s.min() == 0.0


def pin_similarity_cosine(o):
    """Cosine metric: numpy formulation with library norms; closed-form cases."""
    for dtype, seed in ((wk.F32, 111), (wk.BF16, 112)):
        c = rng_case(seed, dtype, 1, 24, 6, 10)
        c["w_gate_up"][5] = c["w_gate_up"][2]
        c["w_down"][5] = c["w_down"][2]                       # exact twin of expert 2
        if dtype == wk.F32:
            c["w_gate_up"][4] = c["w_gate_up"][1]
            c["w_down"][4] = np.float32(-2.0) * c["w_down"][1]   # expert 4 = -2 x expert 1: cosine -1
            c["w_gate_up"][3] = c["w_gate_up"][0]
            c["w_down"][3] = np.float32(0.5) * c["w_down"][0]    # expert 3 = expert 0 / 2: cosine +1
        cal = wk.to_storage(wk.std_normal(seed, "cal", 3 * 5 * 24), dtype).reshape(3, 5, 24)
        s = o.similarity_cosine(cal, c["w_gate_up"], c["w_down"], dtype)
        N, M = cal.shape[0], c["w_gate_up"].shape[0]
        want = np.zeros((M, M))
        for b in range(N):
            acts = [np_expert(f64(cal[b], dtype), f64(c["w_gate_up"][e], dtype), f64(c["w_down"][e], dtype))
                    for e in range(M)]
            unit = [a / np.linalg.norm(a, axis=1, keepdims=True) for a in acts]
            want += np.array([[np.mean(np.sum(unit[p] * unit[q], axis=1)) for q in range(M)] for p in range(M)])
        want /= N
        assert np.allclose(s, want, rtol=1e-11, atol=1e-13)
        assert np.allclose(s, s.T, rtol=0, atol=1e-15)
        assert np.allclose(np.diag(s), 1.0, atol=1e-14)
        assert s.min() >= -1.0 - 1e-14 and s.max() <= 1.0 + 1e-14
        assert abs(s[2, 5] - 1.0) < 1e-14
        if dtype == wk.F32:
            assert abs(s[1, 4] + 1.0) < 1e-12 and abs(s[0, 3] - 1.0) < 1e-12   # scale-invariant, sign-aware
            fro = o.similarity_frobenius(cal, c["w_gate_up"], c["w_down"], dtype)
            assert fro[0, 3] < 1.0 - 1e-3           # the Frobenius metric is NOT scale-invariant: a different quantity
    # a zero output vector contributes 0: expert 1 with zero down weights
    c = rng_case(113, wk.F32, 1, 16, 3, 4)
    c["w_down"][1] = 0
    cal = wk.std_normal(113, "cal", 2 * 4 * 16).reshape(2, 4, 16)
    s = o.similarity_cosine(cal, c["w_gate_up"], c["w_down"], wk.F32)
    assert np.all(s[1] == 0.0) and np.all(s[:, 1] == 0.0) and abs(s[0, 0] - 1.0) < 1e-14


def _hsic_ustatistic(K, L):
    """Unbiased HSIC as the U-statistic it is defined as (Song et al. 2012): the mean, over all
    ordered 4-tuples (s, t, u, v) of distinct indices, of K_st (L_st + L_uv - 2 L_su).  O(n^4)."""
    n = K.shape[0]
    total, count = 0.0, 0
    for s_, t_, u_, v_ in itertools.permutations(range(n), 4):
        total += K[s_, t_] * (L[s_, t_] + L[u_, v_] - 2.0 * L[s_, u_])
        count += 1
    return total / count


def pin_similarity_cka(o):
    """Linear CKA with the unbiased HSIC estimator: brute force over 4-tuples on tiny batches, the
    invariances the appendix states (isotropic scaling, orthogonal transformations), twins."""
    for dtype, seed in ((wk.F32, 121), (wk.BF16, 122)):
        c = rng_case(seed, dtype, 1, 24, 5, 10)
        c["w_gate_up"][4] = c["w_gate_up"][2]
        c["w_down"][4] = c["w_down"][2]                       # exact twin of expert 2
        cal = wk.to_storage(wk.std_normal(seed, "cal", 2 * 6 * 24), dtype).reshape(2, 6, 24)
        s = o.similarity_cka_linear(cal, c["w_gate_up"], c["w_down"], dtype)
        N, M = cal.shape[0], c["w_gate_up"].shape[0]
        want = np.zeros((M, M))
        for b in range(N):
            acts = [np_expert(f64(cal[b], dtype), f64(c["w_gate_up"][e], dtype), f64(c["w_down"][e], dtype))
                    for e in range(M)]
            grams = [a @ a.T for a in acts]
            h = np.array([[_hsic_ustatistic(grams[p], grams[q]) for q in range(M)] for p in range(M)])
            want += h / np.sqrt(np.outer(np.diag(h), np.diag(h)))
        want /= N
        assert np.allclose(s, want, rtol=1e-9, atol=1e-11), np.abs(s - want).max()
        assert np.allclose(s, s.T, rtol=0, atol=1e-13)
        assert np.allclose(np.diag(s), 1.0, atol=1e-13)
        assert abs(s[2, 4] - 1.0) < 1e-13
    # invariances: expert 1 = 0.5 x expert 0 (isotropic scaling), expert 2 = expert 0 followed by an
    # orthogonal map of the output space; expert 3 independent
    c = rng_case(123, wk.F32, 1, 16, 4, 6)
    q_mat, _ = np.linalg.qr(wk.std_normal(123, "q", 16 * 16).reshape(16, 16))
    c["w_gate_up"][1] = c["w_gate_up"][0]
    c["w_down"][1] = np.float32(0.5) * c["w_down"][0]
    c["w_gate_up"][2] = c["w_gate_up"][0]
    c["w_down"][2] = (q_mat @ c["w_down"][0].astype(np.float64)).astype(np.float32)
    cal = wk.std_normal(123, "cal", 2 * 7 * 16).reshape(2, 7, 16)
    s = o.similarity_cka_linear(cal, c["w_gate_up"], c["w_down"], wk.F32)
    assert abs(s[0, 1] - 1.0) < 1e-12
    assert abs(s[0, 2] - 1.0) < 1e-5          # the rotated weights were rounded to fp32
    assert abs(s[0, 3]) < 0.98
    # an expert with zero output: HSIC of its Gram matrix is 0, every pair with it contributes 0
    c = rng_case(124, wk.F32, 1, 16, 3, 4)
    c["w_down"][1] = 0
    cal = wk.std_normal(124, "cal", 5 * 16).reshape(1, 5, 16)
    s = o.similarity_cka_linear(cal, c["w_gate_up"], c["w_down"], wk.F32)
    assert np.all(s[1] == 0.0) and np.all(s[:, 1] == 0.0) and abs(s[0, 0] - 1.0) < 1e-13


def pin_similarity_cka_kernels(o):
    """CKA with the RBF and the polynomial kernel: Gram matrices written with numpy, HSIC by brute
    force over 4-tuples; invariance under orthogonal maps of the output space; a twin scores 1; the
    polynomial kernel of degree 1 and offset 0 is the linear kernel."""
    for dtype, seed in ((wk.F32, 131), (wk.BF16, 132)):
        c = rng_case(seed, dtype, 1, 24, 4, 10)
        c["w_gate_up"][3] = c["w_gate_up"][1]
        c["w_down"][3] = c["w_down"][1]                       # exact twin of expert 1
        cal = wk.to_storage(wk.std_normal(seed, "cal", 2 * 6 * 24), dtype).reshape(2, 6, 24)
        N, M = cal.shape[0], c["w_gate_up"].shape[0]
        acts = [[np_expert(f64(cal[b], dtype), f64(c["w_gate_up"][e], dtype), f64(c["w_down"][e], dtype))
                 for e in range(M)] for b in range(N)]
        sq = np.array([np.sum((a[:, None, :] - a[None, :, :]) ** 2, axis=2) for a in acts[0]])
        sigma = float(np.sqrt(np.median(sq[sq > 0])))        # kernel values spread over (0, 1)
        kernels = {
            ("rbf", sigma, 0.0): lambda a: np.exp(-np.sum((a[:, None, :] - a[None, :, :]) ** 2, axis=2)
                                                  / (2.0 * sigma ** 2)),
            ("poly", 0.5, 3.0): lambda a: (a @ a.T + 0.5) ** 3,
        }
        for (kind, p0, p1), gram_of in kernels.items():
            s = o.similarity_cka(cal, c["w_gate_up"], c["w_down"], dtype, kind, p0, p1)
            want = np.zeros((M, M))
            for b in range(N):
                grams = [gram_of(a) for a in acts[b]]
                h = np.array([[_hsic_ustatistic(grams[p], grams[q]) for q in range(M)] for p in range(M)])
                want += h / np.sqrt(np.outer(np.diag(h), np.diag(h)))
            want /= N
            assert np.allclose(s, want, rtol=1e-8, atol=1e-10), (kind, np.abs(s - want).max())
            assert np.allclose(s, s.T, rtol=0, atol=1e-13)
            assert abs(s[1, 3] - 1.0) < 1e-12 and np.allclose(np.diag(s), 1.0, atol=1e-12)
        lin = o.similarity_cka_linear(cal, c["w_gate_up"], c["w_down"], dtype)
        assert np.allclose(o.similarity_cka(cal, c["w_gate_up"], c["w_down"], dtype, "poly", 0.0, 1.0), lin,
                           rtol=0, atol=1e-13)
        assert np.array_equal(o.similarity_cka(cal, c["w_gate_up"], c["w_down"], dtype, "linear"), lin)
        rbf = o.similarity_cka(cal, c["w_gate_up"], c["w_down"], dtype, "rbf", sigma)
        assert np.abs(rbf - lin).max() > 1e-3                # a different quantity from the linear kernel
    # both kernels depend on the outputs through inner products and distances only: an orthogonal
    # map of an expert's output space leaves its Gram matrix, hence every CKA value, unchanged
    c = rng_case(133, wk.F32, 1, 16, 3, 6)
    q_mat, _ = np.linalg.qr(wk.std_normal(133, "q", 16 * 16).reshape(16, 16))
    cal = wk.std_normal(133, "cal", 2 * 7 * 16).reshape(2, 7, 16)
    rot = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    rot["w_down"][2] = (q_mat @ c["w_down"][2].astype(np.float64)).astype(np.float32)
    a0 = np_expert(cal[0].astype(np.float64), c["w_gate_up"][0].astype(np.float64), c["w_down"][0].astype(np.float64))
    sq = np.sum((a0[:, None, :] - a0[None, :, :]) ** 2, axis=2)
    sigma = float(np.sqrt(np.median(sq[sq > 0])))
    for kind, p0, p1 in (("rbf", sigma, 0.0), ("poly", float(np.mean(np.sum(a0 * a0, axis=1))), 2.0)):
        a = o.similarity_cka(cal, c["w_gate_up"], c["w_down"], wk.F32, kind, p0, p1)
        b = o.similarity_cka(cal, rot["w_gate_up"], rot["w_down"], wk.F32, kind, p0, p1)
        assert np.abs(a - b).max() < 1e-4, (kind, np.abs(a - b).max())   # rotated weights rounded to fp32


ALL_PINS = [
    pin_similarity_cka, pin_similarity_cka_kernels,
    pin_similarity_cosine,
    pin_router_logits_library, pin_topk_order_and_gate, pin_fig2_behaviour,
    pin_reroute_hand_cases, pin_reroute_against_brute, pin_reroute_invariants, pin_compact,
    pin_expert_closed_form, pin_layer_dense_formulation, pin_shared_experts_closed_form,
    pin_layer_against_brute, pin_disabled_reroute_is_standard_moe, pin_substitution_identity,
    pin_exact_twins, pin_similarity,
]
