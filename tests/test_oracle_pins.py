"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test states the passage it rests on.  The checks are written with numpy / pure Python in a
structure different from the oracle's per-token loops (dense matmuls over all experts, subset
enumeration, library softmax and stable sort), so a dropped term, a wrong sign or index or a
transposed operand in the oracle fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import softmax

from oracle import zeda_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_layer(seed, T, H, I, N, Z, scale_r=1.0):
    r = np.random.default_rng(seed)
    return dict(
        x=r.standard_normal((T, H)).astype(np.float32),
        wr=(scale_r * r.standard_normal((N + Z, H))).astype(np.float32),
        wg=(r.standard_normal((N, I, H)) / math.sqrt(H)).astype(np.float32),
        wu=(r.standard_normal((N, I, H)) / math.sqrt(H)).astype(np.float32),
        wd=(r.standard_normal((N, H, I)) / math.sqrt(I)).astype(np.float32),
    )


def _silu(v):
    return v / (1.0 + np.exp(-v))


def _dense_expert_outputs(L):
    """Y[e, t, :] = W_d[e] (silu(W_g[e] x_t) * (W_u[e] x_t)) for every expert and token, by matmuls."""
    x = L["x"].astype(np.float64)
    g = np.einsum("th,eih->eti", x, L["wg"].astype(np.float64))
    u = np.einsum("th,eih->eti", x, L["wu"].astype(np.float64))
    return np.einsum("eti,ehi->eth", _silu(g) * u, L["wd"].astype(np.float64))


def _static_topk_moe(x, wr, Y, K, bias=None):
    """Textbook static top-K MoE (Section 2.1, first formula): softmax, K largest, weights
    normalised over the K selected, weighted sum of expert outputs Y[e, t, :]."""
    logits = x.astype(np.float64) @ wr.astype(np.float64).T
    if bias is not None:
        logits = logits + bias
    p = softmax(logits, axis=1)
    order = np.argsort(-logits.astype(np.float32), axis=1, kind="stable")[:, :K]
    out = np.zeros((x.shape[0], Y.shape[2]))
    gates = np.take_along_axis(p, order, axis=1)
    gates = gates / gates.sum(axis=1, keepdims=True)
    for t in range(x.shape[0]):
        for j in range(K):
            out[t] += gates[t, j] * Y[order[t, j], t]
    return out, order, gates


def test_z0_is_static_topk_moe():
    # Section 2.1: with no zero experts the dynamic layer is the original y = sum_{i in S} g_i E_i.
    L = _rand_layer(1, T=9, H=24, I=10, N=6, Z=0)
    ref, order, gates = _static_topk_moe(L["x"], L["wr"], _dense_expert_outputs(L), K=3)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], 6, 0, 3, orc.GATE_TOPK_NORM)
    assert np.array_equal(r["ids"], order)
    np.testing.assert_allclose(r["gates"], gates, rtol=1e-12)
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-14)
    assert r["real_slots"] == 9 * 3


def test_zero_experts_equal_experts_with_zero_output():
    # Eq. 1 with the zero experts written out: a static top-K layer over N+N_Z experts whose last
    # N_Z experts return 0 (Z_j(h) = 0), weights normalised over all K selected and not renormalised
    # afterwards (Section 4.3.4).
    N, Z, K = 5, 3, 3
    L = _rand_layer(2, T=40, H=16, I=6, N=N, Z=Z)
    Y = _dense_expert_outputs(L)
    Yaug = np.concatenate([Y, np.zeros((Z,) + Y.shape[1:])], axis=0)
    ref, order, gates = _static_topk_moe(L["x"], L["wr"], Yaug, K)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, orc.GATE_TOPK_NORM)
    assert np.array_equal(r["ids"], order)
    assert (order >= N).any() and (order < N).any()
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(r["gates"], gates, rtol=1e-12)


def test_bias_enters_logits():
    N, Z, K = 4, 2, 2
    L = _rand_layer(3, T=20, H=12, I=5, N=N, Z=Z)
    bias = np.array([0.3, -0.2, 0.0, 0.7, 1.5, -1.0], dtype=np.float32)
    Y = np.concatenate([_dense_expert_outputs(L), np.zeros((Z, 20, 12))], axis=0)
    ref, order, _ = _static_topk_moe(L["x"], L["wr"], Y, K, bias=bias.astype(np.float64))
    r = orc.moe_forward(L["x"], L["wr"], bias, L["wg"], L["wu"], L["wd"], N, Z, K)
    assert np.array_equal(r["ids"], order)
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-14)


def test_all_zero_token_outputs_exact_zero():
    # Eq. 1: the sum over S~(h) ∩ E is empty when all K slots are zero experts.
    N, Z, K = 4, 3, 3
    L = _rand_layer(4, T=6, H=8, I=4, N=N, Z=Z)
    bias = np.zeros(N + Z, dtype=np.float32)
    bias[N:] = 1e4
    r = orc.moe_forward(L["x"], L["wr"], bias, L["wg"], L["wu"], L["wd"], N, Z, K)
    assert (r["ids"] >= N).all()
    assert r["real_slots"] == 0
    assert np.array_equal(r["out"], np.zeros_like(r["out"])) and not np.signbit(r["out"]).any()
    # the renormalised variant has an empty normaliser there: output is 0 as well
    r2 = orc.moe_forward(L["x"], L["wr"], bias, L["wg"], L["wu"], L["wd"], N, Z, K, orc.GATE_REAL_RENORM)
    assert np.array_equal(r2["out"], np.zeros_like(r2["out"]))


def test_gate_normalisations():
    N, Z, K = 6, 4, 4
    L = _rand_layer(5, T=50, H=16, I=4, N=N, Z=Z)
    ids_s, g_soft, logits = orc.route(L["x"], L["wr"], None, N, Z, K, orc.GATE_SOFTMAX, want_logits=True)
    ids_t, g_topk = orc.route(L["x"], L["wr"], None, N, Z, K, orc.GATE_TOPK_NORM)
    ids_r, g_ren = orc.route(L["x"], L["wr"], None, N, Z, K, orc.GATE_REAL_RENORM)
    assert np.array_equal(ids_s, ids_t) and np.array_equal(ids_s, ids_r)
    np.testing.assert_allclose(logits, L["x"].astype(np.float64) @ L["wr"].astype(np.float64).T, rtol=1e-12, atol=1e-13)
    p = np.take_along_axis(softmax(logits, axis=1), ids_s.astype(np.int64), axis=1)
    # softmax probabilities untouched
    np.testing.assert_allclose(g_soft, p, rtol=1e-12)
    # Section 4.3.4: weights are normalised over the K selected (zero experts included) and the
    # survivors keep exactly that value: they are not rescaled after the zero slots are removed.
    np.testing.assert_allclose(g_topk, p / p.sum(axis=1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(g_topk.sum(axis=1), 1.0, rtol=1e-12)
    real = ids_s < N
    assert ((g_topk * real).sum(axis=1)[(~real).any(axis=1)] < 1.0).all()
    # Eq. 7: the renormalised weights sum to one over the active normal experts
    has_real = real.any(axis=1)
    np.testing.assert_allclose((g_ren * real).sum(axis=1)[has_real], 1.0, rtol=1e-12)
    np.testing.assert_allclose(g_ren[real], (p / (p * real).sum(axis=1, keepdims=True))[real], rtol=1e-12)
    # slots are listed by descending logit
    sel = np.take_along_axis(logits, ids_s.astype(np.int64), axis=1)
    assert (np.diff(sel, axis=1) <= 0).all()


def test_renorm_output_is_rescaled_default_output():
    # Eq. 7 = Eq. 1 divided by the sum of the surviving default weights.
    N, Z, K = 5, 3, 3
    L = _rand_layer(6, T=30, H=12, I=5, N=N, Z=Z)
    a = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, orc.GATE_TOPK_NORM)
    b = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, orc.GATE_REAL_RENORM)
    s = (a["gates"] * (a["ids"] < N)).sum(axis=1)
    ok = s > 0
    np.testing.assert_allclose(b["out"][ok], a["out"][ok] / s[ok, None], rtol=1e-11, atol=1e-14)


def test_lower_index_wins_ties_and_order():
    # identical router rows give identical logits: the lower index is selected first
    N, Z, K = 3, 3, 2
    L = _rand_layer(7, T=5, H=8, I=4, N=N, Z=Z)
    L["wr"][:] = L["wr"][0]
    ids, gates = orc.route(L["x"], L["wr"], None, N, Z, K)
    assert np.array_equal(ids, np.tile(np.array([0, 1], dtype=np.int32), (5, 1)))
    np.testing.assert_allclose(gates, 0.5, rtol=1e-12)
    L["wr"][4] = L["wr"][0] * 3  # row 4 now differs; rows 0,1,2,3,5 still tie
    ids, _ = orc.route(L["x"], L["wr"], None, N, Z, K)
    lg = L["x"].astype(np.float64) @ L["wr"].astype(np.float64).T
    for t in range(5):
        exp = [4, 0] if lg[t, 4] > lg[t, 0] else [0, 1]
        assert list(ids[t]) == exp


def test_flop_count_matches_eq9_eq10():
    # Appendix D Eq. 9-10: expert FLOPs = 6 H H_e per (token, normal expert) pair; router 2 (N+N_Z) n H.
    N, Z, K, T, H, I = 6, 4, 3, 64, 16, 8
    L = _rand_layer(8, T=T, H=H, I=I, N=N, Z=Z)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K)
    R = int((r["ids"] < N).sum())
    assert r["real_slots"] == R
    r_ze = 1.0 - R / (T * K)
    assert orc.moe_flops(T, H, I, N, Z, K, r_ze) == pytest.approx(6 * H * I * R + 2 * (N + Z) * T * H, rel=1e-12)
    assert orc.moe_flops(T, H, I, N, 0, K, 0.0) == 6 * K * T * H * I + 2 * N * T * H
    off, _, _ = orc.dispatch(r["ids"], N)
    assert off[N] == R


def test_table13_theoretical_speedups():
    # Appendix D Table 13, theoretical columns, from Eq. 14 / Eq. 18 with Table 12's constants.
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table13_theoretical_speedup.txt")) if l[0] != "#"]
    assert len(rows) == 8
    for length, pre, dec in rows:
        a = 1.0 / orc.flop_ratio(True, float(length), 2048, 4096, 1 / 8, 768, 128, 64, 8, 0.5)
        b = 1.0 / orc.flop_ratio(False, float(length), 2048, 4096, 1 / 8, 768, 128, 64, 8, 0.5)
        assert abs(a - float(pre)) <= 5.01e-4, (length, a, pre)
        assert abs(b - float(dec)) <= 5.01e-4, (length, b, dec)


def test_flop_ratio_is_ratio_of_totals():
    # Eq. 14 is Eq. 13 / Eq. 12: attention (Eq. 11) + MoE (Eq. 9-10) totals, halved and divided by l.
    l, H, Ha, g, He, N, NZ, K, r = 3000.0, 2048, 4096, 0.125, 768, 128, 64, 8, 0.37
    attn = 4 * l * l * Ha + 4 * (1 + g) * l * H * Ha
    ratio = (attn + orc.moe_flops(l, H, He, N, NZ, K, r)) / (attn + orc.moe_flops(l, H, He, N, 0, K, 0.0))
    assert orc.flop_ratio(True, l, H, Ha, g, He, N, NZ, K, r) == pytest.approx(ratio, rel=1e-12)
    attn_d = 2 * l * (l - 1) * Ha + 4 * (1 + g) * l * H * Ha  # Eq. 15
    ratio_d = (attn_d + orc.moe_flops(l, H, He, N, NZ, K, r)) / (attn_d + orc.moe_flops(l, H, He, N, 0, K, 0.0))
    assert orc.flop_ratio(False, l, H, Ha, g, He, N, NZ, K, r) == pytest.approx(ratio_d, rel=1e-12)


def test_brute_force_tiny():
    # Tiny sizes: the top-K set is the K-subset with the largest logit sum; Eq. 1 evaluated with
    # python loops, zero-expert terms g_j * 0 written out.
    T, H, I, N, Z, K = 3, 4, 3, 3, 2, 2
    L = _rand_layer(9, T=T, H=H, I=I, N=N, Z=Z)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K)
    for t in range(T):
        x = [float(v) for v in L["x"][t]]
        logit = [sum(x[h] * float(L["wr"][e, h]) for h in range(H)) for e in range(N + Z)]
        best = max(itertools.combinations(range(N + Z), K), key=lambda s: sum(logit[e] for e in s))
        assert set(best) == set(int(i) for i in r["ids"][t])
        m = max(logit)
        ex = [math.exp(v - m) for v in logit]
        p = [v / sum(ex) for v in ex]
        den = sum(p[e] for e in best)
        y = [0.0] * H
        for e in best:
            if e < N:
                gv = [sum(float(L["wg"][e, i, h]) * x[h] for h in range(H)) for i in range(I)]
                uv = [sum(float(L["wu"][e, i, h]) * x[h] for h in range(H)) for i in range(I)]
                a = [gv[i] / (1 + math.exp(-gv[i])) * uv[i] for i in range(I)]
                Ey = [sum(float(L["wd"][e, h, i]) * a[i] for i in range(I)) for h in range(H)]
            else:
                Ey = [0.0] * H
            for h in range(H):
                y[h] += p[e] / den * Ey[h]
        np.testing.assert_allclose(r["out"][t], y, rtol=1e-11, atol=1e-15)


def test_dense_special_case_matches_numpy():
    # K = N, no zero experts, softmax weights: a dense softmax-weighted mixture, by plain matmuls.
    N, T, H, I = 4, 11, 10, 6
    L = _rand_layer(10, T=T, H=H, I=I, N=N, Z=0)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, 0, N, orc.GATE_SOFTMAX)
    p = softmax(L["x"].astype(np.float64) @ L["wr"].astype(np.float64).T, axis=1)
    ref = np.einsum("te,eth->th", p, _dense_expert_outputs(L))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-14)


def test_single_expert_function():
    L = _rand_layer(11, T=2, H=7, I=5, N=2, Z=0)
    y = orc.expert(L["x"][1], L["wg"][1], L["wu"][1], L["wd"][1])
    np.testing.assert_allclose(y, _dense_expert_outputs(L)[1, 1], rtol=1e-12, atol=1e-15)


def test_copy_expert_identity():
    # Appendix B: y_copy - y_zero = (sum of the weights of the selected zero-compute experts) * h.
    N, Z, K = 5, 3, 3
    L = _rand_layer(12, T=25, H=12, I=5, N=N, Z=Z)
    a = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K)
    b = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, copy_expert=True)
    zsum = (a["gates"] * (a["ids"] >= N)).sum(axis=1)
    assert (zsum > 0).any()
    np.testing.assert_allclose(b["out"] - a["out"], zsum[:, None] * L["x"].astype(np.float64), rtol=1e-10, atol=1e-13)


def test_token_permutation_and_scaling_invariants():
    N, Z, K = 5, 3, 3
    L = _rand_layer(13, T=20, H=12, I=5, N=N, Z=Z)
    a = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, want_y_slot=True)
    perm = np.random.default_rng(0).permutation(20)
    b = orc.moe_forward(L["x"][perm], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K)
    assert np.array_equal(b["out"], a["out"][perm]) and np.array_equal(b["ids"], a["ids"][perm])
    # scaling W_d of one expert by c scales exactly that expert's terms
    e, c = 2, 4.0  # a power of two: the scaled fp32 weights are exact
    wd2 = L["wd"].copy()
    wd2[e] *= c
    d = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], wd2, N, Z, K)
    contrib = np.zeros_like(a["out"])
    ys = a["y_slot"].reshape(20, K, 12)
    for t in range(20):
        for j in range(K):
            if a["ids"][t, j] == e:
                contrib[t] += a["gates"][t, j] * ys[t, j]
    np.testing.assert_allclose(d["out"], a["out"] + (c - 1.0) * contrib, rtol=1e-10, atol=1e-13)
    # y_slot rows of zero-expert slots are zero
    assert not ys[a["ids"] >= N].any()


def test_dispatch_is_stable_sort_and_combine_recovers_output():
    N, Z, K, T = 7, 5, 4, 33
    L = _rand_layer(14, T=T, H=8, I=4, N=N, Z=Z)
    r = orc.moe_forward(L["x"], L["wr"], None, L["wg"], L["wu"], L["wd"], N, Z, K, want_y_slot=True)
    ids = r["ids"]
    off, sorted_slot, slot_to_row = orc.dispatch(ids, N)
    flat = ids.ravel()
    real = np.flatnonzero(flat < N)
    ref_sorted = real[np.argsort(flat[real], kind="stable")]  # library stable sort by expert id
    R = len(real)
    assert off[N] == R
    assert np.array_equal(sorted_slot[:R], ref_sorted) and (sorted_slot[R:] == -1).all()
    assert np.array_equal(off[:N], np.searchsorted(flat[ref_sorted], np.arange(N), side="left"))
    inv = np.full(T * K, -1, dtype=np.int32)
    inv[ref_sorted] = np.arange(R)
    assert np.array_equal(slot_to_row, inv)
    for e in range(N):
        seg = sorted_slot[off[e]:off[e + 1]]
        assert (flat[seg] == e).all() and (np.diff(seg) > 0).all()
    # Eq. 1 regrouped: gathering expert-sorted rows back reproduces the forward output
    y_rows = r["y_slot"][sorted_slot[:R]]
    out = orc.combine(y_rows, ids, r["gates"], slot_to_row, N)
    np.testing.assert_allclose(out, r["out"], rtol=1e-12, atol=1e-15)


def test_argument_errors():
    L = _rand_layer(15, T=2, H=4, I=2, N=2, Z=1)
    with pytest.raises(ValueError):
        orc.route(L["x"], L["wr"], None, 2, 1, 4)  # K > N + Z
    with pytest.raises(ValueError):
        orc.route(L["x"], L["wr"], None, 2, 1, 1, gate_norm=7)


# ----------------------------------------------------------------------------------------------
# Routing statistics of Section 2.2 (Eq. 4-6)
# ----------------------------------------------------------------------------------------------
def _stats_reference(L, N, Z, K, alpha, w):
    """Eq. 4-6 written out with library softmax, a stable sort and one-hot sums (no per-token loop)."""
    logits = L["x"].astype(np.float64) @ L["wr"].astype(np.float64).T
    p = softmax(logits, axis=1)
    order = np.argsort(-logits.astype(np.float32), axis=1, kind="stable")[:, :K]
    onehot = np.zeros_like(p)
    np.put_along_axis(onehot, order, 1.0, axis=1)
    f, P = onehot.mean(axis=0), p.mean(axis=0)
    fE, PE, fZ, PZ = f[:N].sum(), P[:N].sum(), f[N:].sum(), P[N:].sum()
    LA = alpha * (N + Z) / K * float(f @ P)
    LGA = alpha * (N + Z * w) / K * (fE * PE / N + (fZ * PZ / (Z * w) if Z else 0.0))
    return f, P, fE, PE, fZ, PZ, LA, LGA


@pytest.mark.parametrize("N,Z,K,w", [(6, 3, 2, 2.0), (8, 4, 3, 0.5), (5, 0, 2, 1.0)])
def test_routing_stats_against_the_written_out_definition(N, Z, K, w):
    L = _rand_layer(61, T=97, H=24, I=8, N=N, Z=Z, scale_r=0.7)
    s = orc.routing_stats(L["x"], L["wr"], None, N, Z, K, alpha=0.01, w=w)
    f, P, fE, PE, fZ, PZ, LA, LGA = _stats_reference(L, N, Z, K, 0.01, w)
    np.testing.assert_allclose(s["f"], f, rtol=0, atol=1e-12)
    np.testing.assert_allclose(s["P"], P, rtol=1e-12, atol=1e-15)
    for got, want in ((s["f_E"], fE), (s["P_E"], PE), (s["f_Z"], fZ), (s["P_Z"], PZ), (s["L_A"], LA), (s["L_GA"], LGA)):
        assert got == pytest.approx(want, rel=1e-12, abs=1e-15)
    # invariants: every token fills K slots, probabilities sum to one, r_ZE is the zero group's share of the slots
    assert s["f"].sum() == pytest.approx(K, abs=1e-12) and s["P"].sum() == pytest.approx(1.0, abs=1e-12)
    assert s["r_ze"] == pytest.approx(s["f_Z"] / K, abs=1e-15)


def test_routing_stats_closed_forms():
    # A router whose rows are all equal gives every expert probability 1/(N+Z), whatever is selected, so Eq. 4
    # collapses to alpha * (N+Z)/K * (sum f_i)/(N+Z) = alpha; ties go to the lowest indices, so the K slots are
    # all on normal experts: f_E = K, f_Z = 0, P_E = N/(N+Z), and Eq. 5 gives alpha * (N + Z w)/(N + Z).
    N, Z, K, w, alpha = 7, 5, 3, 2.5, 0.3
    L = _rand_layer(62, T=40, H=16, I=8, N=N, Z=Z)
    L["wr"][:] = L["wr"][0]
    s = orc.routing_stats(L["x"], L["wr"], None, N, Z, K, alpha=alpha, w=w)
    np.testing.assert_allclose(s["P"], 1.0 / (N + Z), rtol=1e-12)
    np.testing.assert_allclose(s["f"], [1.0] * K + [0.0] * (N + Z - K), atol=0)
    assert s["L_A"] == pytest.approx(alpha, rel=1e-12)
    assert s["L_GA"] == pytest.approx(alpha * (N + Z * w) / (N + Z), rel=1e-12)
    # At the balance point of Section 2.2 (slots and probability split N : Z w between the groups) Eq. 5 equals
    # alpha as well.  Built by hand: a bias that sends exactly the share r* = Z w/(N + Z w) of the tokens to
    # zero experts is awkward to construct, so the identity is checked on the formula's own inputs instead:
    r = Z * w / (N + Z * w)
    fE, fZ, PE, PZ = K * (1 - r), K * r, 1 - r, r
    assert alpha * (N + Z * w) / K * (fE * PE / N + fZ * PZ / (Z * w)) == pytest.approx(alpha, rel=1e-12)


def test_routing_stats_bias_moves_slots_to_the_zero_group():
    # a large bias on the zero experts routes every slot there: f_Z = K, r_ZE = 1, and P_Z -> 1
    N, Z, K = 6, 4, 3
    L = _rand_layer(63, T=50, H=16, I=8, N=N, Z=Z, scale_r=0.3)
    bias = np.zeros(N + Z, dtype=np.float32)
    bias[N:] = 40.0
    s = orc.routing_stats(L["x"], L["wr"], bias, N, Z, K)
    assert s["f_Z"] == pytest.approx(K) and s["r_ze"] == pytest.approx(1.0) and s["P_Z"] > 1 - 1e-9
    with pytest.raises(ValueError):
        orc.routing_stats(L["x"], L["wr"], None, N, Z, K, w=0.0)


def test_token_zero_slots_hand_case_and_what_it_must_add_up_to():
    """Section 4.1's token-level r_ZE: a hand case, then, on a routed batch, two identities with functions that do
    not share code with it - the real slots the counting sort places (T*K - sum = offsets[N]) and the batch r_ZE of
    the Section 2.2 statistics (mean of the per-token shares)."""
    ids = np.array([[0, 5, 2], [4, 3, 6], [1, 2, 0], [3, 3, 3]], dtype=np.int32)  # N = 3: ids >= 3 are zero experts
    assert orc.token_zero_slots(ids, 3).tolist() == [1, 3, 0, 3]
    assert orc.token_zero_slots(ids, 7).tolist() == [0, 0, 0, 0]
    assert orc.token_zero_slots(ids[:0], 3).tolist() == []
    N, Z, K = 6, 4, 3
    L = _rand_layer(64, T=90, H=16, I=8, N=N, Z=Z, scale_r=0.4)
    bias = np.zeros(N + Z, dtype=np.float32)
    bias[N:] = 0.2
    tid, _ = orc.route(L["x"], L["wr"], bias, N, Z, K)
    z = orc.token_zero_slots(tid, N)
    assert z.min() >= 0 and z.max() <= K and 0 < z.sum() < 90 * K
    assert [sum(1 for e in row if e >= N) for row in tid.tolist()] == z.tolist()  # written out token by token
    off, _, s2r = orc.dispatch(tid, N)
    assert 90 * K - int(z.sum()) == int(off[N])
    assert np.array_equal((s2r.reshape(90, K) < 0).sum(axis=1), z)
    s = orc.routing_stats(L["x"], L["wr"], bias, N, Z, K)
    assert float(np.mean(z / K)) == pytest.approx(s["r_ze"], rel=1e-12)


# ----------------------------------------------------------------------------------------------
# Router rows of the zero experts (Section 2.1, router initialisation)
# ----------------------------------------------------------------------------------------------
def test_zero_expert_row_initialisation():
    r = np.random.default_rng(71)
    N, Z, H = 9, 5, 40
    wr = (0.3 + 0.05 * r.standard_normal((N, H))).astype(np.float32)
    z = r.standard_normal((Z, H)).astype(np.float32)
    rows, mean, var = orc.init_zero_rows(wr, z)
    # the library routines on the same numbers
    assert mean == pytest.approx(np.mean(wr.astype(np.float64)), rel=1e-13)
    assert var == pytest.approx(np.var(wr.astype(np.float64)), rel=1e-12)
    np.testing.assert_allclose(rows, mean + math.sqrt(var) * z.astype(np.float64), rtol=1e-14)
    # equal original parameters: no spread, every new parameter is that value
    rows, mean, var = orc.init_zero_rows(np.full((N, H), 0.25, dtype=np.float32), z)
    assert var == 0.0 and np.all(rows == 0.25)
    # +a / -a in equal numbers: mean 0, standard deviation a, so the new rows are a * (the draws)
    pm = np.where((np.arange(N * H) % 2) == 0, 0.5, -0.5).astype(np.float32).reshape(N, H)
    rows, mean, var = orc.init_zero_rows(pm, z)
    assert mean == 0.0 and var == 0.25
    np.testing.assert_array_equal(rows, 0.5 * z.astype(np.float64))
    # many draws: the new parameters have the mean and the variance of the old ones (sampling error ~ 1/sqrt(n))
    rows, mean, var = orc.init_zero_rows(wr, r.standard_normal((2000, H)).astype(np.float32))
    assert np.mean(rows) == pytest.approx(mean, abs=4 * math.sqrt(var / rows.size))
    assert np.var(rows) == pytest.approx(var, rel=0.03)


# ----------------------------------------------------------------------------------------------
# Pre-norm of the layer-stack workload (the paper's layer has no norm: Appendix D leaves norms and residuals out
# of its model; the stack of benchmark configuration 5 chains layers as x <- x + MoE(RMSNorm(x)))
# ----------------------------------------------------------------------------------------------
def test_rmsnorm_hand_cases():
    # x = (3, 4): mean of squares 12.5, so without eps the row is divided by sqrt(12.5)
    out = orc.rmsnorm(np.array([[3.0, 4.0]]), None, 0.0)
    np.testing.assert_allclose(out, np.array([[3.0, 4.0]]) / math.sqrt(12.5), rtol=1e-15)
    assert out[0, 0] == pytest.approx(0.8485281374238570, rel=1e-14)  # 3 / sqrt(12.5), typed in
    # a unit-RMS row is left alone; scaling the input by c > 0 changes nothing when eps = 0
    np.testing.assert_allclose(orc.rmsnorm(np.array([[1.0, -1.0, 1.0, -1.0]]), None, 0.0), [[1.0, -1.0, 1.0, -1.0]], rtol=1e-15)
    x = np.random.default_rng(3).standard_normal((5, 24))
    np.testing.assert_allclose(orc.rmsnorm(37.5 * x, None, 0.0), orc.rmsnorm(x, None, 0.0), rtol=1e-13)
    # the mean is over the H entries of the row (not a sum, not over rows): rows of different scale are
    # normalised separately, and every output row has mean square 1
    xs = x * np.array([1e-3, 1.0, 10.0, 1e3, 1e5])[:, None]
    np.testing.assert_allclose(np.mean(orc.rmsnorm(xs, None, 0.0) ** 2, axis=1), np.ones(5), rtol=1e-13)


def test_rmsnorm_written_out_definition_gamma_and_eps():
    r = np.random.default_rng(17)
    x = r.standard_normal((7, 48)) * 1.7
    gamma = r.uniform(0.5, 1.5, 48)
    eps = 0.37  # large on purpose: an eps outside the root, or added to the sum instead of the mean, shows
    want = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps) * gamma[None, :]
    np.testing.assert_allclose(orc.rmsnorm(x, gamma, eps), want, rtol=1e-14)
    # gamma scales each column and nothing else
    np.testing.assert_allclose(orc.rmsnorm(x, gamma, eps), orc.rmsnorm(x, None, eps) * gamma[None, :], rtol=1e-15)
    assert not np.allclose(orc.rmsnorm(x, None, eps), orc.rmsnorm(x, None, 0.0), rtol=1e-3)
    # an all-zero row: eps alone is under the root, the result is exactly zero (no 0/0)
    z = np.zeros((1, 16))
    out = orc.rmsnorm(z, None, 1e-6)
    assert np.all(out == 0.0) and not np.isnan(out).any()
    # a row far smaller than sqrt(eps) is scaled by 1/sqrt(eps), not normalised to unit size
    tiny = np.full((1, 16), 1e-9)
    np.testing.assert_allclose(orc.rmsnorm(tiny, None, 1e-6), tiny / math.sqrt(1e-6 + 1e-18), rtol=1e-14)
    np.testing.assert_allclose(orc.rmsnorm(tiny, None, 1e-6), tiny * 1e3, rtol=1e-9)
