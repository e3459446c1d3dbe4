"""Forward variants the paper describes next to the default layer: the copy expert of Appendix B, and the
NET baseline of Section 3.1 (the static layer with half the slots: Z = 0, K/2)."""
import numpy as np
import pytest
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth, zeda

pytestmark = pytest.mark.gpu

from gpu_util import desc_of, forward, full_parity  # noqa: E402


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("dtype,seed", [("bf16", 101), ("f32", 102)])
def test_copy_expert_layer_matches_oracle(dtype, seed):
    w = synth.Workload("copy", T=500, H=256, I=128, N=10, Z=6, K=4, dtype=dtype, seed=seed, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.3)
    _say("copy expert", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, copy_expert=True)
    _say(st)
    # Appendix B: y_copy - y_zero = (sum of the routing weights of the token's parameter-free slots) * h
    zero = forward(w, L)
    ids, gates = zero["topk_ids"].numpy(), zero["topk_gates"].numpy().astype(np.float64)
    gz = np.where(ids >= w.N, gates, 0.0).sum(axis=1)
    x = synth.to_numpy_f32(L["x"]).astype(np.float64)
    diff = res["out"].double().numpy() - zero["out"].double().numpy()
    want = gz[:, None] * x
    tol = 2e-2 if dtype == "bf16" else 1e-5 * np.abs(want).max()
    assert np.max(np.abs(diff - want)) <= tol
    assert (gz > 0).any() and (gz == 0).any()


def test_copy_expert_combine_alone_with_all_slots_free():
    # a token whose slots are all parameter-free returns (sum of its weights) * h, the others the usual sum
    rng = np.random.default_rng(9)
    T, H, N, Z, K = 70, 128, 5, 4, 3
    ids = rng.integers(0, N + Z, size=(T, K)).astype(np.int32)
    ids[3] = [N, N + 1, N + 3]
    gates = rng.random((T, K)).astype(np.float32)
    off, ss, s2r = orc.dispatch(ids, N)
    R = int(off[N])
    y = (0.3 * torch.randn(T * K, H, dtype=torch.float32))
    x = torch.randn(T, H, dtype=torch.float32)
    d = zeda.make_desc(T, H, 64, N, Z, K, "f32", free_expert=zeda.EXPERT_COPY)
    out = torch.full((T, H), float("nan"), dtype=torch.float32, device="cuda")
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    zeda.zeda_combine(d, y.cuda(), dev(ids), dev(gates), dev(s2r), out, x=x.cuda())
    torch.cuda.synchronize()
    ref = orc.combine(y.numpy().astype(np.float64)[:max(R, 1)], ids, gates.astype(np.float64), s2r, N)
    ref += np.where(ids >= N, gates.astype(np.float64), 0.0).sum(axis=1)[:, None] * x.numpy().astype(np.float64)
    got = out.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) <= 1e-5 * np.abs(ref).max()
    np.testing.assert_allclose(got[3], gates[3].astype(np.float64).sum() * x.numpy()[3], rtol=1e-5, atol=1e-6)
    with pytest.raises(zeda.ZedaError):
        zeda.zeda_combine(d, y.cuda(), dev(ids), dev(gates), dev(s2r), out)  # the layer input is required in this mode


def test_net_baseline_static_layer_with_half_the_slots():
    # Section 3.1's NET: no parameter-free experts, K/2 slots per token - the same path at Z = 0
    w = synth.CONFIGS["c2_qwen_prefill"].with_(Z=0, K=4, recipe="plain", T=768)
    _say("NET", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tokens=np.arange(0, w.T, 3))
    _say(st)
    assert st["R"] == w.T * w.K and st["r_ze"] == 0.0


# Further workloads: the paper's own zero-expert count on the Qwen3 shape (N_Z = 64, so 192 router rows), its
# decode concurrency of 32, and a layer with the router of its second model (N = 64, K = 4, N_Z = 32).
@pytest.mark.parametrize("name,sample", [("n1_qwen_nz64_prefill", 256), ("n1_qwen_nz64_decode32", None),
                                         ("n1_glm_like_prefill", 256)])
def test_further_workloads(name, sample):
    w = synth.CONFIGS[name]
    _say(name, w)
    L = harness.gapped_layer(w, "cuda")
    tokens = None if sample is None else np.sort(np.random.default_rng(1).choice(w.T, size=sample, replace=False))
    res, st = full_parity(w, L, tokens=tokens, tiled=True)
    _say(st)
    if w.T >= 1024:
        assert abs(st["r_ze"] - 0.5) < 0.03


@pytest.mark.parametrize("T", [2048, 8192])
def test_sequence_length_sweep_ends(T):
    # the paper varies the sequence length between 2k and 8k: both ends on the Qwen3 layer, sampled tokens
    w = synth.CONFIGS["c2_qwen_prefill"].with_(T=T, seed=21)
    _say("T sweep", w)
    L = harness.gapped_layer(w, "cuda")
    tokens = np.sort(np.random.default_rng(2).choice(w.T, size=128, replace=False))
    res, st = full_parity(w, L, tokens=tokens, tiled=True)
    _say(st)


# Batch routing statistics of Section 2.2 (f_i, P_i, group sums, forward values of Eq. 4-6) against the oracle.
STATS_CASES = [
    dict(T=1000, H=256, I=64, N=10, Z=6, K=4, dtype="bf16", seed=111, zero_bias=0.3),
    dict(T=77, H=132, I=52, N=7, Z=5, K=3, dtype="f32", seed=112, zero_bias=0.2),
    dict(T=300, H=128, I=64, N=9, Z=0, K=2, dtype="bf16", seed=113, zero_bias=0.0),
    dict(T=5000, H=512, I=64, N=128, Z=64, K=8, dtype="bf16", seed=114, zero_bias=0.3),
    dict(T=9000, H=128, I=64, N=40, Z=24, K=8, dtype="bf16", seed=115, zero_bias=0.4),  # too many token blocks to split H
]


@pytest.mark.parametrize("cfg", STATS_CASES, ids=lambda c: "T%d_N%d_Z%d_K%d_%s" % (c["T"], c["N"], c["Z"], c["K"], c["dtype"]))
def test_routing_stats_match_oracle(cfg):
    w = synth.Workload("stats", recipe="zero_bias", x_std=1.0, w_std=0.05, wr_std=0.05, **cfg)
    _say("routing stats", w)
    L = harness.gapped_layer(w, "cuda")
    alpha, gw = 0.01, 2.0
    f, P, summ = zeda.zeda_routing_stats(desc_of(w), L["x"], L["w_router"], L["router_bias"], alpha=alpha, w=gw)
    torch.cuda.synchronize()
    a = harness.to_arrays(L)
    ref = orc.routing_stats(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K, alpha=alpha, w=gw)
    # counts are exact (f = count / T in both; gapped tokens have an unambiguous top-K set)
    np.testing.assert_allclose(f.cpu().numpy().astype(np.float64), ref["f"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(P.cpu().numpy().astype(np.float64), ref["P"], rtol=2e-5, atol=1e-7)
    got = summ.cpu().numpy().astype(np.float64)
    want = np.array([ref[k] for k in ("f_E", "P_E", "f_Z", "P_Z", "r_ze", "L_A", "L_GA")])
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=1e-7)
    # what the ids of the forward path imply: r_ZE is the share of slots on zero experts
    res = forward(w, L)
    assert got[4] == pytest.approx(1.0 - int(res["num_real"].item()) / (w.T * w.K), abs=1e-6)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero_expert_router_rows_initialisation(dtype):
    # Section 2.1: new router rows are Gaussian with the mean and variance of the original router parameters
    N, Z, H = 24, 8, 256
    g = torch.Generator().manual_seed(3)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    wr = torch.empty((N + Z, H), dtype=tdt)
    wr[:N] = (0.1 + 0.02 * torch.randn((N, H), generator=g)).to(tdt)
    wr[N:] = float("nan")
    z = torch.randn((Z, H), generator=g, dtype=torch.float32)
    d = zeda.make_desc(1, H, 64, N, Z, 2, dtype)
    dev = wr.cuda()
    stats = zeda.zeda_init_zero_expert_rows(d, dev, z.cuda())
    torch.cuda.synchronize()
    rows, mean, var = orc.init_zero_rows(wr[:N].float().numpy(), z.numpy())
    got = dev.float().cpu().numpy()
    assert np.array_equal(got[:N], wr[:N].float().numpy())  # the original rows are untouched
    np.testing.assert_allclose(stats.cpu().numpy(), [mean, var], rtol=1e-6)
    tol = 2.0 ** -8 if dtype == "bf16" else 1e-6  # one rounding of the result to the element type
    np.testing.assert_allclose(got[N:], rows, rtol=tol, atol=1e-7)
