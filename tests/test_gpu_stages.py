"""Each C-ABI entry point on its own against the oracle: the router, the dispatch on hand-made id
patterns (empty experts, all-zero, single expert), the expert FFN fed with the oracle's dispatch, and the
combine fed with arbitrary per-slot rows."""
import numpy as np
import pytest
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth, zeda

pytestmark = pytest.mark.gpu

from gpu_util import check_float, desc_of  # noqa: E402


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("gate_norm", [zeda.GATE_SOFTMAX, zeda.GATE_TOPK_NORM, zeda.GATE_REAL_RENORM])
def test_route_alone(dtype, gate_norm):
    w = synth.Workload("route", T=203, H=384, I=64, N=70, Z=27, K=6, dtype=dtype, seed=51, recipe="zero_bias",
                       wr_std=0.05, zero_bias=0.35)
    print(w, gate_norm, flush=True)
    L = harness.gapped_layer(w, "cuda", gate_norm=gate_norm)
    d = desc_of(w, gate_norm)
    ids = torch.full((w.T, w.K), -1, dtype=torch.int32, device="cuda")
    gates = torch.full((w.T, w.K), float("nan"), dtype=torch.float32, device="cuda")
    zeda.zeda_route(d, L["x"], L["w_router"], L["router_bias"], ids, gates)
    torch.cuda.synchronize()
    a = harness.to_arrays(L)
    rid, rg = orc.route(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K, gate_norm)
    assert np.array_equal(ids.cpu().numpy(), rid)
    np.testing.assert_allclose(gates.cpu().numpy().astype(np.float64), rg, rtol=2e-5, atol=1e-7)
    # without the bias pointer the router is the paper's plain one
    zeda.zeda_route(d, L["x"], L["w_router"], None, ids, gates)
    torch.cuda.synchronize()
    rid0, _, lg = orc.route(a["x"], a["w_router"], None, w.N, w.Z, w.K, gate_norm, want_logits=True)
    safe = harness.topk_gaps(lg, w.K) >= harness.GAP
    assert safe.mean() > 0.8 and np.array_equal(ids.cpu().numpy()[safe], rid0[safe])


@pytest.mark.parametrize("T,H", [(203, 1024), (64, 2048), (5, 512), (1000, 384)])
def test_route_with_scratch_splits_the_hidden_dimension(T, H):
    # few token blocks: with scratch several workgroups share a block (each a slice of H) and a second kernel
    # selects; the result must be the oracle's either way
    w = synth.Workload("route_ws", T=T, H=H, I=64, N=70, Z=27, K=6, dtype="bf16", seed=52, recipe="zero_bias",
                       wr_std=0.05, zero_bias=0.35)
    print(w, flush=True)
    L = harness.gapped_layer(w, "cuda")
    d = desc_of(w)
    nbytes = zeda.route_workspace_bytes(d)
    assert (nbytes > 0) == (H % 128 == 0 and T < 256 * 32)
    a = harness.to_arrays(L)
    rid, rg = orc.route(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K)
    for ws in (torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda"), None):
        ids = torch.full((w.T, w.K), -1, dtype=torch.int32, device="cuda")
        gates = torch.full((w.T, w.K), float("nan"), dtype=torch.float32, device="cuda")
        zeda.zeda_route(d, L["x"], L["w_router"], L["router_bias"], ids, gates, ws=ws)
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), rid)
        np.testing.assert_allclose(gates.cpu().numpy().astype(np.float64), rg, rtol=2e-5, atol=1e-7)


@pytest.mark.parametrize("T, N, Z", [(8192, 128, 32), (8193, 128, 32), (9001, 70, 26), (12288, 128, 32), (12301, 30, 10),
                                     (13000, 150, 42), (12500, 200, 56)])
def test_route_of_many_tokens(T, N, Z):
    # above 8192 tokens the bf16 router gives a workgroup 64 tokens instead of 32 (routers of up to 192
    # experts; wider ones keep the 32-token blocks): exact ids and gates against the oracle, ragged last block
    w = synth.Workload("route_wide", T=T, H=256, I=64, N=N, Z=Z, K=6, dtype="bf16", seed=53, recipe="zero_bias",
                       wr_std=0.08, zero_bias=0.3)
    print(w, flush=True)
    L = harness.gapped_layer(w, "cuda")
    d = desc_of(w)
    ids = torch.full((w.T, w.K), -1, dtype=torch.int32, device="cuda")
    gates = torch.full((w.T, w.K), float("nan"), dtype=torch.float32, device="cuda")
    zeda.zeda_route(d, L["x"], L["w_router"], L["router_bias"], ids, gates)
    torch.cuda.synchronize()
    a = harness.to_arrays(L)
    rid, rg = orc.route(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K)
    assert np.array_equal(ids.cpu().numpy(), rid)
    np.testing.assert_allclose(gates.cpu().numpy().astype(np.float64), rg, rtol=2e-5, atol=1e-7)


def _dispatch(ids_np, N, Z, K):
    T = ids_np.shape[0]
    d = zeda.make_desc(T, 128, 64, N, Z, K, "bf16")
    ids = _dev(ids_np.astype(np.int32))
    S = T * K
    off = torch.full((N + 1,), -5, dtype=torch.int32, device="cuda")
    ss = torch.full((max(S, 1),), -5, dtype=torch.int32, device="cuda")
    s2r = torch.full((max(S, 1),), -5, dtype=torch.int32, device="cuda")
    nr = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(zeda.dispatch_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    zeda.zeda_dispatch(d, ids, off, ss, s2r, nr, ws)
    torch.cuda.synchronize()
    roff, rss, rs2r = orc.dispatch(ids_np.astype(np.int32), N)
    R = int(roff[N])
    assert np.array_equal(off.cpu().numpy(), roff)
    assert int(nr.item()) == R
    assert np.array_equal(ss.cpu().numpy()[:R], rss[:R])
    assert np.array_equal(s2r.cpu().numpy()[:S], rs2r)
    return R


def test_dispatch_patterns():
    rng = np.random.default_rng(3)
    N, Z, K = 37, 11, 5
    # random ids (slots of one token need not be distinct for the dispatch)
    assert _dispatch(rng.integers(0, N + Z, size=(1000, K)), N, Z, K) > 0
    # only three experts ever used: most experts are empty
    assert _dispatch(rng.choice([2, 17, 36, N + 3], size=(513, K)), N, Z, K) > 0
    # every slot on a zero expert
    assert _dispatch(np.full((300, K), N + 1), N, Z, K) == 0
    # every slot on the last normal expert; a single token; sizes around the 256- and 4096-slot boundaries
    assert _dispatch(np.full((64, K), N - 1), N, Z, K) == 64 * K
    assert _dispatch(rng.integers(0, N + Z, size=(1, K)), N, Z, K) >= 0
    for T in (51, 52, 819, 820, 4097):
        _dispatch(rng.integers(0, N + Z, size=(T, K)), N, Z, K)
    # the widest pool
    _dispatch(rng.integers(0, 256, size=(700, 16)), 200, 56, 16)


def test_dispatch_large_skewed():
    # config-4-like size: 131072 slots, Zipf-like skew with empty experts
    rng = np.random.default_rng(4)
    N, Z, K, T = 128, 32, 8, 16384
    p = np.arange(1, N + Z + 1, dtype=np.float64) ** -1.3
    p[5] = p[77] = 0.0
    ids = rng.choice(N + Z, size=(T, K), p=p / p.sum())
    assert _dispatch(ids, N, Z, K) > 0


@pytest.mark.parametrize("cfg", [
    dict(T=900, H=256, I=192, N=5, Z=3, K=3, dtype="bf16"),   # several token tiles per expert, ragged tails
    dict(T=50, H=128, I=64, N=9, Z=3, K=4, dtype="bf16"),     # decode-sized tile
    dict(T=40, H=132, I=52, N=6, Z=2, K=2, dtype="f32"),
], ids=lambda c: "%s_T%d" % (c["dtype"], c["T"]))
def test_expert_ffn_alone(cfg):
    w = synth.Workload("ffn", seed=61, recipe="zero_bias", w_std=0.06, wr_std=0.05, zero_bias=0.2, **cfg)
    print(w, flush=True)
    L = synth.make_layer(w, "cuda")
    a = harness.to_arrays(L)
    ref = harness.oracle_forward(w, a, want_y_slot=True)
    off, ss, s2r = orc.dispatch(ref["ids"], w.N)
    R = int(off[w.N])
    d = desc_of(w)
    S = w.T * w.K
    ssd = ss.copy()
    ssd[R:] = 0
    y = torch.full((S, w.H), float("nan"), dtype=w.torch_dtype, device="cuda")
    ws = torch.empty(zeda.expert_ffn_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    zeda.zeda_expert_ffn(d, L["x"], L["w_gate"], L["w_up"], L["w_down"], _dev(off), _dev(ssd), _dev(np.array([R], dtype=np.int32)), y, ws)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy()
    check_float(w, got[:R], ref["y_slot"][ss[:R]], "y_slot")
    assert np.isnan(got[R:]).all()  # rows past R are not written


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_combine_alone(dtype):
    rng = np.random.default_rng(7)
    T, H, N, Z, K = 333, 256, 11, 5, 4
    ids = rng.integers(0, N + Z, size=(T, K)).astype(np.int32)
    ids[7] = N + 1  # a token with no real slot
    gates = rng.random((T, K)).astype(np.float32)
    off, ss, s2r = orc.dispatch(ids, N)
    R = int(off[N])
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    y = (0.3 * torch.randn(T * K, H, dtype=torch.float32)).to(tdt)
    y[R:] = float("nan")  # never read
    d = zeda.make_desc(T, H, 64, N, Z, K, dtype)
    out = torch.full((T, H), float("nan"), dtype=tdt, device="cuda")
    zeda.zeda_combine(d, y.cuda(), _dev(ids), _dev(gates), _dev(s2r), out)
    torch.cuda.synchronize()
    ref = orc.combine(y.float().numpy().astype(np.float64)[:max(R, 1)], ids, gates.astype(np.float64), s2r, N)
    got = out.float().cpu().numpy()
    w = synth.Workload("c", T=T, H=H, I=64, N=N, Z=Z, K=K, dtype=dtype, seed=0, recipe="plain")
    if dtype == "bf16":
        # the output itself is rounded to bf16 once: compare against that rounding with a matching tolerance
        assert np.max(np.abs(got - ref)) <= 2e-2 and harness.rel_l2(got, ref) <= 1e-2
    else:
        check_float(w, got, ref, "out")
    assert not got[7].any()


@pytest.mark.parametrize("T, N, Z, K", [(4096, 128, 32, 8), (4097, 128, 32, 8), (6144, 128, 32, 8), (7000, 5, 3, 7),
                                        (16384, 128, 32, 8), (65536, 256, 0, 8), (50000, 1, 3, 1)])
def test_dispatch_of_long_slot_lists(T, N, Z, K):
    # above 32768 slots the dispatch runs in its segmented form (two kernels, per-segment counts
    # in the workspace): random ids, ragged last segment, one expert only, the widest router, and the sizes of the
    # 8k and 16k-token benchmark configurations; everything is compared bit for bit with the oracle's counting sort
    S = T * K
    g = torch.Generator().manual_seed(T + N)
    ids = torch.randint(0, N + Z, (T, K), generator=g, dtype=torch.int32)
    if N > 2:
        ids[ids == 1] = 0  # an empty expert in the middle of the list
    d = zeda.make_desc(T, 128, 64, N, Z, K, "bf16")
    need = zeda.dispatch_workspace_bytes(d)
    assert need >= ((S + 2047) // 2048) * N * 4 if S > 32768 else need > 0
    dev = ids.cuda()
    off = torch.full((N + 1,), -7, dtype=torch.int32, device="cuda")
    ss = torch.full((S,), -7, dtype=torch.int32, device="cuda")
    s2r = torch.full((S,), -7, dtype=torch.int32, device="cuda")
    nreal = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    zeda.zeda_dispatch(d, dev, off, ss, s2r, nreal, ws)
    torch.cuda.synchronize()
    roff, rss, rs2r = orc.dispatch(ids.numpy(), N)
    R = int(roff[N])
    assert int(nreal.item()) == R
    assert np.array_equal(off.cpu().numpy(), roff)
    assert np.array_equal(ss.cpu().numpy()[:R], rss[:R]) and (ss.cpu().numpy()[R:] == -7).all()
    assert np.array_equal(s2r.cpu().numpy(), rs2r.reshape(-1))


@pytest.mark.parametrize("T, N, Z, K, dtype", [(203, 70, 27, 6, "bf16"), (1, 3, 2, 5, "bf16"), (1000, 5, 0, 2, "bf16"),
                                               (77, 7, 5, 3, "f32")])
def test_token_zero_slots_against_the_oracle(T, N, Z, K, dtype):
    # token-level zero-expert usage (Section 4.1): the ids the GPU router wrote, counted per token; overwrite, then
    # accumulate a second time (the sum over two layers)
    w = synth.Workload("tz", T=T, H=128, I=64, N=N, Z=Z, K=K, dtype=dtype, seed=57, recipe="zero_bias", wr_std=0.08,
                       zero_bias=0.3)
    print(w, flush=True)
    L = harness.gapped_layer(w, "cuda")
    d = desc_of(w)
    ids = torch.empty((w.T, w.K), dtype=torch.int32, device="cuda")
    gates = torch.empty((w.T, w.K), dtype=torch.float32, device="cuda")
    zeda.zeda_route(d, L["x"], L["w_router"], L["router_bias"], ids, gates)
    a = harness.to_arrays(L)
    rid, _ = orc.route(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K)
    ref = orc.token_zero_slots(rid, w.N)
    zs = torch.full((w.T,), -9, dtype=torch.int32, device="cuda")
    zeda.zeda_token_zero_slots(d, ids, zs)
    torch.cuda.synchronize()
    assert np.array_equal(zs.cpu().numpy(), ref)
    zeda.zeda_token_zero_slots(d, ids, zs, accumulate=True)
    torch.cuda.synchronize()
    assert np.array_equal(zs.cpu().numpy(), 2 * ref)
    with pytest.raises(zeda.ZedaError):
        zeda.zeda_token_zero_slots(d, None, zs)
