"""benchmark configuration 5: a chain of MoE layers with RMSNorm + residual between them (no attention).

Inputs of layers >= 1 cannot be re-drawn to keep a logit gap, so each checked layer is teacher-forced: the
oracle gets the GPU's own normalised input of that layer, routing is compared on the tokens whose oracle gap is
>= 1e-3 (the number of excluded tokens is printed), and the expert arithmetic on a sample of tokens."""
import numpy as np
import pytest
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth, zeda
from paper_2605_18643_amd.stack import EPS, MoeStack

pytestmark = pytest.mark.gpu

from gpu_util import check_float  # noqa: E402


def _say(*a):
    print(*a, flush=True)


def test_rmsnorm_and_residual_kernels():
    for dt, tol in ((torch.bfloat16, 6e-3), (torch.float32, 2e-6)):
        x = (torch.randn(67, 384) * 1.7).to(dt).cuda()
        g = (torch.rand(384) + 0.5).to(dt).cuda()
        out = torch.empty_like(x)
        zeda.zeda_rmsnorm(x, g, EPS, out)
        ref = orc.rmsnorm(x.float().cpu().numpy(), g.float().cpu().numpy(), EPS)
        np.testing.assert_allclose(out.float().cpu().numpy(), ref, rtol=tol, atol=tol * 1e-2)
        zeda.zeda_rmsnorm(x, None, EPS, out)
        np.testing.assert_allclose(out.float().cpu().numpy(), orc.rmsnorm(x.float().cpu().numpy(), None, EPS), rtol=tol, atol=tol * 1e-2)
        y = torch.randn(67, 384).to(dt).cuda()
        want = (x.float() + y.float()).to(dt)
        zeda.zeda_residual_add(x, y)
        assert torch.equal(x, want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("copy_expert", [False, True])
def test_block_forward_against_the_oracle(dtype, copy_expert):
    # one pre-norm residual block in one call: x_res += layer(xn), xn_next = RMSNorm(x_res) * gamma
    w = synth.Workload("block", T=333, H=256, I=128, N=8, Z=4, K=3, dtype=dtype, seed=77, recipe="zero_bias",
                       x_std=1.0, w_std=0.06, wr_std=0.2, zero_bias=0.2)
    _say("block forward:", w, "copy expert" if copy_expert else "zero expert")
    xn = synth.draw_tokens(w, "cuda")
    wr, bias = synth.draw_router(w, "cuda")
    wg, wu, wd = synth.draw_experts(w, "cuda")
    g = torch.Generator().manual_seed(5)
    x_res0 = (torch.randn(w.T, w.H, generator=g) * 2.0).to(w.torch_dtype).cuda()
    gamma = (torch.rand(w.H, generator=g) + 0.5).to(w.torch_dtype).cuda()
    desc = zeda.make_desc(w.T, w.H, w.I, w.N, w.Z, w.K, w.dtype,
                          free_expert=zeda.EXPERT_COPY if copy_expert else zeda.EXPERT_ZERO)
    ws = torch.empty(zeda.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    nreal = torch.zeros(1, dtype=torch.int32, device="cuda")
    x_res, xn_next = x_res0.clone(), torch.empty_like(xn)
    zeda.zeda_moe_block_forward(desc, xn, x_res, wr, bias, wg, wu, wd, gamma, EPS, xn_next, nreal, ws)
    torch.cuda.synchronize()
    a = [synth.to_numpy_f32(v) for v in (xn, wr, bias, wg, wu, wd)]
    r = orc.moe_forward(*a, w.N, w.Z, w.K, copy_expert=copy_expert)
    assert np.array_equal(zeda.ws_views(desc, ws)["topk_ids"].cpu().numpy(), r["ids"])
    assert int(nreal.item()) == int((r["ids"] < w.N).sum())
    want = x_res0.double().cpu().numpy() + r["out"]
    got = x_res.double().cpu().numpy()
    # one rounding of the sum to the element type, on top of the expert arithmetic's own error
    step = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    assert np.max(np.abs(got - want)) <= step * np.max(np.abs(want)) + (2e-2 if dtype == "bf16" else 1e-5)
    assert harness.rel_l2(got, want) < (1e-2 if dtype == "bf16" else 1e-5)
    # the norm is taken of the row as stored
    ref_n = orc.rmsnorm(synth.to_numpy_f32(x_res), synth.to_numpy_f32(gamma), EPS)
    tol = 6e-3 if dtype == "bf16" else 2e-6
    np.testing.assert_allclose(xn_next.float().cpu().numpy(), ref_n, rtol=tol, atol=tol * 1e-2)
    # the three-call form gives the same stream up to the extra rounding of its separate layer output
    y = torch.empty_like(xn)
    zeda.zeda_moe_forward(desc, xn, wr, bias, wg, wu, wd, y, nreal, ws)
    x3 = x_res0.clone()
    zeda.zeda_residual_add(x3, y)
    torch.cuda.synchronize()
    assert harness.rel_l2(x3.double().cpu().numpy(), got) < (4e-3 if dtype == "bf16" else 1e-6)
    # no next input wanted; and the next input written over the layer's own input
    x_b = x_res0.clone()
    zeda.zeda_moe_block_forward(desc, xn, x_b, wr, bias, wg, wu, wd, None, EPS, None, nreal, ws)
    xn_io = xn.clone()
    x_c = x_res0.clone()
    zeda.zeda_moe_block_forward(desc, xn_io, x_c, wr, bias, wg, wu, wd, gamma, EPS, xn_io, nreal, ws)
    torch.cuda.synchronize()
    assert torch.equal(x_b, x_res) and torch.equal(x_c, x_res) and torch.equal(xn_io, xn_next)


def test_block_forward_rows_wider_than_one_pass():
    # H / 8 > 256: a thread keeps several pieces of the row between the add and the norm
    w = synth.Workload("block_wide", T=70, H=2048 + 512, I=64, N=4, Z=2, K=2, dtype="bf16", seed=78, recipe="zero_bias",
                       x_std=1.0, w_std=0.03, wr_std=0.05, zero_bias=0.2)
    _say("block forward, wide rows:", w)
    xn = synth.draw_tokens(w, "cuda")
    wr, bias = synth.draw_router(w, "cuda")
    wg, wu, wd = synth.draw_experts(w, "cuda")
    x_res0 = torch.randn(w.T, w.H, generator=torch.Generator().manual_seed(6)).to(w.torch_dtype).cuda()
    desc = zeda.make_desc(w.T, w.H, w.I, w.N, w.Z, w.K, w.dtype)
    ws = torch.empty(zeda.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    nreal = torch.zeros(1, dtype=torch.int32, device="cuda")
    x_res, xn_next = x_res0.clone(), torch.empty_like(xn)
    zeda.zeda_moe_block_forward(desc, xn, x_res, wr, bias, wg, wu, wd, None, EPS, xn_next, nreal, ws)
    torch.cuda.synchronize()
    r = orc.moe_forward(*[synth.to_numpy_f32(v) for v in (xn, wr, bias, wg, wu, wd)], w.N, w.Z, w.K)
    want = x_res0.double().cpu().numpy() + r["out"]
    assert harness.rel_l2(x_res.double().cpu().numpy(), want) < 1e-2
    np.testing.assert_allclose(xn_next.float().cpu().numpy(), orc.rmsnorm(synth.to_numpy_f32(x_res), None, EPS),
                               rtol=6e-3, atol=6e-5)
    too_wide = zeda.make_desc(8, 8192 + 128, 64, 4, 2, 2, "bf16")
    with pytest.raises(zeda.ZedaError) as ei:
        zeda.zeda_moe_block_forward(too_wide, xn, x_res, wr, bias, wg, wu, wd, None, EPS, None, nreal, ws)
    assert ei.value.status == zeda.ZEDA_EUNSUPPORTED


@pytest.mark.parametrize("fused", [False, True])
def test_tiny_fp32_stack_end_to_end(fused):
    # four small fp32 layers: the whole chain against the oracle chain (routing compared where unambiguous)
    w = synth.Workload("tiny_stack", T=96, H=128, I=64, N=8, Z=4, K=2, dtype="f32", seed=900, recipe="zero_bias",
                       x_std=1.0, w_std=0.08, wr_std=0.2, zero_bias=0.1)
    st = MoeStack(w, layers=4)
    x = synth.draw_tokens(w, "cuda")
    ref = x.double().cpu().numpy()
    ids_gpu = []
    if fused:  # no hook in the one-call-per-layer chain: routing is then only checked through the final stream
        out = st.forward(x.clone())
    else:
        out = st.forward(x.clone(), hook=lambda l, s: ids_gpu.append(zeda.ws_views(s.desc, s.ws)["topk_ids"].clone()))
    torch.cuda.synchronize()
    # A token whose routing is ambiguous in some layer may legitimately differ from then on; the chain is
    # token by token (no layer mixes rows), so every other token must follow the oracle chain to the end.
    ever_unsafe = np.zeros(w.T, dtype=bool)
    for l, p in enumerate(st.weights):
        xn = orc.rmsnorm(ref, None, EPS).astype(np.float32)
        a = {k: synth.to_numpy_f32(v) for k, v in p.items()}
        r = orc.moe_forward(xn, a["w_router"], a["router_bias"], a["w_gate"], a["w_up"], a["w_down"], w.N, w.Z, w.K)
        _, _, lg = orc.route(xn, a["w_router"], a["router_bias"], w.N, w.Z, w.K, want_logits=True)
        ever_unsafe |= harness.topk_gaps(lg, w.K) < harness.GAP
        if not fused:
            assert np.array_equal(ids_gpu[l].cpu().numpy()[~ever_unsafe], r["ids"][~ever_unsafe]), f"layer {l}"
        ref = ref + r["out"]
    keep = ~ever_unsafe
    _say("tokens left out of the comparison (near-tie in some layer):", int(ever_unsafe.sum()), "of", w.T)
    assert keep.sum() >= w.T // 2
    got = out.double().cpu().numpy()
    assert harness.rel_l2(got[keep], ref[keep]) < 1e-5
    assert np.max(np.abs(got[keep] - ref[keep])) <= 1e-5 * np.max(np.abs(ref[keep]))
    assert np.isfinite(got).all()


def test_config5_stack_teacher_forced():
    w = synth.CONFIGS["c5_stack_layer"]
    layers = 48
    _say("config 5:", w, "layers", layers)
    st = MoeStack(w, layers)
    x = synth.draw_tokens(w, "cuda")
    check = (0, 1, 23, 47)
    kept = {}

    def hook(l, s):
        if l in check:
            v = zeda.ws_views(s.desc, s.ws)
            kept[l] = (s.xn.clone(), s.y.clone(), v["topk_ids"].clone(), v["expert_offsets"].clone())

    st.forward(x, hook=hook)
    torch.cuda.synchronize()
    nreal = st.num_real.cpu().numpy()
    _say("r_ZE per layer: min %.3f max %.3f mean %.3f" % tuple(f(1 - nreal / (w.T * w.K)) for f in (np.min, np.max, np.mean)))
    assert 0.35 < (1 - nreal / (w.T * w.K)).mean() < 0.65
    rng = np.random.default_rng(5)
    for l in check:
        xn, y, ids, off = kept[l]
        p = st.weights[l]
        a = {k: synth.to_numpy_f32(v) for k, v in p.items()}
        xn_h = synth.to_numpy_f32(xn)
        rid, _, lg = orc.route(xn_h, a["w_router"], a["router_bias"], w.N, w.Z, w.K, want_logits=True)
        safe = harness.topk_gaps(lg, w.K) >= harness.GAP
        ids_h = ids.cpu().numpy()
        assert np.array_equal(ids_h[safe], rid[safe]), f"layer {l}"
        # dispatch is exact for the ids the GPU actually used
        roff, _, _ = orc.dispatch(ids_h, w.N)
        assert np.array_equal(off.cpu().numpy(), roff)
        tok = np.sort(rng.choice(np.flatnonzero(safe), size=1024, replace=False))
        r = orc.moe_forward(xn_h[tok], a["w_router"], a["router_bias"], a["w_gate"], a["w_up"], a["w_down"], w.N, w.Z, w.K)
        rl2, mabs = check_float(w, y.float().cpu().numpy()[tok], r["out"], f"layer {l} output")
        _say(f"layer {l}: {int((~safe).sum())} of {w.T} tokens excluded from the routing comparison; "
             f"sampled output rel-L2 {rl2:.2e} max-abs {mabs:.2e}; r_ZE {1 - nreal[l] / (w.T * w.K):.3f}")
    assert np.isfinite(x.float().cpu().numpy()).all()


def test_config5_fused_chain_teacher_forced():
    # the one-call-per-layer chain at full size: for each checked layer the oracle gets the GPU's own normalised
    # input and stream, and must reproduce the routing, the dispatch, the new stream rows and the next input
    w = synth.CONFIGS["c5_stack_layer"]
    layers = 48
    _say("config 5, fused blocks:", w, "layers", layers)
    st = MoeStack(w, layers, tiled=True)
    x = synth.draw_tokens(w, "cuda")
    check = (0, 1, 23, 47)
    before, after = {}, {}

    def hook(l, s, xs):
        if l - 1 in check:  # layer l-1 has run: its routing tables, the new stream and the next layer's input
            v = zeda.ws_views(s.desc, s.ws)
            after[l - 1] = (xs.clone(), s.xn.clone(), v["topk_ids"].clone(), v["expert_offsets"].clone())
        if l in check:
            before[l] = (xs.clone(), s.xn.clone())

    st.forward(x, hook=hook, fused=True)
    torch.cuda.synchronize()
    nreal = st.num_real.cpu().numpy()
    assert 0.35 < (1 - nreal / (w.T * w.K)).mean() < 0.65
    rng = np.random.default_rng(6)
    for l in check:
        x0, xn = before[l]
        x1, xn1, ids, off = after[l]
        a = {k: synth.to_numpy_f32(v) for k, v in st.weights[l].items() if k in ("w_router", "router_bias")}
        wg, wu, wd = synth.draw_experts(w, "cuda", l)  # the stack holds them tiled: the oracle wants them row-major
        xn_h = synth.to_numpy_f32(xn)
        rid, _, lg = orc.route(xn_h, a["w_router"], a["router_bias"], w.N, w.Z, w.K, want_logits=True)
        safe = harness.topk_gaps(lg, w.K) >= harness.GAP
        ids_h = ids.cpu().numpy()
        assert np.array_equal(ids_h[safe], rid[safe]), f"layer {l}"
        roff, _, _ = orc.dispatch(ids_h, w.N)
        assert np.array_equal(off.cpu().numpy(), roff)
        tok = np.sort(rng.choice(np.flatnonzero(safe), size=1024, replace=False))
        r = orc.moe_forward(xn_h[tok], a["w_router"], a["router_bias"], *[synth.to_numpy_f32(v) for v in (wg, wu, wd)],
                            w.N, w.Z, w.K)
        want = x0.double().cpu().numpy()[tok] + r["out"]
        got = x1.double().cpu().numpy()[tok]
        rl2, mabs = harness.rel_l2(got, want), float(np.max(np.abs(got - want)))
        # the expert arithmetic's tolerance plus the one bf16 rounding of the stream row
        assert rl2 < 1e-2 and mabs <= 2e-2 + 2.0 ** -8 * float(np.max(np.abs(want))), (l, rl2, mabs)
        if l + 1 < layers:
            np.testing.assert_allclose(synth.to_numpy_f32(xn1)[tok], orc.rmsnorm(synth.to_numpy_f32(x1)[tok], None, EPS),
                                       rtol=6e-3, atol=6e-5)
        _say(f"layer {l}: {int((~safe).sum())} of {w.T} tokens excluded from the routing comparison; "
             f"sampled stream rows rel-L2 {rl2:.2e} max-abs {mabs:.2e}; r_ZE {1 - nreal[l] / (w.T * w.K):.3f}")
    assert np.isfinite(x.float().cpu().numpy()).all()


def test_stack_with_tiled_weights_matches_row_major_bit_for_bit():
    # same k order and the same accumulation order in both weight layouts: the chained output is identical
    w = synth.Workload("stack_tiled", T=300, H=256, I=128, N=8, Z=4, K=2, dtype="bf16", seed=91, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.3)
    _say("stack, tiled against row-major:", w)
    x0 = synth.draw_tokens(w, "cuda")
    outs = []
    for tiled in (False, True):
        st = MoeStack(w, layers=3, tiled=tiled)
        outs.append(st.forward(x0.clone()).clone())
        torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    assert np.isfinite(outs[0].float().cpu().numpy()).all()


@pytest.mark.parametrize("fused", [False, True])
def test_stack_token_level_zero_slots(fused):
    # per token, the zero-expert slots summed over the layers (Section 4.1's token-level r_ZE times layers * K): every
    # layer's share is checked against the oracle's count on the ids that layer's router wrote, and the total against
    # the real-slot counts the layers report
    w = synth.Workload("stack_tz", T=150, H=256, I=128, N=8, Z=4, K=3, dtype="bf16", seed=93, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.3)
    _say("stack, token-level zero slots, fused" if fused else "stack, token-level zero slots, three calls per layer", w)
    st = MoeStack(w, layers=4)
    per_layer = []

    def hook(l, stack, *rest):
        # fused: called before layer l, so the ids in the workspace are layer l-1's; unfused: after layer l
        if fused and l == 0:
            return
        torch.cuda.synchronize()
        per_layer.append(orc.token_zero_slots(zeda.ws_views(stack.desc, stack.ws)["topk_ids"].cpu().numpy(), w.N))

    tz = torch.full((w.T,), 123, dtype=torch.int32, device="cuda")
    st.forward(synth.draw_tokens(w, "cuda"), hook=hook, fused=fused, token_zero=tz)
    torch.cuda.synchronize()
    assert len(per_layer) == 4
    got = tz.cpu().numpy()
    assert np.array_equal(got, np.sum(per_layer, axis=0))
    assert int(got.sum()) == 4 * w.T * w.K - int(st.num_real.sum().item())
    assert got.min() >= 0 and got.max() <= 4 * w.K
