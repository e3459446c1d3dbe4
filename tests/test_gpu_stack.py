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


def test_tiny_fp32_stack_end_to_end():
    # four small fp32 layers: the whole chain against the oracle chain (routing compared where unambiguous)
    w = synth.Workload("tiny_stack", T=96, H=128, I=64, N=8, Z=4, K=2, dtype="f32", seed=900, recipe="zero_bias",
                       x_std=1.0, w_std=0.08, wr_std=0.2, zero_bias=0.1)
    st = MoeStack(w, layers=4)
    x = synth.draw_tokens(w, "cuda")
    ref = x.double().cpu().numpy()
    ids_gpu = []
    out = st.forward(x.clone(), hook=lambda l, s: ids_gpu.append(zeda.ws_views(s.desc, s.ws)["topk_ids"].clone()))
    torch.cuda.synchronize()
    excluded = 0
    for l, p in enumerate(st.weights):
        xn = orc.rmsnorm(ref, None, EPS).astype(np.float32)
        a = {k: synth.to_numpy_f32(v) for k, v in p.items()}
        r = orc.moe_forward(xn, a["w_router"], a["router_bias"], a["w_gate"], a["w_up"], a["w_down"], w.N, w.Z, w.K)
        _, _, lg = orc.route(xn, a["w_router"], a["router_bias"], w.N, w.Z, w.K, want_logits=True)
        safe = harness.topk_gaps(lg, w.K) >= harness.GAP
        excluded += int((~safe).sum())
        assert np.array_equal(ids_gpu[l].cpu().numpy()[safe], r["ids"][safe])
        ref = ref + r["out"]
    _say("tokens excluded from the routing comparison over 4 layers:", excluded)
    got = out.double().cpu().numpy()
    # a token whose routing is ambiguous may legitimately differ afterwards: compare the others
    assert harness.rel_l2(got, ref) < 1e-3 or excluded > 0
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
        tok = np.sort(rng.choice(np.flatnonzero(safe), size=96, replace=False))
        r = orc.moe_forward(xn_h[tok], a["w_router"], a["router_bias"], a["w_gate"], a["w_up"], a["w_down"], w.N, w.Z, w.K)
        rl2, mabs = check_float(w, y.float().cpu().numpy()[tok], r["out"], f"layer {l} output")
        _say(f"layer {l}: {int((~safe).sum())} of {w.T} tokens excluded from the routing comparison; "
             f"sampled output rel-L2 {rl2:.2e} max-abs {mabs:.2e}; r_ZE {1 - nreal[l] / (w.T * w.K):.3f}")
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
