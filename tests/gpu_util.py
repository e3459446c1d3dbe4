"""Helpers of the GPU parity tests: run the HIP library through its C ABI, collect every intermediate
result, and compare with the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth, zeda

# bf16 weights with fp32 accumulation: max-abs 2e-2 and relative L2 1e-2; fp32: 1e-5 relative (norm-wise
# and max-abs relative to the largest reference magnitude).
BF16_MAX_ABS, BF16_REL_L2, F32_REL = 2e-2, 1e-2, 1e-5


def desc_of(w: synth.Workload, gate_norm=zeda.GATE_TOPK_NORM, weight_layout=zeda.WEIGHTS_ROW_MAJOR, copy_expert=False):
    return zeda.make_desc(w.T, w.H, w.I, w.N, w.Z, w.K, w.dtype, gate_norm, weight_layout,
                          zeda.EXPERT_COPY if copy_expert else zeda.EXPERT_ZERO)


def tiled_layer(w: synth.Workload, L):
    """The same layer with its expert weights repacked by zeda_pack_expert_weights."""
    Lt = dict(L)
    Lt["w_gate"], Lt["w_up"], Lt["w_down"] = zeda.zeda_pack_expert_weights(desc_of(w), L["w_gate"], L["w_up"], L["w_down"])
    return Lt


def forward(w: synth.Workload, L, gate_norm=zeda.GATE_TOPK_NORM, tiled=False, copy_expert=False):
    """zeda_moe_forward on device tensors L; returns host copies of the output and of all intermediates.
    tiled: repack the expert weights first and run the tiled-layout path.  copy_expert: Appendix B's variant."""
    d = desc_of(w, gate_norm, zeda.WEIGHTS_TILED if tiled else zeda.WEIGHTS_ROW_MAJOR, copy_expert)
    if tiled:
        L = tiled_layer(w, L)
    ws = torch.empty(zeda.workspace_bytes(d), dtype=torch.uint8, device="cuda")
    out = torch.full((w.T, w.H), float("nan"), dtype=w.torch_dtype, device="cuda")
    nreal = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    zeda.zeda_moe_forward(d, L["x"], L["w_router"], L["router_bias"], L["w_gate"], L["w_up"], L["w_down"], out, nreal, ws)
    torch.cuda.synchronize()
    v = zeda.ws_views(d, ws)
    res = {k: t.detach().cpu() for k, t in v.items()}
    res["out"] = out.cpu()
    res["num_real_out"] = int(nreal.item())
    return res


def gate_rtol(w, max_logit: float) -> float:
    """Relative tolerance of a routing weight.  2e-5 covers fp32 exp, sum and division against fp64.  On top of that
    the GPU accumulates a logit in fp32 over H products (the oracle in fp64): an absolute error of about
    sqrt(H) * 2^-24 * |logit|, and a weight's relative error is the error of a difference of two logits."""
    return 2e-5 + 2.0 * np.sqrt(w.H) * 2.0 ** -24 * max_logit if w.dtype == "bf16" else 2e-5


def check_routing(w, res, ref_ids, ref_gates, max_logit: float = 1.0):
    ids = res["topk_ids"].numpy()
    assert np.array_equal(ids, ref_ids), f"{int((ids != ref_ids).any(axis=1).sum())} tokens routed differently"
    np.testing.assert_allclose(res["topk_gates"].numpy().astype(np.float64), ref_gates, rtol=gate_rtol(w, max_logit), atol=1e-7)


def check_dispatch(w, res, ref_ids):
    off, ss, s2r = orc.dispatch(ref_ids, w.N)
    R = int(off[w.N])
    assert np.array_equal(res["expert_offsets"].numpy(), off)
    assert int(res["num_real"].item()) == R and res["num_real_out"] == R
    assert np.array_equal(res["sorted_slot"].numpy()[:R], ss[:R])
    assert np.array_equal(res["slot_to_row"].numpy(), s2r)
    return off, ss, s2r, R


def check_float(w, got: np.ndarray, ref: np.ndarray, what: str):
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    rl2, mabs = harness.rel_l2(got, ref), harness.max_abs(got, ref)
    if w.dtype == "bf16":
        assert rl2 <= BF16_REL_L2 and mabs <= BF16_MAX_ABS, f"{what}: rel-L2 {rl2:.3e}, max-abs {mabs:.3e}"
    else:
        scale = float(np.max(np.abs(ref))) if ref.size else 0.0
        assert rl2 <= F32_REL and mabs <= F32_REL * max(scale, 1e-30), f"{what}: rel-L2 {rl2:.3e}, max-abs {mabs:.3e} (scale {scale:.3e})"
    return rl2, mabs


def full_parity(w: synth.Workload, L, gate_norm=zeda.GATE_TOPK_NORM, tokens=None, tiled=False, copy_expert=False):
    """Whole-layer parity.  With `tokens` (sorted indices, or a function of the reference ids, offsets and
    slot_to_row that returns them) the oracle's expert arithmetic runs on those rows only; routing and dispatch
    are always checked on every token."""
    a = harness.to_arrays(L)
    res = forward(w, L, gate_norm, tiled, copy_expert)
    ref_ids, ref_gates, logits = orc.route(a["x"], a["w_router"], a["router_bias"], w.N, w.Z, w.K, gate_norm, want_logits=True)
    check_routing(w, res, ref_ids, ref_gates, float(np.max(np.abs(logits))) if logits.size else 1.0)
    off, ss, s2r, R = check_dispatch(w, res, ref_ids)
    if callable(tokens):
        tokens = tokens(ref_ids, off, s2r)
    ref = harness.oracle_forward(w, a, gate_norm, copy_expert=copy_expert, tokens=tokens, want_y_slot=True)
    tok = np.arange(w.T) if tokens is None else np.asarray(tokens)
    assert np.array_equal(ref["ids"], ref_ids[tok])
    out = res["out"].float().numpy()[tok]
    stats = {"R": R, "r_ze": 1.0 - R / max(1, w.T * w.K), "nonempty": int((np.diff(off) > 0).sum())}
    stats["out"] = check_float(w, out, ref["out"], "out")
    # all-zero tokens are exact zeros (with copy experts they carry the copy term instead)
    allzero = (ref_ids[tok] >= w.N).all(axis=1)
    assert copy_expert or not out[allzero].any()
    # per-slot expert outputs, expert-sorted rows of the sampled tokens
    slots = (tok[:, None] * w.K + np.arange(w.K)[None, :]).ravel()
    rows = s2r[slots]
    real = rows >= 0
    if real.any():
        y = res["y_slot"].float().numpy()[rows[real]]
        stats["y_slot"] = check_float(w, y, ref["y_slot"][real], "y_slot")
    return res, stats
