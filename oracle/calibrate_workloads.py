"""Finds the zero-expert logit bias of the "zero_bias" workloads (run once; the value is pasted into
paper_2605_18643_amd/synth.py as QWEN_ZERO_BIAS).  Calls only the oracle and the input generator.

    python -m oracle.calibrate_workloads

Bisection on beta until the mean number of zero-expert slots per token, as routed by the oracle on
T=8192 tokens of the layer, is K/2 (Qwen3 shape N=128, Z=32, K=8, H=2048: 4.0 of 8); the same for the
other "zero_bias" layer shapes in synth.CONFIGS.
"""
from __future__ import annotations

import numpy as np

from paper_2605_18643_amd import synth
from . import zeda_oracle as orc


def mean_zero_slots(w: synth.Workload, beta: float, x, wr) -> float:
    bias = np.zeros(w.NE, dtype=np.float32)
    bias[w.N:] = beta
    ids, _ = orc.route(x, wr, bias, w.N, w.Z, w.K)
    return float((ids >= w.N).sum(axis=1).mean())


def calibrate(w: synth.Workload) -> float:
    """beta for which half of the K slots of w's layer land on zero experts (T=8192 tokens, seed 12345)."""
    w = w.with_(T=8192, seed=12345)
    wr_t, _ = synth.draw_router(w)
    x = synth.to_numpy_f32(synth.draw_tokens(w))
    wr = synth.to_numpy_f32(wr_t)
    lo, hi = -3.0, 3.0
    for _ in range(26):
        mid = 0.5 * (lo + hi)
        if mean_zero_slots(w, mid, x, wr) < 0.5 * w.K:
            lo = mid
        else:
            hi = mid
    beta = round(0.5 * (lo + hi), 4)
    print(f"{w.name}: N={w.N} Z={w.Z} K={w.K} H={w.H}: beta = {beta}, mean zero slots = {mean_zero_slots(w, beta, x, wr):.3f}")
    return beta


def main() -> None:
    calibrate(synth.CONFIGS["c2_qwen_prefill"])
    for name in ("c2_qwen_prefill", "c3_qwen_decode", "c5_stack_layer"):
        c = synth.CONFIGS[name]
        wr_c, _ = synth.draw_router(c)
        xc = synth.to_numpy_f32(synth.draw_tokens(c))
        print(name, "mean zero slots at its beta:", mean_zero_slots(c, c.zero_bias, xc, synth.to_numpy_f32(wr_c)))
    # the further workloads: the paper's own N_Z = 64 on the Qwen3 shape, and a GLM-4.7-Flash-like router
    for name in ("n1_qwen_nz64_prefill", "n1_glm_like_prefill"):
        calibrate(synth.CONFIGS[name])


if __name__ == "__main__":
    main()
