"""Finds the zero-expert logit bias of the "zero_bias" workloads (run once; the value is pasted into
paper_2605_18643_amd/synth.py as QWEN_ZERO_BIAS).  Calls only the oracle and the input generator.

    python -m oracle.calibrate_workloads

Bisection on beta until the mean number of zero-expert slots per token, as routed by the oracle on
T=8192 tokens of the Qwen3-shaped layer (N=128, Z=32, K=8, H=2048), is 4.0 of 8.
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


def main() -> None:
    w = synth.CONFIGS["c2_qwen_prefill"].with_(T=8192, seed=12345)
    wr_t, _ = synth.draw_router(w)
    x = synth.to_numpy_f32(synth.draw_tokens(w))
    wr = synth.to_numpy_f32(wr_t)
    lo, hi = 0.0, 3.0
    for _ in range(24):
        mid = 0.5 * (lo + hi)
        if mean_zero_slots(w, mid, x, wr) < 0.5 * w.K:
            lo = mid
        else:
            hi = mid
    beta = round(0.5 * (lo + hi), 4)
    print("beta =", beta, "mean zero slots =", mean_zero_slots(w, beta, x, wr))
    for name in ("c2_qwen_prefill", "c3_qwen_decode", "c5_stack_layer"):
        c = synth.CONFIGS[name]
        wr_c, _ = synth.draw_router(c)
        xc = synth.to_numpy_f32(synth.draw_tokens(c))
        print(name, "mean zero slots at beta:", mean_zero_slots(c, beta, xc, synth.to_numpy_f32(wr_c)))


if __name__ == "__main__":
    main()
