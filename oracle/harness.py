"""Oracle-side helpers shared by the tests, the smoke check and the CPU-baseline leg of the benchmark.

TEST INFRASTRUCTURE ONLY (never imported by the product package).  Everything numeric here goes
through oracle/zeda_oracle.c; this file only draws inputs (paper_2605_18643_amd.synth), asks the
oracle about them and compares arrays.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from paper_2605_18643_amd import synth
from . import zeda_oracle as orc

GAP = 1e-3  # minimum spacing between neighbouring fp32 logits among a token's top K+1


def topk_gaps(logits: np.ndarray, K: int) -> np.ndarray:
    """Smallest spacing between neighbouring values among each token's K+1 largest fp32 logits
    (K largest if there are only K candidates)."""
    l32 = logits.astype(np.float32)
    kk = min(K + 1, l32.shape[1])
    top = -np.sort(-l32, axis=1)[:, :kk].astype(np.float64)
    if kk < 2:
        return np.full(l32.shape[0], np.inf)
    return np.min(top[:, :-1] - top[:, 1:], axis=1)


def gapped_layer(w: synth.Workload, device="cpu", layer: int = 0, max_rounds: int = 64,
                 gate_norm: int = orc.GATE_TOPK_NORM, planted: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Draw a layer whose routing is unambiguous: rows of x whose top K+1 fp32 logits (oracle, double
    accumulation, rounded once) have a neighbouring pair closer than GAP are re-drawn with the next
    attempt counter until none is left.  Returns the tensors of synth.make_layer plus `attempt`,
    `redrawn` (number of tokens moved at least once).  planted: explicit routing plan of the "planted" recipe
    (see synth.draw_tokens)."""
    attempt = torch.zeros(w.T, dtype=torch.int64)
    wr_t, bias_t = synth.draw_router(w, "cpu", layer)
    wr = synth.to_numpy_f32(wr_t)
    bias = synth.to_numpy_f32(bias_t)
    for _ in range(max_rounds):
        x = synth.to_numpy_f32(synth.draw_tokens(w, "cpu", attempt, layer, planted))
        _, _, logits = orc.route(x, wr, bias, w.N, w.Z, w.K, gate_norm, want_logits=True)
        bad = topk_gaps(logits, w.K) < GAP
        if not bad.any():
            break
        attempt[torch.from_numpy(bad)] += 1
    else:
        raise RuntimeError("gap enforcement did not converge")
    out = synth.make_layer(w, device, attempt, layer, planted)
    out["attempt"] = attempt
    out["redrawn"] = int((attempt > 0).sum())
    return out


def to_arrays(layer: Dict[str, object]) -> Dict[str, Optional[np.ndarray]]:
    """Host float32 copies (exact) of a layer's tensors for the oracle."""
    keys = ("x", "w_router", "router_bias", "w_gate", "w_up", "w_down")
    return {k: synth.to_numpy_f32(layer.get(k)) for k in keys}


def oracle_forward(w: synth.Workload, arrays: Dict[str, Optional[np.ndarray]], gate_norm: int = orc.GATE_TOPK_NORM,
                   copy_expert: bool = False, tokens: Optional[np.ndarray] = None, want_y_slot: bool = False):
    """Run the oracle on all tokens, or on the rows listed in `tokens`."""
    x = arrays["x"] if tokens is None else np.ascontiguousarray(arrays["x"][tokens])
    return orc.moe_forward(x, arrays["w_router"], arrays["router_bias"], arrays["w_gate"], arrays["w_up"],
                           arrays["w_down"], w.N, w.Z, w.K, gate_norm, copy_expert, want_y_slot)


def rel_l2(a: np.ndarray, ref: np.ndarray) -> float:
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.linalg.norm((a - ref).ravel())
    n = np.linalg.norm(ref.ravel())
    return float(d / n) if n > 0 else float(d)


def max_abs(a: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(ref, dtype=np.float64)))) if a.size else 0.0
