"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
Routing and dispatch are checked on every token; the oracle's expert arithmetic runs on all tokens where it
finishes in seconds (configs 2 and 3) and on a sample of tokens at T=16384 (config 4)."""
import numpy as np
import pytest
import torch

from oracle import harness
from paper_2605_18643_amd import synth

pytestmark = pytest.mark.gpu

from gpu_util import full_parity  # noqa: E402


def _say(*a):
    print(*a, flush=True)


# bench.py times the tiled weight layout; the row-major layout is the other one the library accepts
LAYOUTS = pytest.mark.parametrize("tiled", [True, False], ids=["tiled", "row_major"])


@LAYOUTS
def test_config3_decode_full(tiled):
    w = synth.CONFIGS["c3_qwen_decode"]
    _say("config 3", w, "tiled" if tiled else "row-major")
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=tiled)
    _say(st)
    assert 0.35 < st["r_ze"] < 0.65 and st["nonempty"] < w.N


@LAYOUTS
def test_config2_prefill_full(tiled):
    w = synth.CONFIGS["c2_qwen_prefill"]
    _say("config 2", w, "tiled" if tiled else "row-major")
    L = harness.gapped_layer(w, "cuda")
    _say("redrawn tokens:", L["redrawn"])
    res, st = full_parity(w, L, tiled=tiled)
    _say(st)
    assert abs(st["r_ze"] - 0.5) < 0.02 and st["nonempty"] == w.N


def test_config2_static_layer_z0():
    # the Z=0 layer the speedup is quoted against: same weights, router restricted to the normal experts
    w = synth.CONFIGS["c2_qwen_prefill"].with_(Z=0, recipe="plain", T=1024)
    _say("config 2 at Z=0", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tokens=np.arange(0, w.T, 4))
    _say(st)
    assert st["R"] == w.T * w.K


def test_config2_static_layer_z0_full_size_tiled():
    # the same at T=4096 in the layout bench.py times: the experts average exactly 256 rows, half of them a few more,
    # which is where the GEMM kernel switches to its 320-row token tile
    w = synth.CONFIGS["c2_qwen_prefill"].with_(Z=0, recipe="plain")
    _say("config 2 at Z=0, full size, tiled", w)
    L = harness.gapped_layer(w, "cuda")
    tokens = np.sort(np.random.default_rng(1).choice(w.T, size=256, replace=False))
    res, st = full_parity(w, L, tokens=tokens, tiled=True)
    load = np.diff(res["expert_offsets"].numpy())
    _say(st, "rows per expert: min", load.min(), "max", load.max(), "above 256:", int((load > 256).sum()))
    assert st["R"] == w.T * w.K and (load > 256).sum() > w.N // 4 and load.max() <= 320


@LAYOUTS
def test_config4_hetero_prefill_sampled(tiled):
    w = synth.CONFIGS["c4_hetero_prefill"]
    _say("config 4", w, "tiled" if tiled else "row-major")
    L = harness.gapped_layer(w, "cuda")
    _say("redrawn tokens:", L["redrawn"])
    tokens = np.sort(np.random.default_rng(0).choice(w.T, size=192, replace=False))
    res, st = full_parity(w, L, tokens=tokens, tiled=tiled)
    _say(st)
    zc = (res["topk_ids"].numpy() >= w.N).sum(axis=1)
    hist = np.bincount(zc, minlength=9) / w.T
    assert abs(hist[6:9].sum() - 0.6) < 0.02 and abs(hist[0:2].sum() - 0.4) < 0.02
    load = np.diff(res["expert_offsets"].numpy())
    _say("rows per expert: max", load.max(), "min", load.min(), "empty", int((load == 0).sum()))
    assert load.max() > 8 * load.mean()


def test_maximum_slot_count():
    # T*K just under the 2^24 limit of the interface (16.7 M slots, several GB of intermediates): the indices,
    # offsets and the permutation are checked on every slot, the arithmetic on sampled tokens
    w = synth.Workload("max_slots", T=2_097_000, H=128, I=64, N=6, Z=2, K=8, dtype="bf16", seed=7, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.1)
    assert w.T * w.K < (1 << 24)
    _say("maximum slot count", w)
    L = harness.gapped_layer(w, "cuda")
    tokens = np.sort(np.random.default_rng(3).choice(w.T, size=256, replace=False))
    res, st = full_parity(w, L, tokens=tokens, tiled=True)
    _say(st)
    assert st["R"] > (1 << 23)
