"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
Routing and dispatch are checked on every token, and so is the expert arithmetic of configs 2, 3 and 4 (the oracle
needs seconds for them); the T=8192 static layer and the 16.7 M-slot case compare sampled tokens."""
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
    res, st = full_parity(w, L, tiled=True)  # every token
    load = np.diff(res["expert_offsets"].numpy())
    _say(st, "rows per expert: min", load.min(), "max", load.max(), "above 256:", int((load > 256).sum()))
    assert st["R"] == w.T * w.K and (load > 256).sum() > w.N // 4 and load.max() <= 320


def test_config5_layer_static_z0_at_8192_tokens():
    # one layer of the Z=0 leg of the 48-layer stack (the baseline its speed-up is quoted against): T=8192, every
    # slot real, experts at about 512 rows, i.e. two or three token tiles each.  Routing and dispatch on every token;
    # the arithmetic on 1024 tokens, half of them chosen among those with a slot in a row past the 512th of its expert
    w = synth.CONFIGS["c5_stack_layer"].with_(Z=0, recipe="plain")
    _say("config 5 layer at Z=0", w)
    L = harness.gapped_layer(w, "cuda")

    def sample(ref_ids, off, s2r):
        rng = np.random.default_rng(2)
        within = s2r.reshape(w.T, w.K) - off[ref_ids]  # row of every slot inside its expert
        late = np.flatnonzero((within >= 512).any(axis=1))
        assert late.size >= 512
        pick = set(rng.choice(late, size=512, replace=False).tolist())
        pick |= set(rng.choice(w.T, size=512, replace=False).tolist())
        return np.array(sorted(pick))

    res, st = full_parity(w, L, tokens=sample, tiled=True)
    load = np.diff(res["expert_offsets"].numpy())
    _say(st, "rows per expert: min", load.min(), "max", load.max(), "above 512:", int((load > 512).sum()))
    assert st["R"] == w.T * w.K and (load > 512).sum() > w.N // 4


def _planted_loads_plan(T, K, N, Z, loads):
    """A routing plan (bool [T, N+Z], K entries per row) in which normal expert e gets exactly loads[e] slots and the
    remaining slots go to zero experts.  The T*K expert labels, sorted, are dealt out column by column (slot rank j
    of token t takes label j*T + t), so the K labels of a token are distinct as long as no expert has more than T."""
    loads = np.asarray(loads, dtype=np.int64)
    n_zero = T * K - int(loads.sum())
    assert loads.size == N and loads.max() <= T and 0 <= n_zero <= T * min(Z, 1) * K
    labels = np.concatenate([np.repeat(np.arange(N), loads), N + (np.arange(n_zero) // T) % max(Z, 1)])
    assert labels.size == T * K
    plan = np.zeros((T, N + Z), dtype=bool)
    for j in range(K):
        plan[np.arange(T), labels[j * T:(j + 1) * T]] = True
    assert (plan.sum(axis=1) == K).all()
    return plan


@LAYOUTS
def test_expert_loads_around_the_token_tile_boundaries(tiled):
    # prescribed rows per expert, each in a window where the tiling of an expert's rows changes: just above and at
    # the end of (512, 640], (768, 960], (1024, 1280], just above 1280, and small ones next to them; every token
    # is compared.  Shape of the benchmark layers (H=2048, I=768); T*K/N = 1000 rows per expert if all were real.
    loads = [513, 640, 769, 960, 1025, 1280, 1281, 1340, 64, 1]
    T, K, N, Z = 5000, 2, 10, 4
    w = synth.Workload("tile_windows", T=T, H=2048, I=768, N=N, Z=Z, K=K, dtype="bf16", seed=31, recipe="planted")
    _say("loads at tile boundaries", w, loads, "tiled" if tiled else "row-major")
    plan = _planted_loads_plan(T, K, N, Z, loads)
    L = harness.gapped_layer(w, "cuda", planted=plan)
    res, st = full_parity(w, L, tiled=tiled)
    got = np.diff(res["expert_offsets"].numpy())
    _say(st, "rows per expert:", got.tolist())
    assert got.tolist() == loads


@LAYOUTS
def test_config4_hetero_prefill_full(tiled):
    w = synth.CONFIGS["c4_hetero_prefill"]
    _say("config 4", w, "tiled" if tiled else "row-major")
    L = harness.gapped_layer(w, "cuda")
    _say("redrawn tokens:", L["redrawn"])
    res, st = full_parity(w, L, tiled=tiled)  # every token: a 7804-row expert next to 68-row ones
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
