"""GPU parity on seeded random layer shapes: whole-layer forward through the C ABI against the CPU oracle, over a
spread of token counts, widths, router sizes, top-K values and gate normalisations inside the library's documented
limits, alternating the two expert-weight layouts.  The fixed lists of the other parity tests pick their shapes by
hand; this one is there for the combinations nobody thought of.  Expert weights are drawn with std 0.8/sqrt(H), so that outputs stay
O(1) at every width and the absolute bf16 tolerance means the same thing in every case."""
import random

import pytest

from oracle import harness
from paper_2605_18643_amd import synth, zeda

pytestmark = pytest.mark.gpu

from gpu_util import full_parity  # noqa: E402

CASES = 64
TOKENS = [1, 2, 7, 31, 33, 64, 65, 127, 129, 255, 300, 511, 777, 1025, 2049, 4097]


def draw_case(rng: random.Random, i: int) -> dict:
    N = rng.choice([1, 2, 3, 5, 8, 13, 31, 32, 33, 64, 100])
    Z = rng.choice([0, 0, 1, 2, 4, 7, 16, 32])
    K = rng.randint(1, min(16, N + Z))
    H = 128 * rng.choice([1, 2, 3, 4, 6, 8])
    I = 64 * rng.choice([1, 2, 3, 5, 8, 12])
    T = rng.choice(TOKENS)
    if T * K * H * I > 1.5e10 or N * H * I > 3e7:  # keep the oracle's share of a case to about a second
        T = min(T, 300)
    return dict(T=T, H=H, I=I, N=N, Z=Z, K=K, seed=1000 + i, zero_bias=rng.choice([0.0, 0.2, 0.5, 1.0]))


@pytest.mark.parametrize("block", range(4))
def test_random_shapes_match_oracle(block):
    rng = random.Random(20260518 + block)
    per_block = CASES // 4
    for j in range(per_block):
        i = block * per_block + j
        cfg = draw_case(rng, i)
        tiled = bool(i & 1)
        gate_norm = rng.choice([zeda.GATE_TOPK_NORM, zeda.GATE_SOFTMAX, zeda.GATE_REAL_RENORM])
        print("random shape", i, cfg, "tiled" if tiled else "row_major", "gate_norm", gate_norm, flush=True)
        w = synth.Workload("random", dtype="bf16", recipe="zero_bias", x_std=1.0, w_std=0.8 / cfg["H"] ** 0.5,
                           wr_std=0.05, **cfg)
        L = harness.gapped_layer(w, "cuda", gate_norm=gate_norm)
        full_parity(w, L, gate_norm, tiled=tiled)
