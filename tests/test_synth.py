"""The synthetic-input generator: reproducible bits, the stated distributions, and the routing
statistics each workload recipe promises (measured with the oracle's router). No GPU."""
import numpy as np
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth


def test_generator_is_reproducible_and_chunk_independent():
    a = synth.normal_flat(100_000, synth.make_key(3, 1), 0.02, "cpu")
    b = synth.normal_flat(100_000, synth.make_key(3, 1), 0.02, "cpu")
    assert torch.equal(a, b)
    old = synth._CHUNK_CPU
    try:
        synth._CHUNK_CPU = 777
        c = synth.normal_flat(100_000, synth.make_key(3, 1), 0.02, "cpu")
    finally:
        synth._CHUNK_CPU = old
    assert torch.equal(a, c)
    d = synth.normal_flat(1000, synth.make_key(3, 1), 0.02, "cpu", start=5000)
    assert torch.equal(d, a[5000:6000])
    assert not torch.equal(a, synth.normal_flat(100_000, synth.make_key(3, 2), 0.02, "cpu"))


def test_hash_matches_python_integers():
    idx = torch.tensor([0, 1, 2, 12345, (1 << 32) - 1, (1 << 32) + 7, (1 << 40) + 3], dtype=torch.int64)
    key = synth.make_key(9, 9)
    got = synth.hash_u32(idx, key).tolist()
    k2 = synth._fmix32_py(key ^ 0x5BD1E995)
    for i, g in zip(idx.tolist(), got):
        lo, hi = i & 0xFFFFFFFF, i >> 32
        h = synth._fmix32_py(lo ^ key)
        h = synth._fmix32_py(((h + k2) & 0xFFFFFFFF) ^ ((hi * 0x9E3779B1) & 0xFFFFFFFF))
        assert g == h


def test_normal_moments():
    z = synth.normal_flat(1 << 21, synth.make_key(1, 2, 3), 1.0, "cpu").double().numpy()
    assert abs(z.mean()) < 3e-3 and abs(z.std() - 1) < 3e-3
    assert abs((z ** 3).mean()) < 1e-2 and abs((z ** 4).mean() - 3) < 3e-2
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 3e-3


def test_row_redraw_moves_only_that_row():
    w = synth.CONFIGS["c1_tiny_f32"]
    a = synth.draw_tokens(w)
    att = torch.zeros(w.T, dtype=torch.int64)
    att[5] = 1
    b = synth.draw_tokens(w, attempt=att)
    same = (a == b).all(dim=1)
    assert not same[5] and same[torch.arange(w.T) != 5].all()


def test_gapped_layer_has_the_gap():
    w = synth.CONFIGS["c1_tiny_f32"]
    L = harness.gapped_layer(w)
    a = harness.to_arrays(L)
    _, _, logits = orc.route(a["x"], a["w_router"], None, w.N, w.Z, w.K, want_logits=True)
    assert harness.topk_gaps(logits, w.K).min() >= harness.GAP
    assert L["redrawn"] > 0  # config 1's logits are narrow: some rows must have moved


def test_zero_bias_recipe_gives_half_zero_slots():
    # config 2: on average ~4 of the 8 selected slots are zero experts, real load roughly uniform
    w = synth.CONFIGS["c2_qwen_prefill"]
    wr, bias = synth.draw_router(w)
    x = synth.draw_tokens(w)
    ids, _ = orc.route(synth.to_numpy_f32(x), synth.to_numpy_f32(wr), synth.to_numpy_f32(bias), w.N, w.Z, w.K)
    assert abs((ids >= w.N).sum(axis=1).mean() - 4.0) <= 0.05
    load = np.bincount(ids[ids < w.N], minlength=w.N)
    assert load.min() > 0.6 * load.mean() and load.max() < 1.4 * load.mean()


def test_planted_recipe_matches_its_plan():
    # config 4 (fewer tokens): 60 % easy tokens with 6-8 zero slots, 40 % hard with 0-1, Zipf(1.1) popularity
    w = synth.CONFIGS["c4_hetero_prefill"].with_(T=4096)
    wr, bias = synth.draw_router(w)
    assert bias is None
    x = synth.draw_tokens(w)
    ids, _ = orc.route(synth.to_numpy_f32(x), synth.to_numpy_f32(wr), None, w.N, w.Z, w.K)
    plan = synth.planted_plan(w)
    planted = np.where(plan["planted"])[1].reshape(w.T, w.K)
    assert np.array_equal(np.sort(ids, axis=1), np.sort(planted, axis=1))
    zc = (ids >= w.N).sum(axis=1)
    hist = np.bincount(zc, minlength=9) / w.T
    assert abs(hist[6:9].sum() - 0.6) < 0.03 and abs(hist[0:2].sum() - 0.4) < 0.03 and hist[2:6].sum() == 0
    # popularity: the most popular expert is far above the mean load and the tail is far below
    load = np.bincount(ids[ids < w.N], minlength=w.N)
    assert load.max() > 8 * load.mean() and np.sort(load)[:16].mean() < 0.25 * load.mean()
    # the drawn popularity is the Zipf law itself
    p = np.sort(plan["popularity"])[::-1]
    np.testing.assert_allclose(p / p[0], np.arange(1, w.N + 1) ** -1.1, rtol=1e-12)
