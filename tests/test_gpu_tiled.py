"""The tiled expert-weight layout: the packing kernel against the layout written out in numpy, and whole-layer
parity with the CPU oracle (which always sees the row-major weights) through the tiled-layout GEMM path."""
import numpy as np
import pytest
import torch

from oracle import harness
from paper_2605_18643_amd import synth, zeda

pytestmark = pytest.mark.gpu

from gpu_util import desc_of, forward, full_parity  # noqa: E402


def _say(*a):
    print(*a, flush=True)


def tiled_reference(w: np.ndarray) -> np.ndarray:
    """include/zeda.h, zeda_pack_expert_weights: [mats, F, Kd] -> blocks (rb, kb) of 32 rows x 32 columns, rb
    fastest; inside a block 32 rows of four 8-element pieces, piece p of row r at position p ^ ((r >> 2) & 3)."""
    mats, F, Kd = w.shape
    b = w.reshape(mats, F // 32, 32, Kd // 32, 4, 8).transpose(0, 3, 1, 2, 4, 5)  # mats, kb, rb, r, p, 8
    out = np.empty_like(b)
    for r in range(32):
        for p in range(4):
            out[:, :, :, r, p ^ ((r >> 2) & 3), :] = b[:, :, :, r, p, :]
    return out.reshape(mats, F, Kd)


def test_pack_matches_layout_definition():
    w = synth.Workload("pack", T=8, H=256, I=192, N=5, Z=3, K=2, dtype="bf16", seed=71, recipe="plain")
    _say("pack", w)
    g = torch.Generator().manual_seed(5)
    # distinct bf16 bit patterns, so that any misplaced element shows
    tens = [torch.randint(0, 1 << 15, shape, generator=g, dtype=torch.int16).cuda().view(torch.bfloat16)
            for shape in ((w.N, w.I, w.H), (w.N, w.I, w.H), (w.N, w.H, w.I))]
    d = desc_of(w)
    got = zeda.zeda_pack_expert_weights(d, *tens)
    torch.cuda.synchronize()
    for t, o in zip(tens, got):
        ref = tiled_reference(t.view(torch.int16).cpu().numpy())
        assert np.array_equal(o.view(torch.int16).cpu().numpy(), ref)
    # any subset may be packed alone
    only_down = zeda.zeda_pack_expert_weights(d, None, None, tens[2])
    assert only_down[0] is None and only_down[1] is None and torch.equal(only_down[2].view(torch.int16), got[2].view(torch.int16))


def test_pack_rejects_fp32_and_overlap():
    w = synth.Workload("pack_bad", T=8, H=128, I=64, N=2, Z=0, K=1, dtype="f32", seed=72, recipe="plain")
    x = torch.zeros((w.N, w.I, w.H), dtype=torch.float32, device="cuda")
    with pytest.raises(zeda.ZedaError) as e:
        zeda.zeda_pack_expert_weights(desc_of(w), x, None, None)
    assert e.value.status == zeda.ZEDA_EUNSUPPORTED
    wb = w.with_(dtype="bf16")
    xb = torch.zeros((wb.N, wb.I, wb.H), dtype=torch.bfloat16, device="cuda")
    rc = zeda.lib().zeda_pack_expert_weights(__import__("ctypes").byref(desc_of(wb)), xb.data_ptr(), None, None, xb.data_ptr(), None,
                                             None, None)
    assert rc == zeda.ZEDA_EINVAL


TILED_CASES = [
    # several token tiles per expert with a ragged tail (wide tile configuration)
    dict(T=1000, H=256, I=256, N=6, Z=4, K=3, seed=81, zero_bias=0.3),
    # widths that only the narrow tile configuration divides
    dict(T=600, H=384, I=192, N=10, Z=6, K=4, seed=82, zero_bias=0.4),
    # decode-sized batches
    dict(T=64, H=256, I=128, N=12, Z=4, K=4, seed=83, zero_bias=0.4),
    dict(T=3, H=256, I=128, N=12, Z=4, K=4, seed=84, zero_bias=0.4),
    # static layer, top-1
    dict(T=257, H=128, I=64, N=5, Z=0, K=1, seed=85, zero_bias=0.0),
]


@pytest.mark.parametrize("cfg", TILED_CASES, ids=lambda c: "T%d_H%d_I%d_N%d_Z%d_K%d" % (c["T"], c["H"], c["I"], c["N"], c["Z"], c["K"]))
def test_small_layers_tiled(cfg):
    w = synth.Workload("small_tiled", dtype="bf16", recipe="zero_bias", x_std=1.0, w_std=0.05, wr_std=0.05, **cfg)
    _say("tiled", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=True)
    _say(st)
    # same arithmetic in the same order as the row-major path: identical bits
    plain = forward(w, L)
    assert torch.equal(res["out"].view(torch.int16), plain["out"].view(torch.int16))


def test_config2_prefill_full_tiled():
    w = synth.CONFIGS["c2_qwen_prefill"]
    _say("config 2, tiled weights", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=True)
    _say(st)
    assert abs(st["r_ze"] - 0.5) < 0.02 and st["nonempty"] == w.N


def test_config3_decode_full_tiled():
    w = synth.CONFIGS["c3_qwen_decode"]
    _say("config 3, tiled weights", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=True)
    _say(st)


# The GEMM loop treats the chunks of an item differently depending on whether the loads in flight all belong to
# the item (its first chunks) or reach into the next item (its last `ring depth` chunks): widths whose chunk
# counts fall below, at and just above the ring depth, for both k-chunk widths (32 tiled, 64 row-major), with
# enough rows per expert for several items per workgroup and a ragged last tile.
CHUNK_EDGE_WIDTHS = [(128, 64), (128, 128), (256, 64), (256, 192), (384, 320), (640, 128)]


@pytest.mark.parametrize("tiled", [False, True], ids=["row_major", "tiled"])
@pytest.mark.parametrize("H, I", CHUNK_EDGE_WIDTHS, ids=lambda v: str(v))
def test_chunk_counts_around_the_ring_depth(H, I, tiled):
    w = synth.Workload("chunk_edges", T=700, H=H, I=I, N=3, Z=2, K=2, dtype="bf16", seed=86 + H + I, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.2)
    _say("chunk edges", "tiled" if tiled else "row-major", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=tiled)
    assert st["R"] > 0 and np.isfinite(res["out"].float().numpy()).all()


# Expert loads just above the 256-row token tile: the tiled path then launches the kernel that holds two tile
# geometries and picks, on the device, the 320-row one when it saves passes over expert weights.  Cases: every
# expert in (256, 320] (static layer), about half of them there (zero experts present), loads well above the window
# (the kernel falls back to 256-row tiles), and loads spread on both sides of it.
ADAPTIVE_CASES = [
    dict(T=2300, H=256, I=128, N=8, Z=0, K=1, seed=91, zero_bias=0.0),
    dict(T=1150, H=256, I=128, N=8, Z=4, K=4, seed=92, zero_bias=0.45),
    dict(T=1700, H=256, I=256, N=8, Z=4, K=4, seed=93, zero_bias=0.2),
    dict(T=1150, H=512, I=128, N=6, Z=6, K=3, seed=94, zero_bias=0.1),
]


@pytest.mark.parametrize("cfg", ADAPTIVE_CASES, ids=lambda c: "T%d_H%d_I%d_N%d_Z%d_K%d" % (c["T"], c["H"], c["I"], c["N"], c["Z"], c["K"]))
def test_loads_around_the_wide_token_tile(cfg):
    w = synth.Workload("adaptive", dtype="bf16", recipe="zero_bias", x_std=1.0, w_std=0.05, wr_std=0.05, **cfg)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L, tiled=True)
    rows = np.diff(res["expert_offsets"].numpy())
    _say("adaptive", w, "rows per expert", rows.tolist())
    assert st["R"] > 0
