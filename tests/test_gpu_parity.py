"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded inputs.
Routing indices and dispatch arrays are compared bit for bit, floating-point results within the stated
tolerances (tests/gpu_util.py)."""
import numpy as np
import pytest
import torch

from oracle import harness, zeda_oracle as orc
from paper_2605_18643_amd import synth, zeda

pytestmark = pytest.mark.gpu

from gpu_util import check_float, desc_of, forward, full_parity  # noqa: E402


def _say(*a):
    print(*a, flush=True)


def test_generator_same_bits_on_gpu():
    k = synth.make_key(42, 1)
    a = synth.normal_flat(300_000, k, 0.02, "cpu", torch.bfloat16)
    b = synth.normal_flat(300_000, k, 0.02, "cuda", torch.bfloat16).cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    att = torch.arange(16) % 3
    w = synth.CONFIGS["c3_qwen_decode"].with_(T=16)
    assert torch.equal(synth.draw_tokens(w, "cpu", att).float(), synth.draw_tokens(w, "cuda", att).float().cpu())


@pytest.mark.parametrize("gate_norm", [zeda.GATE_TOPK_NORM, zeda.GATE_SOFTMAX, zeda.GATE_REAL_RENORM])
def test_config1_tiny_fp32(gate_norm):
    w = synth.CONFIGS["c1_tiny_f32"]
    _say("config 1", w, "gate_norm", gate_norm)
    L = harness.gapped_layer(w, "cuda", gate_norm=gate_norm)
    res, st = full_parity(w, L, gate_norm)
    _say(st)
    assert st["R"] > 0


SMALL_BF16 = [
    # several token tiles per expert with a ragged tail, zero experts present
    dict(T=1000, H=256, I=192, N=6, Z=4, K=3, seed=11, zero_bias=0.3),
    # one expert-row per tile at most, many experts, K=8
    dict(T=96, H=384, I=128, N=40, Z=24, K=8, seed=12, zero_bias=0.5),
    # static layer (Z=0), top-1
    dict(T=257, H=128, I=64, N=5, Z=0, K=1, seed=13, zero_bias=0.0),
    # the widest router the library accepts, K=16
    dict(T=130, H=128, I=64, N=200, Z=56, K=16, seed=14, zero_bias=0.2),
    # decode-sized token counts (the skinny tile configurations)
    dict(T=20, H=256, I=128, N=12, Z=4, K=4, seed=15, zero_bias=0.4),
    dict(T=64, H=256, I=128, N=12, Z=4, K=4, seed=16, zero_bias=0.4),
    dict(T=1, H=256, I=128, N=12, Z=4, K=4, seed=17, zero_bias=0.4),
    # a single normal expert next to zero experts (every real slot in one group, one long run of token tiles)
    dict(T=700, H=128, I=64, N=1, Z=3, K=2, seed=18, zero_bias=0.1),
    # every expert selected by every token (K = N + Z): routing only orders them
    dict(T=90, H=128, I=64, N=3, Z=2, K=5, seed=19, zero_bias=0.1),
]


@pytest.mark.parametrize("cfg", SMALL_BF16, ids=lambda c: "T%d_H%d_I%d_N%d_Z%d_K%d" % (c["T"], c["H"], c["I"], c["N"], c["Z"], c["K"]))
def test_small_bf16_layers(cfg):
    w = synth.Workload("small", dtype="bf16", recipe="zero_bias", x_std=1.0, w_std=0.05, wr_std=0.05, **cfg)
    _say("small bf16", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L)
    _say(st)


def test_small_fp32_layer_with_zero_experts_and_ragged_sizes():
    w = synth.Workload("small_f32", T=77, H=132, I=52, N=7, Z=5, K=3, dtype="f32", seed=21, recipe="zero_bias",
                       x_std=1.0, w_std=0.08, wr_std=0.08, zero_bias=0.2)
    _say("small fp32", w)
    L = harness.gapped_layer(w, "cuda")
    res, st = full_parity(w, L)
    _say(st)


def test_all_tokens_on_zero_experts_gives_exact_zero_and_no_rows():
    w = synth.Workload("allzero", T=70, H=128, I=64, N=6, Z=8, K=4, dtype="bf16", seed=31, recipe="zero_bias",
                       zero_bias=50.0)
    L = harness.gapped_layer(w, "cuda")
    res = forward(w, L)
    assert int(res["num_real"].item()) == 0 and not res["expert_offsets"].numpy().any()
    assert (res["slot_to_row"].numpy() == -1).all()
    assert not res["out"].float().numpy().any()
    assert (res["topk_ids"].numpy() >= w.N).all()


def test_forward_is_deterministic():
    w = synth.Workload("det", T=700, H=256, I=128, N=9, Z=5, K=4, dtype="bf16", seed=41, recipe="zero_bias", zero_bias=0.3)
    L = synth.make_layer(w, "cuda")
    a, b = forward(w, L), forward(w, L)
    for k in ("topk_ids", "topk_gates", "expert_offsets", "slot_to_row", "out"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k
    R = int(a["num_real"].item())
    assert torch.equal(a["sorted_slot"][:R], b["sorted_slot"][:R])
    assert torch.equal(a["y_slot"][:R].view(torch.int16), b["y_slot"][:R].view(torch.int16))


def test_empty_batch_is_a_no_op_on_every_entry_point():
    # T = 0: nothing is launched that could touch memory; dispatch still publishes all-zero offsets
    w = synth.Workload("empty", T=0, H=128, I=64, N=5, Z=3, K=2, dtype="bf16", seed=1, recipe="plain")
    d = zeda.make_desc(0, w.H, w.I, w.N, w.Z, w.K, "bf16")
    L = synth.make_layer(w.with_(T=4), "cuda")
    x0 = L["x"]  # any valid pointer: no row of it is read (a NULL pointer would be an argument error even at T = 0)
    guard = torch.full((8, w.H), 7.0, dtype=torch.bfloat16, device="cuda")  # a buffer that must stay untouched
    ws = torch.empty(max(zeda.workspace_bytes(d), 256), dtype=torch.uint8, device="cuda")
    nreal = torch.full((1,), -3, dtype=torch.int32, device="cuda")
    zeda.zeda_moe_forward(d, x0, L["w_router"], None, L["w_gate"], L["w_up"], L["w_down"], guard, nreal, ws)
    ids = torch.full((4,), -9, dtype=torch.int32, device="cuda")
    gates = torch.full((4,), -9.0, dtype=torch.float32, device="cuda")
    zeda.zeda_route(d, x0, L["w_router"], None, ids, gates)
    off = torch.full((w.N + 1,), -5, dtype=torch.int32, device="cuda")
    ss = torch.full((4,), -5, dtype=torch.int32, device="cuda")
    s2r = torch.full((4,), -5, dtype=torch.int32, device="cuda")
    nr = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    zeda.zeda_dispatch(d, ids, off, ss, s2r, nr, ws)
    zeda.zeda_combine(d, guard, ids, gates, s2r, guard)
    torch.cuda.synchronize()
    assert (guard.float() == 7.0).all() and (ids == -9).all() and (gates == -9.0).all()
    assert not off.cpu().numpy().any() and int(nr.item()) == 0 and (ss == -5).all() and (s2r == -5).all()
    assert int(nreal.item()) == 0  # the whole-layer call reports R = 0


def test_stream_read_probe_reads_and_rejects_bad_arguments():
    """The measurement aid: runs over a buffer with a ragged tail (not a multiple of a workgroup's run), writes
    nothing, and turns unaligned arguments into ZEDA_EINVAL."""
    buf = torch.arange((3 * 256 * 1024 + 4096) // 4, dtype=torch.int32, device="cuda")
    sink = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    zeda.zeda_stream_read_probe(buf, sink)
    zeda.zeda_stream_read_probe(buf[:4], sink)  # 16 bytes
    torch.cuda.synchronize()
    assert int(sink.item()) == 7
    with pytest.raises(zeda.ZedaError) as e:
        zeda.zeda_stream_read_probe(buf[1:5], sink)  # 4 bytes past a 16-byte boundary
    assert e.value.status < 0
    with pytest.raises(zeda.ZedaError):
        zeda.zeda_stream_read_probe(buf[:5], sink)  # 20 bytes


def test_mfma_probe_runs_and_rejects_bad_arguments():
    sink = torch.zeros(4 * 256, dtype=torch.float32, device="cuda")
    flops = zeda.zeda_mfma_probe(4, 3, sink)
    torch.cuda.synchronize()
    assert flops == 2.0 * 32 * 32 * 16 * 8 * 3 * 4 * 4
    assert torch.isfinite(sink).all() and float(sink.abs().sum()) > 0.0
    for wg, it in ((0, 3), (4, 0)):
        with pytest.raises(zeda.ZedaError):
            zeda.lib()  # (argument checks run on the host)
            zeda._check(zeda.lib().zeda_mfma_probe(wg, it, zeda._ptr(sink), None), "zeda_mfma_probe")


def test_overlap_probe_modes_and_bad_arguments():
    buf = torch.arange((3 << 20) // 4, dtype=torch.int32, device="cuda")  # 3 MiB: three workgroups
    n = 3 * 512
    sink = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    for place in (0, zeda.PROBE_SPLIT_SIMD):
        for mode in (zeda.PROBE_READ, zeda.PROBE_MFMA, zeda.PROBE_READ | zeda.PROBE_MFMA):
            sink.zero_()
            zeda.zeda_overlap_probe(buf, 800, mode | place, sink)
            torch.cuda.synchronize()
            wrote = int((sink[:n] != 0).sum())
            # only the multiplying waves leave their sums: four of eight waves, or six with the readers on a SIMD of their own
            assert wrote == (0 if not mode & zeda.PROBE_MFMA else 3 * 64 * (6 if place else 4)), (mode, place, wrote)
            assert torch.isfinite(sink[: n + 2]).all()
            cycles, ticks = (int(v) for v in sink[n + 2: n + 6].view(torch.int64).cpu())
            assert cycles > 0 and ticks > 0 and 100.0 < 100.0 * cycles / ticks < 3000.0  # a plausible shader clock
    for bad in (dict(mode=0), dict(mode=4), dict(mode=8), dict(mfmas=-1)):
        with pytest.raises(zeda.ZedaError):
            zeda.zeda_overlap_probe(buf, bad.get("mfmas", 8), bad.get("mode", 3), sink)
    with pytest.raises(zeda.ZedaError):
        zeda._check(zeda.lib().zeda_overlap_probe(zeda._ptr(buf), (1 << 20) + 16, 8, 3, zeda._ptr(sink), None), "zeda_overlap_probe")
