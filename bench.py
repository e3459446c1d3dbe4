#!/usr/bin/env python3
"""Benchmark of the ZEDA MoE-layer forward path on one MI355X.

One step = one zeda_moe_forward over the Qwen3-30B-A3B-shaped prefill layer (T=4096, H=2048, I=768,
N=128 normal + Z=32 zero experts, K=8, bf16, about half of the slots on zero experts), inputs resident
in HBM.  Prints ONE JSON line: tokens/s, the roofline of the dominant kernel (gate/up grouped GEMM)
from HIP-event timings taken in this run, and the CPU oracle timed on the host cores beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2605_18643_amd import synth, zeda  # noqa: E402

METRIC = "MoE-layer tokens/s (Qwen3-30B-A3B shape, ~50% zero slots) + MFMA util %"
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
# Counters cannot be read from inside this process.  These are RECORDED values of earlier rocprofv3 --pmc runs of this
# same program (the summaries and their command lines are under profiles/); they are reported, labelled as recorded,
# only for the workload and weight layout they were measured on, and are re-measured whenever the GEMM kernel changes.
#   traffic: HBM bytes per launch of the gate/up kernel (FETCH_SIZE x 2 KiB + WRITE_SIZE x 1 KiB, both scales read off
#   a plain copy kernel in the same runs); mfma_busy_pct: SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x cycles of the launch)
RECORDED_COUNTERS = {
    ("c2_qwen_prefill", "tiled"): {"traffic": 898.3e6, "traffic_source": "profiles/ffn_kernels_c2_qwen_prefill_hbm_traffic.txt",
                                   "mfma_busy_pct": {"gateup": 31.9, "down": 26.5},
                                   "mfma_busy_source": "profiles/ffn_kernels_c2_qwen_prefill_mfma_lds_counters.txt"},
    ("c4_hetero_prefill", "tiled"): {"mfma_busy_pct": {"gateup": 49.0, "down": 39.9},
                                     "mfma_busy_source": "profiles/ffn_kernels_c4_hetero_prefill_mfma_lds_counters.txt"},
}
CPU_BASELINE_SECONDS = 12.0      # the oracle keeps making passes over its token sample until this much time has gone by


def run_layer(w: synth.Workload, L, steps: int, warmup: int, lead_in=None):
    """Times `steps` forward passes (whole-path wall time) and, in a second loop of the same length,
    each stage with HIP events recorded between the kernels on the launch stream.
    lead_in = (steps, warmup): a long back-to-back run of the same step, timed the same way, directly in front of the
    warm-up (nothing but one synchronise in between), so that the region asked for starts on a chip at its working
    clocks; its wall time per step is returned as lead_in_ms."""
    d = zeda.make_desc(w.T, w.H, w.I, w.N, w.Z, w.K, w.dtype, weight_layout=L.get("weight_layout", zeda.WEIGHTS_ROW_MAJOR))
    ws = torch.empty(zeda.workspace_bytes(d), dtype=torch.uint8, device="cuda")
    out = torch.empty((w.T, w.H), dtype=w.torch_dtype, device="cuda")
    nreal = torch.zeros(1, dtype=torch.int32, device="cuda")
    args = (d, L["x"], L["w_router"], L["router_bias"], L["w_gate"], L["w_up"], L["w_down"], out, nreal, ws)
    lead_in_ms = None
    if lead_in:
        for _ in range(lead_in[1]):
            zeda.zeda_moe_forward(*args)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(lead_in[0]):
            zeda.zeda_moe_forward(*args)
        torch.cuda.synchronize()
        lead_in_ms = (time.perf_counter() - t0) / lead_in[0] * 1e3
    for _ in range(warmup):
        zeda.zeda_moe_forward(*args)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        zeda.zeda_moe_forward(*args)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    n_ev = len(zeda.STAGES) + 1
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(steps)]
    for row in evs:
        for e in row:
            e.record()  # creates the underlying hipEvent_t
    torch.cuda.synchronize()
    for row in evs:
        zeda.zeda_moe_forward_events(*args, row)
    torch.cuda.synchronize()
    stage_ms = np.zeros(len(zeda.STAGES))
    for row in evs:
        for i in range(len(zeda.STAGES)):
            stage_ms[i] += row[i].elapsed_time(row[i + 1])
    stage_ms /= steps
    v = zeda.ws_views(d, ws)
    off = v["expert_offsets"].cpu().numpy()
    R = int(nreal.item())
    return {"wall_s": wall, "stage_ms": stage_ms, "R": R, "nonempty": int((np.diff(off) > 0).sum()),
            "max_rows": int(np.diff(off).max()), "out": out, "lead_in_ms": lead_in_ms}


def time_stack(layers: int, steps: int, warmup: int, tiled: bool):
    """benchmark configuration 5: the chained stack at Z=32 and at Z=0 (same expert weights, router restricted to the
    normal experts); one step = one pass of all layers over T=8192 tokens."""
    from paper_2605_18643_amd.stack import MoeStack

    w = synth.CONFIGS["c5_stack_layer"]
    res = {}
    x0 = synth.draw_tokens(w, "cuda")
    st = MoeStack(w, layers, tiled=tiled)
    for name, stack in (("z32", st), ("z0", st.static_twin())):
        x = x0.clone()
        for _ in range(max(1, warmup)):
            stack.forward(x.copy_(x0))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            stack.forward(x.copy_(x0))
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        res[name] = {"ms_per_pass": dt * 1e3, "real_slots": int(stack.num_real.sum().item())}
        if name == "z32":
            # one more pass, untimed: per token, the share of its slots over all layers that landed on zero experts
            # (the token-level r_ZE of Section 4.1; the per-layer one is 1 - real slots / slots of that layer)
            tz = torch.zeros(w.T, dtype=torch.int32, device="cuda")
            stack.forward(x.copy_(x0), token_zero=tz)
            torch.cuda.synchronize()
            share = tz.float().cpu().numpy() / (layers * w.K)
            per_layer = 1.0 - stack.num_real.float().cpu().numpy() / (w.T * w.K)
            res[name]["token_r_ze"] = {"mean": float(share.mean()), "min": float(share.min()), "max": float(share.max()),
                                       "p10": float(np.percentile(share, 10)), "p90": float(np.percentile(share, 90))}
            res[name]["layer_r_ze"] = {"min": float(per_layer.min()), "max": float(per_layer.max())}
    del st
    torch.cuda.empty_cache()
    return w, {"layers": layers, "T": w.T, "steps": steps, "warmup": warmup,
               "tokens_per_s": w.T / (res["z32"]["ms_per_pass"] * 1e-3),
               "z32": res["z32"], "z0": res["z0"],
               "stack_speedup_vs_z0": res["z0"]["ms_per_pass"] / res["z32"]["ms_per_pass"],
               "expert_flop_reduction": 1.0 - res["z32"]["real_slots"] / max(1, res["z0"]["real_slots"])}


def stack_bench(a) -> int:
    w, r = time_stack(a.layers, a.steps, max(1, a.warmup // 2), a.weights == "tiled")
    out = {"metric": "48-layer MoE stack tokens/s (Qwen3-30B-A3B layer shape, T=8192, ~50% zero slots)",
           "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
           "warmup": a.warmup, "ms_per_step": r["z32"]["ms_per_pass"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
           "config": {"workload": "c5_stack", "layers": a.layers, "T": w.T, "H": w.H, "I": w.I, "N": w.N, "Z": w.Z, "K": w.K,
                      "weight_layout": a.weights},
           "z32": r["z32"], "z0": r["z0"],
           "stack_speedup_vs_z0": r["stack_speedup_vs_z0"],
           "expert_flop_reduction": r["expert_flop_reduction"]}
    print(json.dumps(out))
    return 0


def overlap_probe(buf: torch.Tensor):
    """How far a CU overlaps HBM streaming with matrix work: zeda_overlap_probe timed with the reads alone, the MFMAs
    alone - their number chosen so that both take about equally long - and both together, over the same buffer, for
    its two placements of the waves (every SIMD holding a reading and a multiplying wave; the readers on a SIMD of
    their own)."""
    nbytes = (buf.numel() * buf.element_size()) >> 20 << 20
    flat = buf.view(-1).view(torch.uint8)[:nbytes]
    wgs = nbytes >> 20
    sink = torch.zeros(wgs * 512 + 8, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(mode, mfmas, reps=6):
        for _ in range(2):
            zeda.zeda_overlap_probe(flat, mfmas, mode, sink)
        e0.record()
        for _ in range(reps):
            zeda.zeda_overlap_probe(flat, mfmas, mode, sink)
        e1.record()
        torch.cuda.synchronize()
        clk = sink[wgs * 512 + 2: wgs * 512 + 6].view(torch.int64).cpu().numpy()  # cycles, 100 MHz ticks (last launch)
        return e0.elapsed_time(e1) / reps * 1e3, 100.0 * float(clk[0]) / max(1.0, float(clk[1]))

    out = {"bytes": nbytes,
           "note": "one kernel, one workgroup of eight waves per CU: some waves stream 1 MiB from HBM, the others issue "
                   "register-only MFMAs; hidden_frac = (read + mfma - both) / min(read, mfma): 1 = perfect overlap, "
                   "0 = the times add up"}
    for name, place, n_mfma_waves in (("same_simd", 0, 4), ("split_simd", zeda.PROBE_SPLIT_SIMD, 6)):
        t_read, _ = timed(zeda.PROBE_READ | place, 0)
        mfmas = 1600
        mfmas = max(8, int(mfmas * t_read / timed(zeda.PROBE_MFMA | place, mfmas)[0]) // 8 * 8)  # about as long as the reads
        (t_read, mhz_read), (t_mfma, mhz_mfma), (t_both, mhz_both) = (
            timed(zeda.PROBE_READ | place, 0), timed(zeda.PROBE_MFMA | place, mfmas),
            timed(zeda.PROBE_READ | zeda.PROBE_MFMA | place, mfmas))
        out[name] = {"mfmas_per_wave": mfmas, "mfma_waves": n_mfma_waves, "read_alone_us": t_read, "mfma_alone_us": t_mfma,
                     "both_us": t_both, "read_alone_gbs": nbytes / (t_read * 1e-6) / 1e9,
                     "mfma_alone_tflops": 2.0 * 32 * 32 * 16 * mfmas * n_mfma_waves * wgs / (t_mfma * 1e-6) / 1e12,
                     "hidden_frac": (t_read + t_mfma - t_both) / min(t_read, t_mfma),
                     # shader clock while each ran (cycle counter over 100 MHz counter, one mid-launch wave)
                     "shader_clock_mhz": {"read_alone": mhz_read, "mfma_alone": mhz_mfma, "both": mhz_both}}
    return out


def pack_layer(w, L):
    """The layer with its expert weights in the library's tiled layout (packed once, as when a model is loaded)."""
    L = dict(L)
    L["w_gate"], L["w_up"], L["w_down"] = zeda.zeda_pack_expert_weights(
        zeda.make_desc(w.T, w.H, w.I, w.N, w.Z, w.K, w.dtype), L["w_gate"], L["w_up"], L["w_down"])
    L["weight_layout"] = zeda.WEIGHTS_TILED
    return L


def static_twin(w, L):
    """The same layer without zero experts: top-K over the N normal experts only, same weights."""
    L0 = dict(L)
    L0["w_router"] = L["w_router"][: w.N].contiguous()
    L0["router_bias"] = None
    return w.with_(Z=0, recipe="plain"), L0


def other_config_legs(tiled: bool):
    """Short legs of benchmark configurations 3, 4 and 5 in the same run as the headline (each with its own
    warm-up; times are HIP-event stage times and wall time per step as for the headline)."""
    legs = {}
    # configuration 3: decode shape, bound by streaming the weights of the experts that were hit
    w = synth.CONFIGS["c3_qwen_decode"]
    L = synth.make_layer(w, "cuda")
    L = pack_layer(w, L) if tiled else L
    r = run_layer(w, L, steps=400, warmup=200)
    w0, L0 = static_twin(w, L)
    r0 = run_layer(w0, L0, steps=400, warmup=100)
    wbytes = 3.0 * w.H * w.I * 2 * r["nonempty"]
    gu_s, dn_s = r["stage_ms"][2] * 1e-3, r["stage_ms"][3] * 1e-3
    legs["c3_qwen_decode"] = {
        "T": w.T, "ms_per_step": r["wall_s"] / 400 * 1e3, "tokens_per_s": w.T * 400 / r["wall_s"],
        "real_slots": r["R"], "nonempty_experts": r["nonempty"], "expert_weight_bytes": wbytes,
        "weights_gbs_in_gemm_kernels": wbytes / (gu_s + dn_s) / 1e9, "hbm_frac_in_gemm_kernels": wbytes / (gu_s + dn_s) / 1e9 / HBM_PEAK_GBS,
        "weights_gbs_whole_step": wbytes / (r["wall_s"] / 400) / 1e9,
        "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, r["stage_ms"])},
        "z0_ms_per_step": r0["wall_s"] / 400 * 1e3, "speedup_vs_z0": r0["wall_s"] / r["wall_s"]}
    del L, L0
    torch.cuda.empty_cache()
    # configuration 4: heterogeneous prefill, the compute-bound regime of the grouped GEMMs
    w = synth.CONFIGS["c4_hetero_prefill"]
    L = synth.make_layer(w, "cuda")
    L = pack_layer(w, L) if tiled else L
    r = run_layer(w, L, steps=150, warmup=100)
    w0, L0 = static_twin(w, L)
    r0 = run_layer(w0, L0, steps=80, warmup=40)
    gu_s, dn_s = r["stage_ms"][2] * 1e-3, r["stage_ms"][3] * 1e-3
    gu_f, dn_f = 4.0 * w.H * w.I * r["R"], 2.0 * w.H * w.I * r["R"]
    legs["c4_hetero_prefill"] = {
        "T": w.T, "ms_per_step": r["wall_s"] / 150 * 1e3, "tokens_per_s": w.T * 150 / r["wall_s"],
        "real_slots": r["R"], "r_ze": 1.0 - r["R"] / (w.T * w.K), "max_rows_per_expert": r["max_rows"],
        "nonempty_experts": r["nonempty"],
        "gateup_tflops": gu_f / gu_s / 1e12, "down_tflops": dn_f / dn_s / 1e12,
        "gateup_mfma_frac": gu_f / gu_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "expert_gemm_mfma_frac": (gu_f + dn_f) / (gu_s + dn_s) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, r["stage_ms"])},
        "z0_ms_per_step": r0["wall_s"] / 80 * 1e3, "speedup_vs_z0": (r0["wall_s"] / 80) / (r["wall_s"] / 150),
        "expert_flop_reduction": 1.0 - r["R"] / max(1, r0["R"])}
    del L, L0
    torch.cuda.empty_cache()
    # configuration 5: the 48-layer chain with and without zero experts
    _, legs["c5_stack"] = time_stack(48, steps=12, warmup=3, tiled=tiled)
    return legs


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 1000 for one layer, 50 for the 48-layer stack)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 200 / 5)")
    ap.add_argument("--workload", default="c2_qwen_prefill", choices=sorted(synth.CONFIGS) + ["c5_stack"],
                    help="c5_stack: the 48-layer chain (RMSNorm + residual, no attention) with and without zero experts")
    ap.add_argument("--layers", type=int, default=48)
    ap.add_argument("--tokens", type=int, default=0, help="override T of the workload (sequence-length sweeps)")
    ap.add_argument("--weights", default="tiled", choices=["tiled", "row_major"],
                    help="storage of the expert weights: packed once into the library's tiled layout (default), or row-major")
    ap.add_argument("--token-sweep", default="",
                    help="comma-separated token counts: times the workload's layer and its Z=0 twin at each of them "
                         "(sequence-length sweep) and prints one JSON line with the table; nothing else is run")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads and writes 2^28 bytes (a yardstick for "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters; outside the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-z0", action="store_true")
    ap.add_argument("--no-sustained", action="store_true",
                    help="skip the cold region and the long back-to-back run that a short timed region (--steps < 500) "
                         "is preceded by")
    ap.add_argument("--cold-start", action="store_true",
                    help="time the steps asked for first, on the idle chip, and run the long back-to-back run after them")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short legs of configurations 3, 4 and 5 that the default run adds after the headline")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context: also time torch.bmm (the vendor GEMM library) on dense batched GEMMs of the expert "
                         "GEMMs' shapes (no gather, no SwiGLU, every expert with the mean row count)")
    a = ap.parse_args()
    # A short run measures the first milliseconds after idle, before the clocks have settled: the default covers
    # about a third of a second of sustained work (the stack's steps are 25 ms each, so 50 of them do).
    stack = a.workload == "c5_stack"
    if a.steps is None:
        a.steps = 50 if stack else 1000
    if a.warmup is None:
        a.warmup = 5 if stack else 200
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (the HIP library has no CPU fallback)", file=sys.stderr)
        return 2
    zeda.lib()
    if a.calibration_copy:
        src = torch.arange(1 << 26, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.bitwise_xor(src, 0x55, out=dst)  # one kernel: 268,435,456 bytes in, 268,435,456 bytes out
        torch.cuda.synchronize()
        del src, dst
    if a.workload == "c5_stack":
        return stack_bench(a)

    w = synth.CONFIGS[a.workload]
    if a.token_sweep:
        rows = []
        for T in (int(v) for v in a.token_sweep.split(",")):
            wt = w.with_(T=T)
            Lt = synth.make_layer(wt, "cuda")
            if a.weights == "tiled" and wt.dtype == "bf16":
                Lt = pack_layer(wt, Lt)
            steps = max(20, min(400, (1 << 21) // T))
            r = run_layer(wt, Lt, steps, steps // 4, lead_in=(steps, steps // 4))
            w0, L0 = static_twin(wt, Lt)
            r0 = run_layer(w0, L0, steps, steps // 4, lead_in=(steps, steps // 4))
            rows.append({"T": T, "steps": steps, "us_per_step": r["wall_s"] / steps * 1e6,
                         "tokens_per_s": T * steps / r["wall_s"], "z0_us_per_step": r0["wall_s"] / steps * 1e6,
                         "speedup_vs_z0": r0["wall_s"] / r["wall_s"], "r_ze": 1.0 - r["R"] / (T * wt.K),
                         "rows_per_expert": r["R"] / max(1, r["nonempty"]),
                         "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, r["stage_ms"])}})
            del Lt, L0
            torch.cuda.empty_cache()
        print(json.dumps({"token_sweep": rows, "workload": w.name, "weight_layout": a.weights, "dtype": w.dtype,
                          "data": "synthetic"}))
        return 0
    if a.tokens > 0:
        w = w.with_(T=a.tokens)
    L = synth.make_layer(w, "cuda")
    L_rowmajor = L
    if a.weights == "tiled" and w.dtype == "bf16":
        # weights are static: packed once, outside the timed region, as when a model is loaded
        L = pack_layer(w, L)
    torch.cuda.synchronize()
    # A short timed region right after idle sits in the clock transient of the chip's first milliseconds of heavy
    # work (a gap of a millisecond is enough to fall back into it).  So a short run (--steps < 500) first takes the
    # same region cold (reported as `cold_start`), then a long back-to-back run (`sustained`) and, with nothing but a
    # synchronise in between - the chip now at its working clocks - the warm-up and the timed steps that were asked
    # for, which are what `value` reports.  --cold-start keeps the old order (value = cold).
    pre = {}
    warm_order = a.steps < 500 and not a.no_sustained and not a.cold_start
    if warm_order:
        rc = run_layer(w, L, a.steps, a.warmup)
        pre["cold_start"] = {"steps": a.steps, "warmup": a.warmup, "ms_per_step": rc["wall_s"] / a.steps * 1e3,
                             "tokens_per_s": w.T * a.steps / rc["wall_s"],
                             "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, rc["stage_ms"])}}
    r = run_layer(w, L, a.steps, a.warmup, lead_in=(600, 150) if warm_order else None)
    if warm_order:
        pre["sustained"] = {"steps": 600, "warmup": 150, "ms_per_step": r["lead_in_ms"],
                            "tokens_per_s": w.T / (r["lead_in_ms"] * 1e-3)}
    ms = r["wall_s"] / a.steps * 1e3
    tokens_per_s = w.T * a.steps / r["wall_s"]

    es = 2 if w.dtype == "bf16" else 4
    R, ne = r["R"], r["nonempty"]
    stage = dict(zip(zeda.STAGES, (float(x) for x in r["stage_ms"])))
    # gate/up grouped GEMM: weights of the non-empty experts once, one x row in and one act row out per real slot
    gu_bytes = 2.0 * w.H * w.I * es * ne + R * (w.H + w.I) * es
    gu_flops = 4.0 * w.H * w.I * R
    dn_bytes = 1.0 * w.H * w.I * es * ne + R * (w.I + w.H) * es
    dn_flops = 2.0 * w.H * w.I * R
    gu_s, dn_s = stage["gateup"] * 1e-3, stage["down"] * 1e-3
    achieved_gbs = gu_bytes / gu_s / 1e9
    recorded = RECORDED_COUNTERS.get((w.name, a.weights if w.dtype == "bf16" else "row_major"), {})
    # the binding roofline of the gate/up kernel on this workload: whichever of its two floors is the longer
    if gu_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) > gu_bytes / (HBM_PEAK_GBS * 1e9) and w.dtype == "bf16":
        achieved_tf = gu_flops / gu_s / 1e12
        roofline = {"kernel": "ffn_bf16_kernel<gate/up>", "bound": "mfma", "achieved": achieved_tf,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved_tf / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": None, "avg_launch_us": gu_s * 1e6, "algorithmic_flops": gu_flops,
                    "algorithmic_bytes": gu_bytes}
    else:
        roofline = {"kernel": "ffn_bf16_kernel<gate/up>", "bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                    "traffic": recorded.get("traffic"), "traffic_source": recorded.get("traffic_source"),
                    "avg_launch_us": gu_s * 1e6, "algorithmic_bytes": gu_bytes}
    ffn_tflops = (gu_flops + dn_flops) / (gu_s + dn_s) / 1e12
    res = {
        "metric": METRIC, "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "H": w.H, "I": w.I, "N": w.N, "Z": w.Z, "K": w.K,
                   "real_slots": R, "r_ze": 1.0 - R / (w.T * w.K), "nonempty_experts": ne, "max_rows_per_expert": r["max_rows"],
                   "weight_layout": "tiled" if L.get("weight_layout") == zeda.WEIGHTS_TILED else "row_major"},
        "roofline": roofline,
        # real-slot FLOPs of both GEMMs over their event-timed durations, against the 2.5 PFLOP/s peak (arithmetic) ...
        "mfma_util_pct": 100.0 * ffn_tflops / MFMA_BF16_PEAK_TFLOPS,
        # ... and the MFMA pipes' busy share by counter, a recorded profile value (null where none was taken)
        "mfma_busy_pct_recorded": recorded.get("mfma_busy_pct"), "mfma_busy_source": recorded.get("mfma_busy_source"),
        "expert_gemm": {"tflops": ffn_tflops, "peak_tflops": MFMA_BF16_PEAK_TFLOPS,
                        "gateup_tflops": gu_flops / gu_s / 1e12, "down_tflops": dn_flops / dn_s / 1e12,
                        "down_gbs": dn_bytes / dn_s / 1e9},
        "stage_us": {k: v * 1e3 for k, v in stage.items()},
        # algorithmic bytes of every stage over its event-timed duration
        "stage_gbs": {
            "route": (w.T * w.H * es + (w.N + w.Z) * w.H * es + w.T * w.K * 8) / (stage["route"] * 1e-3) / 1e9,
            "dispatch": (w.T * w.K * 12 + w.N * 4) / (stage["dispatch"] * 1e-3) / 1e9,
            "gateup": achieved_gbs,
            "down": dn_bytes / dn_s / 1e9,
            "combine": (R * w.H * es + w.T * w.H * es) / (stage["combine"] * 1e-3) / 1e9,
        },
    }
    res["config"]["mean_rows_per_expert"] = R / max(1, ne)

    if w.dtype == "bf16":
        # Yardstick for the HBM-bound kernels: the library's plain streaming-read kernel over the three expert weight
        # tensors of this layer in turn (more than the caches hold), timed with events on the launch stream.
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        bufs = [L["w_gate"], L["w_up"], L["w_down"]]
        for b in bufs:
            zeda.zeda_stream_read_probe(b, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 8
        e0.record()
        for _ in range(reps):
            for b in bufs:
                zeda.zeda_stream_read_probe(b, sink)
        e1.record()
        torch.cuda.synchronize()
        nbytes = sum(b.numel() * b.element_size() for b in bufs) * reps
        stream_gbs = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
        res["hbm_stream_read"] = {"gbs": stream_gbs, "frac_of_peak": stream_gbs / HBM_PEAK_GBS,
                                  "bytes_per_launch": bufs[0].numel() * bufs[0].element_size(),
                                  "note": "plain contiguous read of the expert weights by zeda_stream_read_probe: what HBM "
                                          "delivers on this machine to a kernel that does nothing else"}
        if roofline["bound"] == "hbm":
            roofline["frac_of_stream_read"] = achieved_gbs / stream_gbs
        # Yardstick for the compute-heavy kernels: the library's register-only MFMA loop (no memory traffic), two
        # workgroups per CU, long enough to reach the clock the chip holds under it.
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        msink = torch.empty(2 * cus * 256, dtype=torch.float32, device="cuda")
        zeda.zeda_mfma_probe(2 * cus, 20000, msink)
        e0.record()
        flops = sum(zeda.zeda_mfma_probe(2 * cus, 20000, msink) for _ in range(4))
        e1.record()
        torch.cuda.synchronize()
        mfma_tf = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
        probe_buf = torch.randint(0, 2 ** 31 - 1, (1536 << 18,), dtype=torch.int32, device="cuda")  # 1.5 GiB: six MiB per CU
        res["overlap_probe"] = overlap_probe(probe_buf)
        del probe_buf

    if not a.no_z0 and w.Z > 0:
        # the same kernels on the static layer: no zero experts, top-K over the N normal experts only
        w0, L0 = static_twin(w, L)
        r0 = run_layer(w0, L0, a.steps, a.warmup, lead_in=(300, 100) if warm_order else None)  # (the same way)
        res["z0"] = {"ms_per_step": r0["wall_s"] / a.steps * 1e3, "speedup_vs_z0": r0["wall_s"] / r["wall_s"],
                     "real_slots": r0["R"], "expert_flop_reduction": 1.0 - R / max(1, r0["R"]),
                     "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, r0["stage_ms"])}}

    if a.library_gemm and w.dtype == "bf16" and ne > 0:
        # What the vendor's batched GEMM reaches on this machine for the same amount of matrix work, in the same kind
        # of sustained loop: a yardstick for the MFMA-bound workloads (the nominal peak is not reached by it either).
        m = max(1, -(-R // ne))
        lib = {}
        for name, (kd, nd) in (("gateup", (w.H, 2 * w.I)), ("down", (w.I, w.H))):
            A = torch.randn(ne, m, kd, device="cuda", dtype=torch.bfloat16)
            B = torch.randn(ne, kd, nd, device="cuda", dtype=torch.bfloat16) * 0.02
            C = torch.empty(ne, m, nd, device="cuda", dtype=torch.bfloat16)
            for _ in range(50):
                torch.bmm(A, B, out=C)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                torch.bmm(A, B, out=C)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / 200
            lib[name] = {"us": dt * 1e6, "tflops": 2.0 * ne * m * kd * nd / dt / 1e12, "batch": ne, "rows": m}
            del A, B, C
        res["library_gemm"] = lib

    res.update(pre)
    if a.steps < 500 and not a.no_sustained and a.cold_start:
        rs = run_layer(w, L, 600, 150)
        res["sustained"] = {"steps": 600, "warmup": 150, "ms_per_step": rs["wall_s"] / 600 * 1e3,
                            "tokens_per_s": w.T * 600 / rs["wall_s"],
                            "stage_us": {k: float(v) * 1e3 for k, v in zip(zeda.STAGES, rs["stage_ms"])}}

    if w.name == "c2_qwen_prefill" and a.tokens <= 0 and not a.no_other_configs:
        res["other_configs"] = other_config_legs(a.weights == "tiled")
        if "mfma_probe" in res:
            c4 = res["other_configs"]["c4_hetero_prefill"]
            c4["gateup_frac_of_mfma_probe"] = c4["gateup_tflops"] / res["mfma_probe"]["tflops"]

    if not a.no_cpu_baseline:
        from oracle import harness, zeda_oracle as orc  # CPU-baseline leg only

        arrays = harness.to_arrays(L_rowmajor)
        n_tok = min(w.T, 4096)
        tok = np.arange(n_tok)
        passes, t0 = 0, time.perf_counter()
        while True:  # whole passes over the sample, about CPU_BASELINE_SECONDS of work in all
            ref = harness.oracle_forward(w, arrays, tokens=tok)
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= CPU_BASELINE_SECONDS or passes >= 64:
                break
        got = r["out"][:n_tok].float().cpu().numpy()
        res["cpu_baseline"] = {"value": passes * n_tok / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {n_tok} of {w.T} tokens of {w.name}, {passes} passes, {dt:.1f} s",
                               "gpu_vs_oracle_rel_l2": harness.rel_l2(got, ref["out"])}
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
