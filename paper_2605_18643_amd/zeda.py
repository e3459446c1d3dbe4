"""Thin Python binding of libzeda's C ABI (include/zeda.h): argument marshalling only.

Tensors are PyTorch-ROCm device tensors used as plain device buffers; every step of the layer runs
inside the HIP library.  There is no fallback: if the library is missing, importing the entry points
raises, and nothing here computes on the CPU.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libzeda.so")

ZEDA_OK, ZEDA_EINVAL, ZEDA_EUNSUPPORTED, ZEDA_EWORKSPACE, ZEDA_EHIP = 0, -1, -2, -3, -4
ZEDA_F32, ZEDA_BF16 = 0, 1
GATE_SOFTMAX, GATE_TOPK_NORM, GATE_REAL_RENORM = 0, 1, 2
WEIGHTS_ROW_MAJOR, WEIGHTS_TILED = 0, 1
EXPERT_ZERO, EXPERT_COPY = 0, 1
STAGES = ("route", "dispatch", "gateup", "down", "combine")

EXPORTS = ("zeda_status_string", "zeda_workspace_bytes", "zeda_route_workspace_bytes", "zeda_dispatch_workspace_bytes",
           "zeda_expert_ffn_workspace_bytes", "zeda_workspace_layout", "zeda_route", "zeda_dispatch",
           "zeda_dispatch_noalloc", "zeda_dispatch_noalloc_max_slots",
           "zeda_expert_ffn", "zeda_combine", "zeda_moe_forward", "zeda_moe_forward_events", "zeda_moe_block_forward",
           "zeda_rmsnorm",
           "zeda_residual_add", "zeda_pack_expert_weights", "zeda_routing_stats_workspace_bytes", "zeda_routing_stats",
           "zeda_init_zero_expert_rows", "zeda_stream_read_probe", "zeda_mfma_probe", "zeda_token_zero_slots", "zeda_overlap_probe")


class LayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "H", "I", "N", "Z", "K", "dtype", "gate_norm", "weight_layout",
                                                 "free_expert")]


class WsLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("topk_ids", "topk_gates", "expert_offsets", "sorted_slot",
                                               "slot_to_row", "num_real", "dispatch_ws", "act", "y_slot", "route_ws",
                                               "total")]


class ZedaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_18643_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(LayerDesc)
        L.zeda_status_string.restype = ctypes.c_char_p
        L.zeda_status_string.argtypes = [i32]
        for name in ("zeda_workspace_bytes", "zeda_route_workspace_bytes", "zeda_dispatch_workspace_bytes",
                     "zeda_expert_ffn_workspace_bytes", "zeda_routing_stats_workspace_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [dp]
        L.zeda_workspace_layout.restype = i32
        L.zeda_workspace_layout.argtypes = [dp, ctypes.POINTER(WsLayout)]
        L.zeda_route.restype = i32
        L.zeda_route.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.zeda_dispatch.restype = i32
        L.zeda_dispatch.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.zeda_dispatch_noalloc.restype = i32
        L.zeda_dispatch_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.zeda_dispatch_noalloc_max_slots.restype = i32
        L.zeda_dispatch_noalloc_max_slots.argtypes = []
        L.zeda_expert_ffn.restype = i32
        L.zeda_expert_ffn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.zeda_combine.restype = i32
        L.zeda_combine.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.zeda_moe_forward.restype = i32
        L.zeda_moe_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.zeda_moe_forward_events.restype = i32
        L.zeda_moe_forward_events.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, ctypes.POINTER(vp)]
        L.zeda_moe_block_forward.restype = i32
        L.zeda_moe_block_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, sz, vp]
        L.zeda_rmsnorm.restype = i32
        L.zeda_rmsnorm.argtypes = [i32, i32, i32, vp, vp, ctypes.c_float, vp, vp]
        L.zeda_residual_add.restype = i32
        L.zeda_residual_add.argtypes = [i32, i32, i32, vp, vp, vp]
        L.zeda_routing_stats.restype = i32
        L.zeda_routing_stats.argtypes = [dp, vp, vp, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp, sz, vp]
        L.zeda_init_zero_expert_rows.restype = i32
        L.zeda_init_zero_expert_rows.argtypes = [dp, vp, vp, vp, vp]
        L.zeda_token_zero_slots.restype = i32
        L.zeda_token_zero_slots.argtypes = [dp, vp, vp, i32, vp]
        L.zeda_overlap_probe.restype = i32
        L.zeda_overlap_probe.argtypes = [vp, sz, i32, i32, vp, vp]
        L.zeda_mfma_probe.restype = i32
        L.zeda_mfma_probe.argtypes = [i32, i32, vp, vp]
        L.zeda_stream_read_probe.restype = i32
        L.zeda_stream_read_probe.argtypes = [vp, sz, vp, vp]
        L.zeda_pack_expert_weights.restype = i32
        L.zeda_pack_expert_weights.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().zeda_status_string(int(status)).decode()


def make_desc(T, H, I, N, Z, K, dtype, gate_norm=GATE_TOPK_NORM, weight_layout=0, free_expert=0) -> LayerDesc:
    if isinstance(dtype, torch.dtype):
        dtype = ZEDA_BF16 if dtype == torch.bfloat16 else ZEDA_F32
    elif isinstance(dtype, str):
        dtype = ZEDA_BF16 if dtype == "bf16" else ZEDA_F32
    return LayerDesc(T, H, I, N, Z, K, int(dtype), int(gate_norm), int(weight_layout), int(free_expert))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str) -> None:
    if rc != ZEDA_OK:
        raise ZedaError(rc, where)


def workspace_bytes(desc: LayerDesc) -> int:
    return int(lib().zeda_workspace_bytes(ctypes.byref(desc)))


def dispatch_workspace_bytes(desc: LayerDesc) -> int:
    return int(lib().zeda_dispatch_workspace_bytes(ctypes.byref(desc)))


def expert_ffn_workspace_bytes(desc: LayerDesc) -> int:
    return int(lib().zeda_expert_ffn_workspace_bytes(ctypes.byref(desc)))


def workspace_layout(desc: LayerDesc) -> WsLayout:
    out = WsLayout()
    _check(lib().zeda_workspace_layout(ctypes.byref(desc), ctypes.byref(out)), "zeda_workspace_layout")
    return out


def route_workspace_bytes(desc: LayerDesc) -> int:
    return int(lib().zeda_route_workspace_bytes(ctypes.byref(desc)))


def zeda_route(desc, x, w_router, router_bias, topk_ids, topk_gates, ws=None, stream=None) -> None:
    """ws: uint8 scratch of route_workspace_bytes(desc) or None (see include/zeda.h)."""
    _check(lib().zeda_route(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(topk_ids),
                            _ptr(topk_gates), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "zeda_route")


def zeda_dispatch(desc, topk_ids, expert_offsets, sorted_slot, slot_to_row, num_real, ws, stream=None) -> None:
    _check(lib().zeda_dispatch(ctypes.byref(desc), _ptr(topk_ids), _ptr(expert_offsets), _ptr(sorted_slot),
                               _ptr(slot_to_row), _ptr(num_real), _ptr(ws), ws.numel() * ws.element_size(),
                               _stream(stream)), "zeda_dispatch")


def zeda_dispatch_noalloc(desc, topk_ids, expert_offsets, sorted_slot, slot_to_row, num_real, stream=None) -> None:
    """zeda_dispatch on the library's own static scratch (no workspace argument, nothing allocated)."""
    _check(lib().zeda_dispatch_noalloc(ctypes.byref(desc), _ptr(topk_ids), _ptr(expert_offsets), _ptr(sorted_slot),
                                       _ptr(slot_to_row), _ptr(num_real), _stream(stream)), "zeda_dispatch_noalloc")


def dispatch_noalloc_max_slots() -> int:
    return int(lib().zeda_dispatch_noalloc_max_slots())


def zeda_expert_ffn(desc, x, w_gate, w_up, w_down, expert_offsets, sorted_slot, num_real, y_slot, ws,
                    stream=None) -> None:
    _check(lib().zeda_expert_ffn(ctypes.byref(desc), _ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                 _ptr(expert_offsets), _ptr(sorted_slot), _ptr(num_real), _ptr(y_slot), _ptr(ws),
                                 ws.numel() * ws.element_size(), _stream(stream)), "zeda_expert_ffn")


def zeda_combine(desc, y_slot, topk_ids, topk_gates, slot_to_row, out, x=None, stream=None) -> None:
    """x (the layer input) is only needed with desc.free_expert == EXPERT_COPY."""
    _check(lib().zeda_combine(ctypes.byref(desc), _ptr(y_slot), _ptr(topk_ids), _ptr(topk_gates), _ptr(slot_to_row),
                              _ptr(x), _ptr(out), _stream(stream)), "zeda_combine")


def zeda_moe_forward(desc, x, w_router, router_bias, w_gate, w_up, w_down, out, num_real_out, ws,
                     stream=None) -> None:
    _check(lib().zeda_moe_forward(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate),
                                  _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(num_real_out), _ptr(ws),
                                  ws.numel() * ws.element_size(), _stream(stream)), "zeda_moe_forward")


def zeda_moe_forward_events(desc, x, w_router, router_bias, w_gate, w_up, w_down, out, num_real_out, ws, events,
                            stream=None) -> None:
    """`events`: len(STAGES)+1 recorded-once torch.cuda.Event(enable_timing=True) objects."""
    arr = (ctypes.c_void_p * len(events))(*[ctypes.c_void_p(e.cuda_event) for e in events])
    _check(lib().zeda_moe_forward_events(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                         _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(num_real_out),
                                         _ptr(ws), ws.numel() * ws.element_size(), _stream(stream), arr),
           "zeda_moe_forward_events")


def zeda_moe_block_forward(desc, xn, x_res, w_router, router_bias, w_gate, w_up, w_down, gamma_next, eps: float,
                           xn_next, num_real_out, ws, stream=None) -> None:
    """x_res += layer(xn) in place; xn_next (None to skip, may be xn itself) = RMSNorm(x_res) * gamma_next."""
    _check(lib().zeda_moe_block_forward(ctypes.byref(desc), _ptr(xn), _ptr(x_res), _ptr(w_router), _ptr(router_bias),
                                        _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(gamma_next), float(eps),
                                        _ptr(xn_next), _ptr(num_real_out), _ptr(ws), ws.numel() * ws.element_size(),
                                        _stream(stream)), "zeda_moe_block_forward")


def _dtype_code(t: torch.Tensor) -> int:
    return ZEDA_BF16 if t.dtype == torch.bfloat16 else ZEDA_F32


def zeda_rmsnorm(x, gamma, eps: float, out, stream=None) -> None:
    T, H = x.shape
    _check(lib().zeda_rmsnorm(T, H, _dtype_code(x), _ptr(x), _ptr(gamma), float(eps), _ptr(out), _stream(stream)),
           "zeda_rmsnorm")


def zeda_stream_read_probe(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Measurement aid: one plain streaming read of all bytes of `buf` (contiguous, a multiple of 16 bytes)."""
    _check(lib().zeda_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream(stream)),
           "zeda_stream_read_probe")


def zeda_token_zero_slots(desc, topk_ids, zero_slots, accumulate: bool = False, stream=None) -> None:
    """zero_slots[t] (int32[T], device) = or += the number of token t's K slots on zero experts (Section 4.1)."""
    _check(lib().zeda_token_zero_slots(ctypes.byref(desc), _ptr(topk_ids), _ptr(zero_slots), int(bool(accumulate)),
                                       _stream(stream)), "zeda_token_zero_slots")


PROBE_READ, PROBE_MFMA, PROBE_SPLIT_SIMD = 1, 2, 4


def zeda_overlap_probe(buf: torch.Tensor, mfmas_per_wave: int, mode: int, sink: torch.Tensor, stream=None) -> None:
    """Measurement aid: streaming read of buf (a multiple of 1 MiB) and / or register-only MFMAs in one kernel.
    sink: fp32, at least (MiB of buf) * 512 + 8 elements; the last six of these hold two int64 (shader-clock cycles
    and 100 MHz ticks of one mid-launch wave)."""
    nbytes = buf.numel() * buf.element_size()
    assert sink.dtype == torch.float32 and sink.numel() >= (nbytes >> 20) * 512 + 8
    _check(lib().zeda_overlap_probe(_ptr(buf), nbytes, int(mfmas_per_wave), int(mode), _ptr(sink), _stream(stream)),
           "zeda_overlap_probe")


def zeda_mfma_probe(workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """Measurement aid: launches the register-only MFMA loop; returns the FLOPs of the launch.  sink: fp32, at least
    workgroups * 256 elements."""
    assert sink.dtype == torch.float32 and sink.numel() >= workgroups * 256
    _check(lib().zeda_mfma_probe(int(workgroups), int(iters), _ptr(sink), _stream(stream)), "zeda_mfma_probe")
    return 2.0 * 32 * 32 * 16 * 8 * iters * 4 * workgroups


def zeda_residual_add(x, y, stream=None) -> None:
    T, H = x.shape
    _check(lib().zeda_residual_add(T, H, _dtype_code(x), _ptr(x), _ptr(y), _stream(stream)), "zeda_residual_add")


def zeda_routing_stats(desc, x, w_router, router_bias, alpha=1.0, w=1.0, stream=None):
    """Section 2.2 statistics over the batch of all tokens; allocates the outputs and the scratch.
    Returns device tensors (f[N+Z], P[N+Z], summary[7] = f_E, P_E, f_Z, P_Z, r_ZE, L_A, L_GA)."""
    NE = desc.N + desc.Z
    f = torch.empty(NE, dtype=torch.float32, device=x.device)
    P = torch.empty(NE, dtype=torch.float32, device=x.device)
    summary = torch.empty(7, dtype=torch.float32, device=x.device)
    nbytes = int(lib().zeda_routing_stats_workspace_bytes(ctypes.byref(desc)))
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    _check(lib().zeda_routing_stats(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), float(alpha), float(w),
                                    _ptr(f), _ptr(P), _ptr(summary), _ptr(ws), ws.numel(), _stream(stream)),
           "zeda_routing_stats")
    return f, P, summary


def zeda_init_zero_expert_rows(desc, w_router, normals, stream=None):
    """Fills rows N.. of w_router in place (see include/zeda.h); returns the device tensor {mean, variance}."""
    stats = torch.empty(2, dtype=torch.float32, device=w_router.device)
    _check(lib().zeda_init_zero_expert_rows(ctypes.byref(desc), _ptr(w_router), _ptr(normals), _ptr(stats), _stream(stream)),
           "zeda_init_zero_expert_rows")
    return stats


def zeda_pack_expert_weights(desc, w_gate, w_up, w_down, stream=None):
    """Tiled copies of the three expert tensors (any of them may be None); allocates the outputs."""
    outs = [None if w is None else torch.empty_like(w) for w in (w_gate, w_up, w_down)]
    _check(lib().zeda_pack_expert_weights(ctypes.byref(desc), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(outs[0]),
                                          _ptr(outs[1]), _ptr(outs[2]), _stream(stream)), "zeda_pack_expert_weights")
    return tuple(outs)


def ws_views(desc: LayerDesc, ws: torch.Tensor):
    """Typed views of the intermediate results zeda_moe_forward leaves in its workspace."""
    L = workspace_layout(desc)
    S = desc.T * desc.K
    dt = torch.bfloat16 if desc.dtype == ZEDA_BF16 else torch.float32
    es = 2 if desc.dtype == ZEDA_BF16 else 4
    b = ws.view(torch.uint8)

    def view(off, n, dtype, size):
        return b[off: off + n * size].view(dtype)

    return {
        "topk_ids": view(L.topk_ids, S, torch.int32, 4).view(desc.T, desc.K),
        "topk_gates": view(L.topk_gates, S, torch.float32, 4).view(desc.T, desc.K),
        "expert_offsets": view(L.expert_offsets, desc.N + 1, torch.int32, 4),
        "sorted_slot": view(L.sorted_slot, S, torch.int32, 4),
        "slot_to_row": view(L.slot_to_row, S, torch.int32, 4),
        "num_real": view(L.num_real, 1, torch.int32, 4),
        "act": view(L.act, S * desc.I, dt, es).view(S, desc.I),
        "y_slot": view(L.y_slot, S * desc.H, dt, es).view(S, desc.H),
    }
