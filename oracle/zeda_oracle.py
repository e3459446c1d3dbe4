"""ctypes front end of the CPU oracle (oracle/zeda_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by the
CPU-baseline leg of bench.py; never by the product package.  It marshals numpy arrays
into the C functions and nothing else: all arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zeda_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

GATE_SOFTMAX, GATE_TOPK_NORM, GATE_REAL_RENORM = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP across tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_moe_flops.restype = ctypes.c_double
        _lib.oracle_moe_flops.argtypes = [ctypes.c_double] * 7
        _lib.oracle_flop_ratio.restype = ctypes.c_double
        _lib.oracle_flop_ratio.argtypes = [ctypes.c_int] + [ctypes.c_double] * 9
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_routing_stats.restype = ctypes.c_int
    return _lib


def _f32(a, shape=None) -> Optional[np.ndarray]:
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def route(x, w_router, router_bias, N: int, Z: int, K: int, gate_norm: int = GATE_TOPK_NORM,
          want_logits: bool = False):
    """ids[T,K] int32, gates[T,K] float64 (and logits[T,N+Z] float64)."""
    lib = _load()
    x = _f32(x)
    T, H = x.shape
    wr = _f32(w_router, (N + Z, H))
    b = _f32(router_bias, (N + Z,)) if router_bias is not None else None
    ids = np.empty((T, K), dtype=np.int32)
    gates = np.empty((T, K), dtype=np.float64)
    logits = np.empty((T, N + Z), dtype=np.float64) if want_logits else None
    rc = lib.oracle_route(_p(x), _p(wr), _p(b), T, H, N, Z, K, gate_norm, _p(ids), _p(gates), _p(logits))
    if rc != 0:
        raise ValueError("oracle_route: bad arguments")
    return (ids, gates, logits) if want_logits else (ids, gates)


def moe_forward(x, w_router, router_bias, w_gate, w_up, w_down, N: int, Z: int, K: int,
                gate_norm: int = GATE_TOPK_NORM, copy_expert: bool = False, want_y_slot: bool = False):
    """Eq. 1 for every token.  Returns dict(out[T,H] f64, ids, gates, real_slots, y_slot?)."""
    lib = _load()
    x = _f32(x)
    T, H = x.shape
    wg = _f32(w_gate)
    I = wg.shape[1]
    assert wg.shape == (N, I, H)
    wu = _f32(w_up, (N, I, H))
    wd = _f32(w_down, (N, H, I))
    wr = _f32(w_router, (N + Z, H))
    b = _f32(router_bias, (N + Z,)) if router_bias is not None else None
    out = np.empty((T, H), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    gates = np.empty((T, K), dtype=np.float64)
    y_slot = np.empty((T * K, H), dtype=np.float64) if want_y_slot else None
    real = ctypes.c_int64(0)
    rc = lib.oracle_moe_forward(_p(x), _p(wr), _p(b), _p(wg), _p(wu), _p(wd), T, H, I, N, Z, K, gate_norm,
                                int(bool(copy_expert)), _p(out), _p(ids), _p(gates), _p(y_slot), ctypes.byref(real))
    if rc != 0:
        raise ValueError("oracle_moe_forward: bad arguments")
    res = {"out": out, "ids": ids, "gates": gates, "real_slots": int(real.value)}
    if want_y_slot:
        res["y_slot"] = y_slot
    return res


def expert(x_t, wg_e, wu_e, wd_e) -> np.ndarray:
    """E_e(x_t) for one token row and one expert, float64[H]."""
    lib = _load()
    x_t = _f32(x_t)
    H = x_t.shape[0]
    wg_e = _f32(wg_e)
    I = wg_e.shape[0]
    wu_e = _f32(wu_e, (I, H))
    wd_e = _f32(wd_e, (H, I))
    y = np.empty(H, dtype=np.float64)
    lib.oracle_expert(_p(x_t), _p(wg_e), _p(wu_e), _p(wd_e), H, I, _p(y))
    return y


def dispatch(ids, N: int):
    """offsets[N+1], sorted_slot[T*K] (-1 past the real slots), slot_to_row[T*K] (-1 = zero slot)."""
    lib = _load()
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    offsets = np.empty(N + 1, dtype=np.int32)
    sorted_slot = np.empty(T * K, dtype=np.int32)
    slot_to_row = np.empty(T * K, dtype=np.int32)
    lib.oracle_dispatch(_p(ids), T, K, N, _p(offsets), _p(sorted_slot), _p(slot_to_row))
    return offsets, sorted_slot, slot_to_row


def combine(y_rows, ids, gates, slot_to_row, N: int) -> np.ndarray:
    lib = _load()
    y_rows = np.ascontiguousarray(y_rows, dtype=np.float64)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    gates = np.ascontiguousarray(gates, dtype=np.float64)
    slot_to_row = np.ascontiguousarray(slot_to_row, dtype=np.int32)
    T, K = ids.shape
    H = y_rows.shape[1]
    out = np.empty((T, H), dtype=np.float64)
    lib.oracle_combine(_p(y_rows), _p(ids), _p(gates), _p(slot_to_row), T, H, N, K, _p(out))
    return out


def rmsnorm(x, gamma=None, eps: float = 1e-6) -> np.ndarray:
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    T, H = x.shape
    g = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float64)
    out = np.empty_like(x)
    lib.oracle_rmsnorm(_p(x), _p(g), T, H, ctypes.c_double(eps), _p(out))
    return out


def routing_stats(x, w_router, router_bias, N: int, Z: int, K: int, alpha: float = 1.0, w: float = 1.0):
    """Section 2.2, Eq. 4-6 on the batch of all tokens: dict(f[N+Z], P[N+Z], f_E, P_E, f_Z, P_Z, r_ze, L_A, L_GA)."""
    lib = _load()
    x = _f32(x)
    T, H = x.shape
    wr = _f32(w_router, (N + Z, H))
    b = _f32(router_bias, (N + Z,)) if router_bias is not None else None
    f = np.empty(N + Z, dtype=np.float64)
    P = np.empty(N + Z, dtype=np.float64)
    summ = np.empty(7, dtype=np.float64)
    rc = lib.oracle_routing_stats(_p(x), _p(wr), _p(b), T, H, N, Z, K, ctypes.c_double(alpha), ctypes.c_double(w), _p(f),
                                  _p(P), _p(summ))
    if rc != 0:
        raise ValueError("oracle_routing_stats: bad arguments")
    keys = ("f_E", "P_E", "f_Z", "P_Z", "r_ze", "L_A", "L_GA")
    return {"f": f, "P": P, **{k: float(v) for k, v in zip(keys, summ)}}


def token_zero_slots(ids, N: int) -> np.ndarray:
    """Token-level zero-expert usage (Section 4.1, "Zero Expert Activation Dynamics": tokens differ in their r_ZE): for
    every token the number of its K selected slots that are zero experts (id >= N).  A token's r_ZE in one layer is
    this count over K; over a model, the sum of the counts of its layers over layers * K."""
    ids = np.asarray(ids)
    out = np.zeros(ids.shape[0], dtype=np.int64)
    for j in range(ids.shape[1]):
        out += ids[:, j] >= N
    return out


def init_zero_rows(w_router_normal, normals):
    """Section 2.1, router initialisation: rows[Z,H] = mean + std * normals, (mean, variance) of the N*H originals."""
    lib = _load()
    wr = _f32(w_router_normal)
    N, H = wr.shape
    z = _f32(normals)
    Z = z.shape[0]
    assert z.shape == (Z, H)
    rows = np.empty((Z, H), dtype=np.float64)
    stats = np.empty(2, dtype=np.float64)
    if lib.oracle_init_zero_rows(_p(wr), _p(z), N, Z, H, _p(rows), _p(stats)) != 0:
        raise ValueError("oracle_init_zero_rows: bad arguments")
    return rows, float(stats[0]), float(stats[1])


def moe_flops(n, H, He, N, NZ, K, r_ze) -> float:
    return float(_load().oracle_moe_flops(n, H, He, N, NZ, K, r_ze))


def flop_ratio(prefill: bool, l, H, Hattn, gkv, He, N, NZ, K, r_ze) -> float:
    return float(_load().oracle_flop_ratio(int(prefill), l, H, Hattn, gkv, He, N, NZ, K, r_ze))
