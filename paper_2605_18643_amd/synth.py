"""Seeded synthetic inputs for one ZEDA MoE layer.

This module only draws numbers.  It holds none of the layer's arithmetic (no
router projection, no top-k, no expert FFN): the CPU oracle and the HIP library
both consume what it returns, and neither is imported here.

Bulk tensors come from a counter-based generator built from exact integer
operations (a 32-bit finaliser-style mixer applied to the element index and a
key) followed by a lookup into a 2^20-entry table of standard-normal quantiles.
Every step is either integer arithmetic on values below 2^63, a table gather,
or one IEEE multiply, so the same call yields the same bits on the CPU and on a
GPU: large tensors can be drawn directly in HBM and copied to the host for the
oracle.

Workloads follow the shapes the paper states for Qwen3-30B-A3B (Appendix D,
Table 12: H=2048, H_e=768, N=128, K=8) with about half of the selected slots on
zero experts (Section 3.2 reports r_ZE of 51.2 %), token-level heterogeneity
(Section 4.1) and no systematic trend across the 48 layers (Section 4.1).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_TABLE_BITS = 20
_CHUNK_CPU = 1 << 18   # temporaries stay cache-resident
_CHUNK_GPU = 1 << 24

# Tags that separate the streams of one workload.
TAG_X, TAG_WR, TAG_WG, TAG_WU, TAG_WD, TAG_PLAN, TAG_PERM = 1, 2, 3, 4, 5, 6, 7


# ----------------------------------------------------------------------------
# integer mixer (values are uint32 carried in int64 tensors / python ints)
# ----------------------------------------------------------------------------
def _mul32_py(x: int, c: int) -> int:
    return (x * c) & _M32


def _fmix32_py(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = _mul32_py(x, 0x85EBCA6B)
    x ^= x >> 13
    x = _mul32_py(x, 0xC2B2AE35)
    x ^= x >> 16
    return x


def make_key(*parts: int) -> int:
    """Fold a tuple of non-negative integers into one 32-bit stream key."""
    k = 0x9E3779B9
    for p in parts:
        p = int(p)
        k = _fmix32_py(k ^ (p & _M32))
        k = _fmix32_py((k + 0x7F4A7C15) ^ ((p >> 32) & _M32))
    return k


def _mul32(x: torch.Tensor, c: int) -> torch.Tensor:
    # x < 2^32 and c < 2^32: split x so that no product reaches 2^63.
    lo = x & 0xFFFF
    hi = x >> 16
    return (lo * c + (((hi * c) & 0xFFFF) << 16)) & _M32


def _fmix32(x: torch.Tensor) -> torch.Tensor:
    x = x ^ (x >> 16)
    x = _mul32(x, 0x85EBCA6B)
    x = x ^ (x >> 13)
    x = _mul32(x, 0xC2B2AE35)
    x = x ^ (x >> 16)
    return x


def hash_u32(index: torch.Tensor, key) -> torch.Tensor:
    """uint32 hash (in int64) of an int64 element index under a stream key.

    `key` is a python int or an int64 tensor broadcastable to `index`."""
    lo = index & _M32
    hi = (index >> 32) & _M32
    if isinstance(key, int):
        k1 = key
        k2 = _fmix32_py(key ^ 0x5BD1E995)
    else:
        k1 = key
        k2 = _fmix32(key ^ 0x5BD1E995)
    h = _fmix32(lo ^ k1)
    h = _fmix32(((h + k2) & _M32) ^ _mul32(hi, 0x9E3779B1))
    return h


# ----------------------------------------------------------------------------
# normal quantile table
# ----------------------------------------------------------------------------
_table_cpu: Optional[torch.Tensor] = None
_table_dev: Dict[str, torch.Tensor] = {}


def _normal_table(device: torch.device) -> torch.Tensor:
    global _table_cpu
    if _table_cpu is None:
        from scipy.special import ndtri

        n = 1 << _TABLE_BITS
        q = (np.arange(n, dtype=np.float64) + 0.5) / n
        _table_cpu = torch.from_numpy(ndtri(q).astype(np.float32))
    key = str(device)
    if key not in _table_dev:
        _table_dev[key] = _table_cpu.to(device)
    return _table_dev[key]


def normal_flat(n: int, key, std: float, device, dtype=torch.float32,
                start: int = 0, row_len: int = 0) -> torch.Tensor:
    """n draws of N(0, std^2), element i keyed by (key, start + i).

    If `key` is an int64 tensor it holds one key per row of `row_len` elements."""
    device = torch.device(device)
    table = _normal_table(device)
    out = torch.empty(n, dtype=dtype, device=device)
    std32 = float(np.float32(std))
    chunk = _CHUNK_CPU if device.type == "cpu" else _CHUNK_GPU
    for c0 in range(0, n, chunk):
        c1 = min(n, c0 + chunk)
        idx = torch.arange(start + c0, start + c1, dtype=torch.int64, device=device)
        if isinstance(key, int):
            h = hash_u32(idx, key)
        else:
            rows = torch.div(idx - start, row_len, rounding_mode="floor")
            h = hash_u32(idx, key.to(device)[rows])
        z = table[h >> (32 - _TABLE_BITS)]
        out[c0:c1] = (z * std32).to(dtype)
    return out


def uniform_cpu(n: int, key: int, start: int = 0) -> np.ndarray:
    """n float64 draws in (0,1); CPU only (used for small routing plans)."""
    idx = torch.arange(start, start + n, dtype=torch.int64)
    h = hash_u32(idx, key).numpy().astype(np.float64)
    return (h + 0.5) / 4294967296.0


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    T: int
    H: int
    I: int
    N: int
    Z: int
    K: int
    dtype: str            # "f32" | "bf16"
    seed: int
    recipe: str           # "plain" | "zero_bias" | "planted"
    x_std: float = 1.0
    w_std: float = 0.02
    wr_std: float = 0.02
    zero_bias: float = 0.0        # beta added to every zero-expert logit ("zero_bias")
    zipf_s: float = 1.1           # real-expert popularity exponent ("planted")
    easy_frac: float = 0.6        # share of easy tokens ("planted")
    plant_x: float = 4.0          # value written on a planted coordinate of x
    plant_w: float = 3.0          # router weight on an expert's own coordinate

    @property
    def NE(self) -> int:
        return self.N + self.Z

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# beta of the "zero_bias" recipe: found by oracle/calibrate_workloads.py so that
# the mean number of zero-expert slots per token is 4.0 +- 0.05 of K=8 at the
# Qwen3-shaped layer (N=128, Z=32, H=2048, x~N(0,1), W_r~N(0,0.02^2)).
QWEN_ZERO_BIAS = 0.6468
# the same calibration for N=128, Z=64, K=8 and for N=64, Z=32, K=4 (H=2048 both): half of the slots
NZ64_ZERO_BIAS = 0.2991
GLM_LIKE_ZERO_BIAS = 0.3092

CONFIGS: Dict[str, Workload] = {
    # benchmark configuration 1: tiny fp32 layer, no bias, seed 0.
    "c1_tiny_f32": Workload("c1_tiny_f32", T=64, H=256, I=128, N=8, Z=4, K=2, dtype="f32", seed=0,
                            recipe="plain", x_std=0.02, w_std=0.02, wr_std=0.05),
    # benchmark configuration 2: Qwen3-30B-A3B-shaped prefill layer, ~4 of 8 slots on zero experts.
    "c2_qwen_prefill": Workload("c2_qwen_prefill", T=4096, H=2048, I=768, N=128, Z=32, K=8, dtype="bf16",
                                seed=1, recipe="zero_bias", zero_bias=QWEN_ZERO_BIAS),
    # benchmark configuration 3: the same layer in a decode shape.
    "c3_qwen_decode": Workload("c3_qwen_decode", T=64, H=2048, I=768, N=128, Z=32, K=8, dtype="bf16",
                               seed=2, recipe="zero_bias", zero_bias=QWEN_ZERO_BIAS),
    # benchmark configuration 4: heterogeneous difficulty + Zipf(1.1) expert popularity.
    "c4_hetero_prefill": Workload("c4_hetero_prefill", T=16384, H=2048, I=768, N=128, Z=32, K=8, dtype="bf16",
                                  seed=3, recipe="planted"),
    # benchmark configuration 5: one layer of the 48-layer stack (T=8192); layer l uses seed 4000 + l.
    "c5_stack_layer": Workload("c5_stack_layer", T=8192, H=2048, I=768, N=128, Z=32, K=8, dtype="bf16",
                               seed=4000, recipe="zero_bias", zero_bias=QWEN_ZERO_BIAS),
    # Further workloads (beyond the five benchmark configurations).  The paper's own zero-expert count on the Qwen3 shape (App. D
    # Table 12: N_Z = 64), prefill and its decode concurrency of 32 ...
    "n1_qwen_nz64_prefill": Workload("n1_qwen_nz64_prefill", T=4096, H=2048, I=768, N=128, Z=64, K=8, dtype="bf16",
                                     seed=11, recipe="zero_bias", zero_bias=NZ64_ZERO_BIAS),
    "n1_qwen_nz64_decode32": Workload("n1_qwen_nz64_decode32", T=32, H=2048, I=768, N=128, Z=64, K=8, dtype="bf16",
                                      seed=12, recipe="zero_bias", zero_bias=NZ64_ZERO_BIAS),
    # ... and a layer with the router of the paper's second model (Section 3.1: N = 64, K = 4, N_Z = 32).  Its
    # hidden sizes are not given in the paper: H and I here are this build's choice.
    "n1_glm_like_prefill": Workload("n1_glm_like_prefill", T=4096, H=2048, I=1536, N=64, Z=32, K=4, dtype="bf16",
                                    seed=13, recipe="zero_bias", zero_bias=GLM_LIKE_ZERO_BIAS),
}


def _row_keys(base_key: int, attempt: Optional[torch.Tensor], T: int) -> torch.Tensor:
    """One key per token; a token's `attempt` counter selects a fresh draw of its row."""
    if attempt is None:
        attempt = torch.zeros(T, dtype=torch.int64)
    a = attempt.to(torch.int64).cpu()
    return _fmix32((_mul32(a + 1, 0x9E3779B1) ^ base_key) & _M32)


def planted_plan(w: Workload) -> Dict[str, np.ndarray]:
    """Routing plan of the "planted" recipe (CPU, float64, small).

    Per token: a class (easy with probability easy_frac, else hard), a zero-slot
    count (uniform on {6,7,8} for easy, {0,1} for hard, clipped to [max(0,K-N), min(K,Z)]),
    that many distinct zero experts chosen uniformly, and K minus that many distinct
    real experts drawn without replacement with probability proportional to a
    Zipf(zipf_s) popularity laid over a seeded permutation of the experts
    (exponential-race sampling: smallest E_i / p_i win)."""
    T, N, Z, K = w.T, w.N, w.Z, w.K
    key = make_key(w.seed, TAG_PLAN)
    u_class = uniform_cpu(T, make_key(key, 1))
    u_count = uniform_cpu(T, make_key(key, 2))
    easy = u_class < w.easy_frac
    zc = np.where(easy, 6 + np.minimum((u_count * 3).astype(np.int64), 2),
                  np.minimum((u_count * 2).astype(np.int64), 1))
    zc = np.clip(zc, max(0, K - N), min(K, Z)).astype(np.int64)
    # popularity
    perm = np.argsort(uniform_cpu(N, make_key(w.seed, TAG_PERM)), kind="stable")
    pop = np.empty(N, dtype=np.float64)
    pop[perm] = (np.arange(1, N + 1, dtype=np.float64)) ** (-w.zipf_s)
    pop /= pop.sum()
    # exponential race for real experts, uniform race for zero experts
    e_real = -np.log(uniform_cpu(T * N, make_key(key, 3))).reshape(T, N) / pop[None, :]
    real_rank = np.argsort(e_real, axis=1, kind="stable")
    planted = np.zeros((T, N + Z), dtype=bool)
    if Z > 0:
        zero_rank = np.argsort(uniform_cpu(T * Z, make_key(key, 4)).reshape(T, Z), axis=1, kind="stable")
    for t in range(T):
        planted[t, real_rank[t, : K - zc[t]]] = True
        if zc[t] > 0:
            planted[t, N + zero_rank[t, : zc[t]]] = True
    return {"easy": easy, "zero_count": zc, "popularity": pop, "planted": planted}


def _plant_coords(w: Workload, seed: int) -> np.ndarray:
    """Hidden coordinate owned by each of the N+Z experts in the "planted" recipe."""
    return np.argsort(uniform_cpu(w.H, make_key(seed, TAG_PERM, 9)), kind="stable")[: w.NE]


def draw_router(w: Workload, device="cpu", layer: int = 0):
    """w_router[N+Z,H] in the workload's dtype and router_bias[N+Z] (fp32) or None."""
    seed = w.seed + layer
    dev = torch.device(device)
    wr = normal_flat(w.NE * w.H, make_key(seed, TAG_WR), w.wr_std, dev, torch.float32).view(w.NE, w.H)
    bias = None
    if w.recipe == "zero_bias":
        bias = torch.zeros(w.NE, dtype=torch.float32)
        bias[w.N:] = w.zero_bias
        bias = bias.to(dev)
    elif w.recipe == "planted":
        coord_t = torch.from_numpy(_plant_coords(w, seed)).to(dev)
        wr[torch.arange(w.NE, device=dev), coord_t] = w.plant_w
    elif w.recipe != "plain":
        raise ValueError(w.recipe)
    return wr.to(w.torch_dtype), bias


def draw_tokens(w: Workload, device="cpu", attempt: Optional[torch.Tensor] = None, layer: int = 0,
                planted: Optional[np.ndarray] = None) -> torch.Tensor:
    """x[T,H] in the workload's dtype.  `attempt[t]` (int64, default 0) re-draws row t; the caller
    uses it to move tokens whose routing would be too close to a tie.
    planted ("planted" recipe only): a bool mask [T, N+Z] with K entries per row that replaces the seeded
    routing plan (tests that need prescribed expert loads)."""
    seed = w.seed + layer
    dev = torch.device(device)
    kx = make_key(seed, TAG_X)
    x = normal_flat(w.T * w.H, _row_keys(kx, attempt, w.T), w.x_std, dev, torch.float32, row_len=w.H).view(w.T, w.H)
    if w.recipe == "planted":
        # Expert e owns hidden coordinate coord[e]; a token carries plant_x there for each expert
        # of its plan and exactly 0 on the coordinates of all other experts.
        if planted is None:
            planted = planted_plan(w.with_(seed=seed))["planted"]
        coord_t = torch.from_numpy(_plant_coords(w, seed)).to(dev)
        mask = torch.from_numpy(np.asarray(planted, dtype=bool)).to(dev)
        x[:, coord_t] = torch.where(mask, torch.tensor(w.plant_x, device=dev), torch.tensor(0.0, device=dev))
    return x.to(w.torch_dtype)


def draw_experts(w: Workload, device="cpu", layer: int = 0):
    """w_gate[N,I,H], w_up[N,I,H], w_down[N,H,I] in the workload's dtype."""
    seed = w.seed + layer
    dt = w.torch_dtype
    N, I, H = w.N, w.I, w.H
    wg = normal_flat(N * I * H, make_key(seed, TAG_WG), w.w_std, device, dt).view(N, I, H)
    wu = normal_flat(N * I * H, make_key(seed, TAG_WU), w.w_std, device, dt).view(N, I, H)
    wd = normal_flat(N * H * I, make_key(seed, TAG_WD), w.w_std, device, dt).view(N, H, I)
    return wg, wu, wd


def make_layer(w: Workload, device="cpu", attempt: Optional[torch.Tensor] = None,
               layer: int = 0, planted: Optional[np.ndarray] = None) -> Dict[str, Optional[torch.Tensor]]:
    """All tensors of one layer: x, w_router, router_bias, w_gate, w_up, w_down.
    `layer` offsets the seed (stack workloads); `planted` as in draw_tokens."""
    wr, bias = draw_router(w, device, layer)
    wg, wu, wd = draw_experts(w, device, layer)
    return {"x": draw_tokens(w, device, attempt, layer, planted), "w_router": wr, "router_bias": bias,
            "w_gate": wg, "w_up": wu, "w_down": wd}


def to_numpy_f32(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """Exact widening of a (bf16 or fp32) tensor to a C-contiguous float32 array on the host."""
    if t is None:
        return None
    return np.ascontiguousarray(t.detach().to("cpu", torch.float32).numpy())
