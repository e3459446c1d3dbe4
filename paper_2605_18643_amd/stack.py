"""The layer-stack workload: L MoE layers chained as x <- x + MoE_l(RMSNorm(x)), no attention (benchmark
config 5).  This file only owns buffers and the order of the C-ABI calls; every step runs in the HIP library."""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

from . import synth, zeda

EPS = 1e-6


class MoeStack:
    """Per-layer weights drawn by synth (layer l uses seed + l) and the scratch for one pass."""

    def __init__(self, w: synth.Workload, layers: int, device="cuda", static: bool = False, tiled: bool = False):
        """tiled: keep the expert weights in the library's tiled layout (packed here, once per layer)."""
        self.w = w if not static else w.with_(Z=0, recipe="plain")
        self.layers = layers
        self.weights: List[Dict[str, Optional[torch.Tensor]]] = []
        for l in range(layers):
            wr, bias = synth.draw_router(w, device, l)
            wg, wu, wd = synth.draw_experts(w, device, l)
            if static:  # the static top-K layer: router restricted to the normal experts, no bias
                wr, bias = wr[: w.N].contiguous(), None
            if tiled:
                wg, wu, wd = zeda.zeda_pack_expert_weights(zeda.make_desc(w.T, w.H, w.I, w.N, 0, w.K, w.dtype), wg, wu, wd)
            self.weights.append({"w_router": wr, "router_bias": bias, "w_gate": wg, "w_up": wu, "w_down": wd})
        ww = self.w
        self.desc = zeda.make_desc(ww.T, ww.H, ww.I, ww.N, ww.Z, ww.K, ww.dtype,
                                   weight_layout=zeda.WEIGHTS_TILED if tiled else zeda.WEIGHTS_ROW_MAJOR)
        self.ws = torch.empty(zeda.workspace_bytes(self.desc), dtype=torch.uint8, device=device)
        self.xn = torch.empty((ww.T, ww.H), dtype=ww.torch_dtype, device=device)
        self.y = torch.empty((ww.T, ww.H), dtype=ww.torch_dtype, device=device)
        self.num_real = torch.zeros(layers, dtype=torch.int32, device=device)

    def static_twin(self) -> "MoeStack":
        """The same stack without zero experts (router restricted to the normal experts, no bias), sharing this
        stack's expert weights and, being run one after the other, its scratch."""
        if self.w.Z == 0:
            return self
        twin = object.__new__(MoeStack)
        twin.w = self.w.with_(Z=0, recipe="plain")
        twin.layers = self.layers
        twin.weights = [dict(p, w_router=p["w_router"][: self.w.N].contiguous(), router_bias=None) for p in self.weights]
        twin.desc = zeda.make_desc(twin.w.T, twin.w.H, twin.w.I, twin.w.N, 0, twin.w.K, twin.w.dtype,
                                   weight_layout=self.desc.weight_layout)
        need = zeda.workspace_bytes(twin.desc)
        twin.ws = self.ws if self.ws.numel() >= need else torch.empty(need, dtype=torch.uint8, device=self.ws.device)
        twin.xn, twin.y = self.xn, self.y
        twin.num_real = torch.zeros_like(self.num_real)
        return twin

    def forward(self, x: torch.Tensor, hook=None, fused: Optional[bool] = None,
                token_zero: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Runs the chain in place on x (the residual stream) and returns it.  The stream is never synchronised.
        token_zero (int32[T], device): receives, per token, the number of its slots that landed on zero experts summed
        over all layers (Section 4.1's token-level r_ZE is that over layers * K).
        fused (default: whenever no hook is given): one zeda_moe_block_forward per layer, whose combine stage adds
        into x and writes the next layer's normalised input; one RMSNorm kernel for the first layer only.
        hook(l, stack, x) is then called before layer l (self.xn is its input, x the stream so far) and once more
        with l = layers after the last one.
        Otherwise three calls per layer, and hook(l, stack) is called after layer l's MoE output is in self.y and
        before the residual add."""
        if fused is None:
            fused = hook is None
        ids = zeda.ws_views(self.desc, self.ws)["topk_ids"] if token_zero is not None else None
        if fused:
            zeda.zeda_rmsnorm(x, None, EPS, self.xn)
            for l, p in enumerate(self.weights):
                if hook is not None:
                    hook(l, self, x)
                last = l == self.layers - 1
                zeda.zeda_moe_block_forward(self.desc, self.xn, x, p["w_router"], p["router_bias"], p["w_gate"],
                                            p["w_up"], p["w_down"], None, EPS, None if last else self.xn,
                                            self.num_real[l: l + 1], self.ws)
                if token_zero is not None:
                    zeda.zeda_token_zero_slots(self.desc, ids, token_zero, accumulate=l > 0)
            if hook is not None:
                hook(self.layers, self, x)
            return x
        for l, p in enumerate(self.weights):
            zeda.zeda_rmsnorm(x, None, EPS, self.xn)
            zeda.zeda_moe_forward(self.desc, self.xn, p["w_router"], p["router_bias"], p["w_gate"], p["w_up"], p["w_down"],
                                  self.y, self.num_real[l: l + 1], self.ws)
            if token_zero is not None:
                zeda.zeda_token_zero_slots(self.desc, ids, token_zero, accumulate=l > 0)
            if hook is not None:
                hook(l, self)
            zeda.zeda_residual_add(x, self.y)
        return x
