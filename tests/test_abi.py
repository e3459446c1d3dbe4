"""The C ABI without a GPU: the library loads, exports every symbol include/zeda.h declares, sizes its
workspaces, and turns every invalid call into an error code before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2605_18643_amd import zeda

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "zeda.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zeda_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = zeda.lib()
    names = _declared_symbols()
    assert {"zeda_route", "zeda_dispatch", "zeda_expert_ffn", "zeda_combine", "zeda_moe_forward"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(zeda.EXPORTS) == set(names)


def test_status_strings():
    assert zeda.status_string(0) == "ZEDA_OK"
    assert zeda.status_string(-1) == "ZEDA_EINVAL"
    assert zeda.status_string(-2) == "ZEDA_EUNSUPPORTED"
    assert zeda.status_string(-3) == "ZEDA_EWORKSPACE"
    assert zeda.status_string(-4) == "ZEDA_EHIP"


def _desc(**kw):
    base = dict(T=4096, H=2048, I=768, N=128, Z=32, K=8, dtype="bf16")
    base.update(kw)
    return zeda.make_desc(**base)


def test_workspace_sizes():
    d = _desc()
    L = zeda.workspace_layout(d)
    S = 4096 * 8
    total = zeda.workspace_bytes(d)
    assert total == L.total and total >= S * (4 + 4 + 4 + 4) + S * 768 * 2 + S * 2048 * 2
    assert zeda.expert_ffn_workspace_bytes(d) >= S * 768 * 2 and zeda.expert_ffn_workspace_bytes(d) <= total
    assert 0 < zeda.dispatch_workspace_bytes(d) <= total
    offs = [L.topk_ids, L.topk_gates, L.expert_offsets, L.sorted_slot, L.slot_to_row, L.num_real, L.dispatch_ws, L.act,
            L.y_slot, L.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    # fp32 doubles the float buffers; Z = 0 and T = 0 are valid layers
    assert zeda.workspace_bytes(_desc(dtype="f32")) > total
    # Z only changes the router's scratch (one logit table row per token and split) and the dispatch region, which
    # also holds the router's per-block counts of every expert
    d0 = _desc(Z=0)
    L0 = zeda.workspace_layout(d0)
    assert (total - zeda.route_workspace_bytes(d) - (L.act - L.dispatch_ws)
            == zeda.workspace_bytes(d0) - zeda.route_workspace_bytes(d0) - (L0.act - L0.dispatch_ws))
    assert L.act - L.dispatch_ws >= (128 + 32) * (4096 // 16)
    assert zeda.workspace_bytes(_desc(T=0)) > 0


@pytest.mark.parametrize("kw, code", [
    (dict(T=-1), zeda.ZEDA_EINVAL), (dict(K=0), zeda.ZEDA_EINVAL), (dict(N=0), zeda.ZEDA_EINVAL),
    (dict(Z=-1), zeda.ZEDA_EINVAL), (dict(N=4, Z=2, K=7), zeda.ZEDA_EINVAL), (dict(H=0), zeda.ZEDA_EINVAL),
    (dict(K=17), zeda.ZEDA_EUNSUPPORTED), (dict(N=250, Z=7), zeda.ZEDA_EUNSUPPORTED),
    (dict(H=2048 + 64), zeda.ZEDA_EUNSUPPORTED), (dict(I=768 + 32), zeda.ZEDA_EUNSUPPORTED),
    (dict(dtype="f32", H=2050), zeda.ZEDA_EUNSUPPORTED), (dict(T=1 << 22), zeda.ZEDA_EUNSUPPORTED),
])
def test_descriptor_validation(kw, code):
    d = _desc(**kw)
    assert zeda.workspace_bytes(d) == 0
    out = zeda.WsLayout()
    assert zeda.lib().zeda_workspace_layout(ctypes.byref(d), ctypes.byref(out)) == code
    # the compute entry points refuse the same descriptor before touching any pointer
    p = ctypes.c_void_p(4096)
    assert zeda.lib().zeda_route(ctypes.byref(d), p, p, None, p, p, None, 0, None) == code
    assert zeda.lib().zeda_moe_forward(ctypes.byref(d), p, p, None, p, p, p, p, None, p, 1 << 40, None) == code


def test_bad_enum_values():
    d = _desc()
    d.dtype = 5
    assert zeda.workspace_bytes(d) == 0
    d = _desc()
    d.gate_norm = 3
    assert zeda.workspace_bytes(d) == 0
    d = _desc()
    d.weight_layout = 2
    assert zeda.workspace_bytes(d) == 0
    d = _desc()
    d.free_expert = 2
    assert zeda.workspace_bytes(d) == 0


def test_tiled_weights_are_bf16_only():
    d = _desc(dtype="bf16")
    d.weight_layout = zeda.WEIGHTS_TILED
    assert zeda.workspace_bytes(d) > 0
    d = _desc(dtype="f32")
    d.weight_layout = zeda.WEIGHTS_TILED
    assert zeda.workspace_bytes(d) == 0
    p = ctypes.c_void_p(4096)
    lib = zeda.lib()
    assert lib.zeda_moe_forward(ctypes.byref(d), p, p, None, p, p, p, p, None, p, 1 << 40, None) == zeda.ZEDA_EUNSUPPORTED
    # the packer: fp32 is refused, a lone input or output pointer is an error, all before any launch
    assert lib.zeda_pack_expert_weights(ctypes.byref(d), p, None, None, ctypes.c_void_p(1 << 30), None, None, None) == zeda.ZEDA_EUNSUPPORTED
    d = _desc(dtype="bf16")
    assert lib.zeda_pack_expert_weights(ctypes.byref(d), p, None, None, None, None, None, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_pack_expert_weights(None, p, None, None, p, None, None, None) == zeda.ZEDA_EINVAL


def test_pointer_and_workspace_errors_return_before_any_launch():
    lib = zeda.lib()
    d = _desc()
    ok = ctypes.c_void_p(1 << 20)       # aligned, never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p((1 << 20) + 8)
    need = zeda.workspace_bytes(d)
    dp = ctypes.byref(d)
    assert lib.zeda_route(dp, None, ok, None, ok, ok, None, 0, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_route(dp, odd, ok, None, ok, ok, None, 0, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_route(dp, ok, ok, odd, ok, ok, None, 0, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_route(dp, ok, ok, None, ok, ok, odd, 1 << 40, None) == zeda.ZEDA_EINVAL
    small = _desc(T=64)  # few token blocks: the router wants scratch for its split-k launch
    assert zeda.route_workspace_bytes(small) > 0
    assert lib.zeda_route(ctypes.byref(small), ok, ok, None, ok, ok, ok, zeda.route_workspace_bytes(small) - 1, None) == zeda.ZEDA_EWORKSPACE
    assert zeda.route_workspace_bytes(_desc(T=16384)) == 0 and zeda.route_workspace_bytes(_desc(dtype="f32", H=256, I=128)) == 0
    assert lib.zeda_dispatch(dp, ok, ok, ok, ok, ok, None, need, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_dispatch(dp, ok, ok, ok, ok, ok, ok, zeda.dispatch_workspace_bytes(d) - 1, None) == zeda.ZEDA_EWORKSPACE
    assert lib.zeda_expert_ffn(dp, ok, ok, ok, ok, ok, ok, ok, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_expert_ffn(dp, ok, ok, ok, ok, ok, ok, ok, ok, ok, zeda.expert_ffn_workspace_bytes(d) - 1, None) == zeda.ZEDA_EWORKSPACE
    assert lib.zeda_combine(dp, ok, ok, ok, ok, None, None, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_combine(dp, ok, ok, ok, odd, None, ok, None) == zeda.ZEDA_EINVAL
    dc = _desc()
    dc.free_expert = zeda.EXPERT_COPY  # the copy-expert variant reads the layer input
    assert lib.zeda_combine(ctypes.byref(dc), ok, ok, ok, ok, None, ok, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_combine(ctypes.byref(dc), ok, ok, ok, ok, odd, ok, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_moe_forward(dp, ok, ok, None, ok, ok, ok, ok, None, ok, need - 1, None) == zeda.ZEDA_EWORKSPACE
    assert lib.zeda_moe_forward(dp, ok, ok, None, ok, None, ok, ok, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert lib.zeda_moe_forward_events(dp, ok, ok, None, ok, ok, ok, ok, None, ok, need, None, None) == zeda.ZEDA_EINVAL


def test_block_forward_argument_checks():
    lib = zeda.lib()
    d = _desc()
    dp = ctypes.byref(d)
    ok, ok2, ok3 = (ctypes.c_void_p(v << 20) for v in (1, 2, 3))
    odd = ctypes.c_void_p((1 << 20) + 8)
    need = zeda.workspace_bytes(d)
    eps = ctypes.c_float(1e-6)
    call = lib.zeda_moe_block_forward
    assert call(dp, ok, None, ok, None, ok, ok, ok, None, eps, ok3, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert call(dp, ok, odd, ok, None, ok, ok, ok, None, eps, ok3, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert call(dp, ok, ok, ok, None, ok, ok, ok, None, eps, ok3, None, ok, need, None) == zeda.ZEDA_EINVAL  # x_res is xn
    assert call(dp, ok, ok2, ok, None, ok, ok, ok, None, eps, ok2, None, ok, need, None) == zeda.ZEDA_EINVAL  # x_res is xn_next
    assert call(dp, ok, ok2, ok, None, ok, ok, ok, None, ctypes.c_float(-1), ok3, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert call(dp, ok, ok2, ok, None, ok, ok, ok, odd, eps, ok3, None, ok, need, None) == zeda.ZEDA_EINVAL
    assert call(dp, ok, ok2, ok, None, ok, ok, ok, None, eps, ok3, None, ok, need - 1, None) == zeda.ZEDA_EWORKSPACE
    wide = _desc(H=8192 + 128)
    assert zeda.workspace_bytes(wide) > 0
    assert call(ctypes.byref(wide), ok, ok2, ok, None, ok, ok, ok, None, eps, ok3, None, ok, 1 << 40, None) == zeda.ZEDA_EUNSUPPORTED


def test_routing_stats_argument_checks():
    lib = zeda.lib()
    d = _desc()
    ok = ctypes.c_void_p(1 << 20)
    need = int(lib.zeda_routing_stats_workspace_bytes(ctypes.byref(d)))
    assert need > 0
    f32 = ctypes.c_float
    dp = ctypes.byref(d)
    assert lib.zeda_routing_stats(dp, ok, ok, None, f32(1), f32(1), ok, ok, ok, ok, need - 1, None) == zeda.ZEDA_EWORKSPACE
    assert lib.zeda_routing_stats(dp, ok, ok, None, f32(1), f32(0), ok, ok, ok, ok, need, None) == zeda.ZEDA_EINVAL  # w > 0
    assert lib.zeda_routing_stats(dp, ok, ok, None, f32(1), f32(1), None, ok, ok, ok, need, None) == zeda.ZEDA_EINVAL
    d0 = _desc(T=0)
    assert lib.zeda_routing_stats(ctypes.byref(d0), ok, ok, None, f32(1), f32(1), ok, ok, ok, ok, 1 << 30, None) == zeda.ZEDA_EINVAL


def test_binding_raises_with_the_status_name():
    d = _desc(K=0)
    with pytest.raises(zeda.ZedaError) as ei:
        zeda.workspace_layout(d)
    assert ei.value.status == zeda.ZEDA_EINVAL and "ZEDA_EINVAL" in str(ei.value)
