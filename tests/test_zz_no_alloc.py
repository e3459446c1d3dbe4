"""zeda_dispatch_noalloc, the dispatch entry point that works on the library's own static scratch (for callers that
cannot allocate): called through the C ABI and compared, bit for bit, with zeda_dispatch on the same ids - two calls
in a row on the shared scratch, the second on a shorter slot list, then the one-kernel form and the size limit."""
import numpy as np
import pytest
import torch

from paper_2605_18643_amd import zeda

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _ids(T, K, N, Z, seed):
    """K distinct experts of N+Z per token (any such list is a valid routing result)."""
    g = torch.Generator().manual_seed(seed)
    return torch.rand(T, N + Z, generator=g).argsort(dim=1)[:, :K].to(torch.int32).contiguous().cuda()


def _both(T, K, N, Z, seed):
    d = zeda.make_desc(T, 256, 128, N, Z, K, "bf16")
    ids = _ids(T, K, N, Z, seed)
    S = T * K
    outs = []
    for which in ("ws", "noalloc"):
        off = torch.full((N + 1,), -7, dtype=torch.int32, device="cuda")
        ss = torch.full((S,), -7, dtype=torch.int32, device="cuda")
        s2r = torch.full((S,), -7, dtype=torch.int32, device="cuda")
        nr = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        if which == "ws":
            ws = torch.empty(zeda.dispatch_workspace_bytes(d), dtype=torch.uint8, device="cuda")
            zeda.zeda_dispatch(d, ids, off, ss, s2r, nr, ws)
        else:
            zeda.zeda_dispatch_noalloc(d, ids, off, ss, s2r, nr)
        torch.cuda.synchronize()
        outs.append((off.cpu().numpy(), ss.cpu().numpy(), s2r.cpu().numpy(), int(nr.item())))
    a, b = outs
    R = a[3]
    assert R == b[3] and 0 < R <= S
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2])
    assert np.array_equal(a[1][:R], b[1][:R]) and (b[1][R:] == -7).all()
    return R


def test_dispatch_noalloc_matches_dispatch_on_two_calls_in_a_row():
    N, Z, K = 128, 32, 8
    _say("zeda_dispatch_noalloc: 65536 slots (segmented form, 32 segments of counts in the static scratch)")
    r1 = _both(8192, K, N, Z, seed=1)
    _say("  real slots", r1, "- then 51200 slots on the same scratch (25 segments: stale counts lie behind them)")
    r2 = _both(6400, K, N, Z, seed=2)
    _say("  real slots", r2, "- then 2400 slots (one-kernel form, no scratch used)")
    r3 = _both(300, K, N, Z, seed=3)
    _say("  real slots", r3)


def test_dispatch_noalloc_rejects_lists_beyond_its_limit():
    lim = zeda.dispatch_noalloc_max_slots()
    assert lim == 524288
    d = zeda.make_desc(lim // 8 + 1, 256, 128, 16, 4, 8, "bf16")
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(zeda.ZedaError) as e:
        zeda.zeda_dispatch_noalloc(d, t, t, t, t, t)
    assert e.value.status == zeda.ZEDA_EUNSUPPORTED
    _say("zeda_dispatch_noalloc: the longest accepted list (", lim, "slots, 256 segments: the whole scratch)")
    _both(lim // 8, 8, 16, 4, seed=4)
