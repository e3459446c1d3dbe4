"""The LDS reads that the kernels issue through inline asm are ordered by hand-written s_waitcnt lgkmcnt values; a
wrong count reads a register before its data has landed and no test of the results is sure to show it.  This
checks the compiled ISA of every kernel with the static checker (a dataflow over each kernel's control-flow graph),
and the checker itself on small planted cases.  No GPU needed: hipcc cross-compiles."""
import importlib.util
import os
from concurrent.futures import ThreadPoolExecutor

from paper_2605_18643_amd import build as zbuild

_spec = importlib.util.spec_from_file_location("lds_wait_check", os.path.join(os.path.dirname(os.path.abspath(__file__)), "lds_wait_check.py"))
lwc = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(lwc)


def _kernel(body: str) -> str:
    return "k:\n" + body + "\ts_endpgm\n.Lfunc_end0:\n"


def test_checker_flags_a_use_before_the_wait():
    bad = _kernel("\tds_read_b128 v[4:7], v1\n\tv_add_f32_e32 v9, v5, v8\n\ts_waitcnt lgkmcnt(0)\n")
    assert [(n, ln) for n, ln, _ in lwc.check(bad)] == [("k", 3)]
    good = _kernel("\tds_read_b128 v[4:7], v1\n\ts_waitcnt lgkmcnt(0)\n\tv_add_f32_e32 v9, v5, v8\n")
    assert lwc.check(good) == []


def test_checker_counts_reads_in_order():
    # two reads, lgkmcnt(1): the older one has landed, the newer one has not
    asm = _kernel("\tds_read_b128 v[4:7], v1\n\tds_read_b128 v[8:11], v1 offset:16\n\ts_waitcnt lgkmcnt(1)\n"
                  "\tv_mov_b32_e32 v20, v4\n\tv_mov_b32_e32 v21, v8\n\ts_waitcnt lgkmcnt(0)\n")
    assert [ln for _, ln, _ in lwc.check(asm)] == [6]
    # overwriting the destination of a read in flight is as wrong as reading it
    asm = _kernel("\tds_read_b32 v4, v1\n\tv_mov_b32_e32 v4, 0\n\ts_waitcnt lgkmcnt(0)\n")
    assert len(lwc.check(asm)) == 1


def test_checker_follows_branches_and_loops():
    # a read issued at the bottom of a loop body is still in flight at its top
    loop = _kernel("\tds_read_b32 v4, v1\n.LBB0_1:\n\tv_add_u32_e32 v5, v4, v5\n\ts_waitcnt lgkmcnt(0)\n"
                   "\tds_read_b32 v4, v1\n\ts_cbranch_scc1 .LBB0_1\n\ts_waitcnt lgkmcnt(0)\n")
    assert [ln for _, ln, _ in lwc.check(loop)] == [4]
    # a wait on only one of two paths does not cover the join
    diamond = _kernel("\tds_read_b32 v4, v1\n\ts_cbranch_scc1 .LBB0_2\n\ts_waitcnt lgkmcnt(0)\n.LBB0_2:\n"
                      "\tv_mov_b32_e32 v6, v4\n\ts_waitcnt lgkmcnt(0)\n")
    assert [ln for _, ln, _ in lwc.check(diamond)] == [6]


def test_compiled_kernels_never_touch_a_register_with_a_read_in_flight(tmp_path):
    sources = [s for s in zbuild.SOURCES if s != "zeda_api.hip"]  # (host entry points only)

    def one(src):
        path = zbuild.device_isa(src, str(tmp_path / (src + ".s")))
        text = open(path).read()
        assert "s_endpgm" in text
        return src, lwc.check(text)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(one, sources))
    for src, found in results:
        assert found == [], f"{src}: {found[:5]}"
    # the GEMM kernels are the ones with hand-counted waits: make sure they were looked at
    assert any(src == "zeda_ffn.hip" for src, _ in results)
