"""Static check of the kernels' ISA (hipcc -S of this package's own sources): LDS reads issued through inline asm
are invisible to the compiler's wait insertion, so the s_waitcnt lgkmcnt values in the sources carry the whole
burden.  This walks the control-flow graph of every kernel and reports any instruction that touches a VGPR
which an LDS read still in flight is going to write.

LDS operations return in order, so the state is the ordered list of destination register sets of the operations in
flight (oldest first); `s_waitcnt lgkmcnt(n)` retires all but the newest n; states meet aligned at the newest end
(position from the end = number of newer operations), which is sound for counted waits.  Scalar memory loads share
the counter and may return out of order; they only ever make a counted wait stricter than assumed here.

    python lds_wait_check.py file.s [...]      exit status 1 if anything is found
"""
from __future__ import annotations

import re
import sys
from typing import List, Tuple

_VRANGE = re.compile(r"v\[(\d+):(\d+)\]")
_VONE = re.compile(r"(?<![\w\[])v(\d+)\b")
_LABEL = re.compile(r"^(\.LBB\d+_\d+):")
_FUNC = re.compile(r"^([A-Za-z_]\w*):")


def _regs(text: str) -> frozenset:
    out = set()
    for m in _VRANGE.finditer(text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _VONE.finditer(text):
        out.add(int(m.group(1)))
    return frozenset(out)


def _join(a: list, b: list) -> list:
    n = max(len(a), len(b))
    return [(a[-k] if k <= len(a) else frozenset()) | (b[-k] if k <= len(b) else frozenset()) for k in range(n, 0, -1)]


def check(asm: str, keep: int = 64) -> List[Tuple[str, int, str]]:
    """Returns (kernel, line number, instruction) for every instruction that uses a register with a read in flight."""
    text = asm.split("\n")
    funcs, cur = [], None
    for i, line in enumerate(text):
        m = _FUNC.match(line)
        if m:
            cur = [m.group(1), i, None]
            funcs.append(cur)
        if line.startswith(".Lfunc_end") and cur:
            cur[2] = i
            cur = None
    found = []
    for name, a, b in funcs:
        if b is None:
            continue
        ins, labels = [], {}
        for i in range(a + 1, b):
            s = text[i].strip()
            m = _LABEL.match(s)
            if m:
                labels[m.group(1)] = len(ins)
                continue
            if not s or s[0] in ";.":
                continue
            s = s.split(";")[0].strip()
            if s:
                op = s.split()[0]
                ins.append((i + 1, op, s[len(op):]))
        if not any(op.startswith("ds_read") for _, op, _ in ins):
            continue
        leaders = {0} | set(labels.values())
        for k, (_, op, _) in enumerate(ins):
            if op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm"):
                leaders.add(k + 1)
        leaders = sorted(x for x in leaders if x < len(ins))
        blocks = [(s0, leaders[j + 1] if j + 1 < len(leaders) else len(ins)) for j, s0 in enumerate(leaders)]
        block_of = {k: j for j, (s0, e) in enumerate(blocks) for k in range(s0, e)}
        succ = []
        for s0, e in blocks:
            _, op, args = ins[e - 1]
            tgt = re.search(r"(\.LBB\d+_\d+)", args)
            out = []
            if op == "s_branch":
                out = [block_of[labels[tgt.group(1)]]]
            elif op.startswith("s_cbranch"):
                out = [block_of[labels[tgt.group(1)]]] + ([block_of[e]] if e < len(ins) else [])
            elif op != "s_endpgm" and e < len(ins):
                out = [block_of[e]]
            succ.append(out)

        def run(j, state, report):
            s0, e = blocks[j]
            fl = list(state)
            for k in range(s0, e):
                ln, op, args = ins[k]
                if op == "s_waitcnt":
                    m = re.search(r"lgkmcnt\((\d+)\)", args)
                    if m:
                        n = int(m.group(1))
                        fl = [] if n == 0 else fl[max(0, len(fl) - n):]
                    continue
                if report:
                    used = _regs(args)
                    if any(used & p for p in fl):
                        found.append((name, ln, (op + args).strip()))
                if op.startswith("ds_read") or op.startswith("ds_bpermute") or op.startswith("ds_swizzle"):
                    fl.append(_regs(args.split(",")[0]))
                elif op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
                    fl.append(frozenset())
            return fl[-keep:]

        state_in = [[] for _ in blocks]
        work = list(range(len(blocks)))
        while work:
            j = work.pop()
            out = run(j, state_in[j], False)
            for s in succ[j]:
                merged = _join(state_in[s], out)
                if merged != state_in[s]:
                    state_in[s] = merged
                    work.append(s)
        for j in range(len(blocks)):
            run(j, state_in[j], True)
    return found


if __name__ == "__main__":
    bad = 0
    for path in sys.argv[1:]:
        for name, ln, what in check(open(path).read()):
            bad += 1
            if bad <= 40:
                print(f"{path}:{ln}: {name}: {what}")
    print("findings:", bad)
    sys.exit(1 if bad else 0)
