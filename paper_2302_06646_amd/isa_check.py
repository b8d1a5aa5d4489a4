"""Check of the compiled gfx950 assembly for one hazard the hardware does not interlock: a vector-ALU, LDS or
memory instruction that reads the result registers of an MFMA has to issue at least eight issue slots after
that MFMA (`v_mfma_f32_16x16x32_f16`: eight passes).  The compiler inserts `s_nop`s for this, but one build of
the fused backward kernel came out with register copies (`v_mov_b64`) of MFMA results two slots behind the MFMA,
at the fall-through of a conditional branch, and produced wrong gradients; the source was restructured so that no
such copies arise, and every build is now checked: `build()` fails if any kernel shows the pattern.

    python -m paper_2302_06646_amd.isa_check file.s [...]      prints the minimum distance per kernel
"""
from __future__ import annotations

import re
import sys

MIN_SLOTS = 8          # what the compiler keeps for the 16x16x32 f16 MFMA everywhere else
_LOOKAHEAD = 48


def _regs(tok: str) -> set:
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def kernels(asm: str):
    """(name, [instruction lines]) of every function in an AMDGPU assembly text."""
    for m in re.finditer(r"^(\S+):\s*(?:;.*)?\n", asm, re.M):
        name = m.group(1)
        if name.startswith(".") or name.startswith("__hip"):
            continue
        end = asm.find(".Lfunc_end", m.end())
        if end < 0:
            continue
        nxt = re.search(r"^[^.\s;]\S*:\s*$", asm[m.end():end], re.M)
        if nxt:                      # another function label before the end marker: not a function body
            continue
        body = [l.strip() for l in asm[m.end():end].split("\n")]
        yield name, [l for l in body if l and not l.startswith(";")]


def min_mfma_read_distance(body):
    """Smallest number of issue slots between an MFMA and the first non-MFMA instruction that reads its result, over
    the fall-through path and the taken side of every branch met on the way (a few levels deep), and that pair of
    lines (None if no MFMA result is read within reach)."""
    labels = {l[:-1]: i for i, l in enumerate(body) if l.endswith(":")}
    best = [None, None]

    def scan(start, dst, slots, mfma_line, depth):
        j = start
        while j < len(body) and j < start + _LOOKAHEAD and slots < 2 * MIN_SLOTS:
            t = body[j]
            j += 1
            if t.endswith(":"):
                continue             # a label: the fall-through path continues
            op = t.split()[0]
            if op in ("s_endpgm", "s_setpc_b64"):
                return
            if op == "s_nop":
                slots += int(t.split()[1]) + 1
                continue
            if op == "s_branch" or op.startswith("s_cbranch"):
                target = labels.get(t.split()[-1])
                if target is not None and depth < 3:
                    scan(target, dst, slots + 1, mfma_line, depth + 1)
                if op == "s_branch":
                    return
                slots += 1
                continue
            toks = [x.strip() for x in (t.split(None, 1)[1] if " " in t else "").split(",")]
            is_store = op.startswith(("ds_write", "ds_store", "global_store", "scratch_store", "buffer_store"))
            srcs = set()
            for x in (toks if is_store else toks[1:]):
                srcs |= _regs(x.split()[0] if x else "")
            if op.startswith("v_mfma"):
                if _regs(toks[0]) & dst:
                    return           # overwritten or chained as accumulator: MFMA-to-MFMA is interlocked
            elif srcs & dst:
                if best[0] is None or slots < best[0]:
                    best[0], best[1] = slots, (mfma_line, t)
                return
            elif not is_store and toks and toks[0] and _regs(toks[0].split()[0]) >= dst:
                return               # the whole result is overwritten by something else
            slots += 1

    for i, line in enumerate(body):
        if not line.startswith("v_mfma"):
            continue
        ops = [t.strip() for t in line.split(None, 1)[1].split(",")]
        scan(i + 1, _regs(ops[0]), 0, line, 0)
    return best[0], best[1]


def check_text(asm: str):
    """List of (kernel, slots, mfma line, reader line) for every kernel whose minimum is below MIN_SLOTS."""
    bad = []
    for name, body in kernels(asm):
        d, where = min_mfma_read_distance(body)
        if d is not None and d < MIN_SLOTS:
            bad.append((name, d, where[0], where[1]))
    return bad


def check_file(path: str):
    with open(path) as f:
        return check_text(f.read())


if __name__ == "__main__":
    rc = 0
    for p in sys.argv[1:]:
        text = open(p).read()
        for name, body in kernels(text):
            d, where = min_mfma_read_distance(body)
            if d is not None:
                flag = "  <-- HAZARD" if d < MIN_SLOTS else ""
                print(f"{p}: {name[:80]}: {d}{flag}")
                if flag:
                    print("     ", where[0], "->", where[1])
                    rc = 1
    sys.exit(rc)
