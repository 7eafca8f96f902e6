"""The generated inner loops (gen_pattern_leaves.py), checked on the CPU by reading the assembly text they emit:

* every code section fits the stride its jump table assumes (a section one instruction too long would shift every
  section behind it, silently);
* the multiply-adds of a section are exactly the sum the method defines for that mask -- acc[kx][r] += w[q] * x[r+ky]
  in the one-column kernel, acc[c+2-kx][r] += w[q] * x[r+ky][c] in the four-column kernel (paper section 6.2: one
  code path per pattern) -- found by executing the text symbolically;
* accumulators, scratch registers and the compiler's registers do not overlap, and every register a block writes is
  in its clobber list.
"""
import importlib.util
import os
import re
from collections import Counter

import pytest

_HERE = os.path.dirname(os.path.abspath(__file__))
_GEN = os.path.join(_HERE, "..", "paper_2001_07710_amd", "csrc", "gen_pattern_leaves.py")
_spec = importlib.util.spec_from_file_location("gen_pattern_leaves", _GEN)
gen = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(gen)


def _literal(tok: str) -> bool:
    """An operand that needs a 32-bit literal after the instruction word (inline constants are -16..64)."""
    tok = tok.strip()
    if tok.startswith("%["):        # a compile-time operand of the asm statement: the chunk mask, an inline constant
        return False
    if re.fullmatch(r"-?\d+", tok):
        return not -16 <= int(tok) <= 64
    if re.fullmatch(r"0x[0-9a-fA-F]+", tok):
        return not 0 <= int(tok, 16) <= 64
    return bool(re.search(r"\d+f-\d+b", tok))      # a label difference


def code_bytes(line: str) -> int:
    """Encoded size of one emitted line (labels and directives: 0)."""
    line = line.strip()
    if not line or line.endswith(":") or line.startswith("."):
        return 0
    op, _, rest = line.partition(" ")
    ops = [o for o in re.split(r",\s*", rest) if o]
    if op.startswith("ds_"):
        return 8
    assert op.startswith(("v_", "s_")), line
    return 4 + (4 if any(_literal(o.split(" ")[0]) for o in ops) else 0)


def sections(lines, align_log2):
    """The code between consecutive alignment directives, in order."""
    out, cur = [], None
    for l in lines:
        if l.strip() == f".p2align {align_log2}":
            if cur is not None:
                out.append(cur)
            cur = []
        elif cur is not None:
            cur.append(l)
    out.append(cur)
    return out


def fmacs(section):
    """(destination, weight register, activation register) of every multiply-add of a section."""
    out = []
    for l in section:
        m = re.fullmatch(r"v_fmac_f32 v(\d+), v(\d+), v(\d+)", l.strip())
        if m:
            out.append(tuple(int(g) for g in m.groups()))
        else:
            assert "fmac" not in l and "v_fma" not in l, l
    return out


def written_vgprs(lines):
    regs = set()
    for l in lines:
        l = l.strip()
        m = re.match(r"(v_fmac_f32|v_mov_b32|v_add_u32) v(\d+),", l)
        if m:
            regs.add(int(m.group(2)))
        m = re.match(r"ds_read_b(32|64|128) v\[?(\d+)(?::(\d+))?\]?,", l)
        if m:
            lo = int(m.group(2))
            hi = int(m.group(3)) if m.group(3) else lo
            regs.update(range(lo, hi + 1))
    return regs


def clobbered(text: str):
    return {int(r) for r in re.findall(r'"v(\d+)"', text)}


@pytest.mark.parametrize("rows8", [False, True])
@pytest.mark.parametrize("nf,slot", [(1, 0), (2, 0), (2, 1)])
def test_one_column_sections(nf, slot, rows8):
    lines = gen.entry_loop(nf, slot, rows8)
    ms = gen.masks()
    assert len(ms) == 255 and ms == sorted(ms)
    secs = sections(lines, gen.LEAF_ALIGN_LOG2)
    # table A, the exit stub, table B, the end label
    assert len(secs) == 2 * len(ms) + 2
    stride = 1 << gen.LEAF_ALIGN_LOG2
    for s in secs:
        assert sum(code_bytes(l) for l in s) <= stride
    rg = gen.Regs(nf)
    base = gen.acc_base(slot)
    for p in (0, 1):
        table = secs[p * (len(ms) + 1):][:len(ms)]
        for mask, sec in zip(ms, table):
            want = Counter()
            q = 0
            for t in range(9):
                if (mask >> t) & 1:
                    ky, kx = divmod(t, 3)
                    if not (rows8 and t >= 6):
                        for r in range(gen.R):
                            want[(base + kx * gen.R + r, rg.w[p] + q, rg.x[p] + r + ky)] += 1
                    q += 1
            assert Counter(fmacs(sec)) == want, (mask, p)
            # what the section requests for the next entry goes to the other register set
            reads = [l for l in sec if l.strip().startswith("ds_read_b128")]
            assert all(f"v[{rg.x[1 - p]}:" in l or f"v[{rg.x[1 - p] + 4}:" in l or f"v[{rg.w[1 - p]}:" in l for l in reads)
    # registers: accumulators on top, scratch below them, all of it above what the compiler may use and clobbered
    accs = set(range(base, base + 3 * gen.R))
    scratch = set(range(rg.first, rg.first + rg.count))
    assert max(accs) < gen.TOP and not (accs & scratch)
    assert rg.first + rg.count == gen.acc_base(nf - 1)
    assert written_vgprs(lines) <= clobbered(gen.clobbers(nf, slot))
    assert written_vgprs(lines) <= accs | scratch


@pytest.mark.parametrize("nf,slot", [(1, 0), (2, 0), (2, 1)])
def test_four_column_sections(nf, slot):
    lines = gen.quad_entry_loop(nf, slot)
    ms = gen.masks()
    secs = sections(lines, gen.QUAD_ALIGN_LOG2)
    assert len(secs) == len(ms) + 1
    stride = 1 << gen.QUAD_ALIGN_LOG2
    for s in secs:
        assert sum(code_bytes(l) for l in s) <= stride
    rg = gen.QuadRegs(nf)
    base = gen.quad_acc_base(slot)
    rq = gen.RQ
    for mask, sec in zip(ms, secs):
        want = Counter()
        q = 0
        for t in range(9):
            if (mask >> t) & 1:
                ky, kx = divmod(t, 3)
                for c in range(4):
                    for r in range(rq):
                        want[(base + 4 * (c + 2 - kx) + r, rg.w + q, rg.x + 4 * (r + ky) + c)] += 1
                q += 1
        assert Counter(fmacs(sec)) == want, mask
        assert sum(want.values()) == 16 * bin(mask).count("1")
    accs = set(range(base, base + 6 * rq))
    scratch = set(range(rg.first, rg.first + rg.count))
    assert max(accs) < gen.TOP and not (accs & scratch)
    assert rg.first + rg.count == gen.quad_acc_base(nf - 1)
    assert written_vgprs(lines) <= clobbered(gen.quad_clobbers(nf, slot))
    assert written_vgprs(lines) <= accs | scratch
    # the patch rows are where the kernel's LDS tile has them: 64 lanes x 16 bytes apart
    first_fetch = [l for l in lines[:40] if l.strip().startswith("ds_read_b128") and f"v{rg.va}" in l]
    assert [int(re.search(r"offset:(\d+)", l).group(1)) for l in first_fetch] == [i * 1024 for i in range(rq + 2)]
    assert gen.QUAD_CH_BYTES == (rq + 2) * 1024


def test_every_four_tap_pattern_of_the_paper_has_a_section():
    ms = gen.masks()
    four = [m for m in ms if bin(m).count("1") == 4]
    assert len(four) == 126                       # C(9,4): every pattern a library can hold (section 4.1)
    assert len(set(ms)) == len(ms) == 255         # plus the fragments of stride-2 layers: 9 + 36 + 84
    # the rank of a mask among them is the section number the packer stores (mask_rank in pconv_host.cpp)
    assert [ms.index(m) for m in (1, 2, 3, 511 - 0b111110000)] == [0, 1, 2, ms.index(15)]
