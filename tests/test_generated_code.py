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


def test_one_column_loop_ends_through_the_exit_slot():
    """No counter: the header the kernel writes behind a filter's last entry carries section number 255, and slot 255
    of both tables leaves the loop after waiting for the fetches in flight.  Every section proper ends in the
    computed jump, and fetches the next header as a pair (section offset, channel offset) into an even register."""
    n = len(gen.masks())
    for nf, slot in [(1, 0), (2, 0), (2, 1)]:
        for rows8 in (False, True):
            secs = sections(gen.entry_loop(nf, slot, rows8), gen.LEAF_ALIGN_LOG2)
            rg = gen.Regs(nf)
            assert rg.m % 2 == 0
            assert [l.strip() for l in secs[n]] == ["s_waitcnt lgkmcnt(0)", "s_branch 8f"]          # table A, slot 255
            assert [l.strip() for l in secs[2 * n + 1]] == ["8:", "s_waitcnt lgkmcnt(0)"]            # table B, slot 255
            for p in (0, 1):
                for sec in secs[p * (n + 1):][:n]:
                    body = [l.strip() for l in sec if not l.strip().endswith(":")]
                    assert body[0] == "s_waitcnt lgkmcnt(0)" and body[-1] == "s_setpc_b64 s[62:63]"
                    assert body[-3] == f"s_add_u32 s62, s{58 if p == 0 else 60}, s65"                # the other table
                    assert not any(l.startswith(("s_cbranch", "s_branch", "s_sub")) for l in body)
                    assert f"ds_read_b64 v[{rg.m}:{rg.m + 1}], v{rg.ve} offset:48" in body
                    assert f"v_add_u32 v{rg.va}, v{rg.m + 1}, %[vlane]" in body


class _Machine:
    """Runs an emitted entry loop on a model of what it touches: scalar and vector registers of one lane, LDS as a
    dictionary of dwords, the section tables as (table base, slot).  Loads complete at once (every use in the text
    is behind an s_waitcnt).  Records, per multiply-add, where its operands were loaded from."""

    def __init__(self, lines, align_log2):
        self.stride = 1 << align_log2
        self.prog, self.slots = [], {}
        # address of every line: the preamble from 0, then sections on multiples of the stride
        first = next(i for i, l in enumerate(lines) if l.strip() == f".p2align {align_log2}")
        self.preamble = [l.strip() for l in lines[:first]]
        secs = sections(lines, align_log2)
        self.secs = [[l.strip() for l in sec] for sec in secs]

    def run(self, lds, vlane, ventry, cnt=None, ccmask=None, max_steps=200):
        v, sreg = {}, {}
        scc = 0
        trace = []           # (slot index in the run of sections, list of (dst, weight source, activation source))
        src = {}             # vector register -> LDS address it was last loaded from
        here = ("pre", 0)
        steps = 0

        def vec(tok):
            tok = tok.strip()
            if tok == "%[vlane]":
                return vlane
            if tok == "%[ventry]":
                return ventry
            if tok.startswith("v"):
                return v[int(tok[1:])]
            return sca(tok)

        def sca(tok):
            tok = tok.strip()
            if tok == "%[cnt]":
                return cnt
            if tok == "%[ccmask]":
                return ccmask
            if re.fullmatch(r"s\d+", tok):
                return sreg[tok]
            return int(tok, 0)

        code = self.preamble
        idx = 0
        fm = []
        while True:
            steps += 1
            assert steps < max_steps * 200, "the loop does not end"
            if idx >= len(code):
                # fell off a section: only the last one may (the end of the block)
                assert here[0] == "sec" and here[1] == len(self.secs) - 1, here
                trace.append((here[1], fm))
                return trace
            l = code[idx]
            idx += 1
            if not l or l.endswith(":") or l.startswith("s_waitcnt") or l.startswith("s_getpc"):
                continue
            op, _, rest = l.partition(" ")
            a = [t.strip() for t in rest.split(",")]
            if op == "v_mov_b32":
                v[int(a[0][1:])] = vec(a[1])
            elif op == "v_add_u32":
                v[int(a[0][1:])] = vec(a[1]) + vec(a[2])
            elif op == "v_readfirstlane_b32":
                sreg[a[0]] = v[int(a[1][1:])]
                assert isinstance(sreg[a[0]], int), "a header that nobody wrote decides a jump or an address"
            elif op.startswith("ds_read_b"):
                m = re.fullmatch(r"v\[?(\d+)(?::(\d+))?\]?", a[0])
                lo = int(m.group(1))
                hi = int(m.group(2)) if m.group(2) else lo
                tail = a[1].split()
                addr = v[int(tail[0][1:])] + (int(tail[1].split(":")[1]) if len(tail) > 1 else 0)
                for k in range(hi - lo + 1):
                    v[lo + k] = lds.get(addr + 4 * k, ("junk", addr + 4 * k))
                    src[lo + k] = addr + 4 * k
            elif op == "v_fmac_f32":
                fm.append((int(a[0][1:]), src[int(a[1][1:])], src[int(a[2][1:])]))
            elif op == "s_add_u32" and a[0] == "s60":
                sreg["s60"] = 0          # s[60:61] = the first table: address 0 of the model
            elif op == "s_add_u32":
                sreg[a[0]] = sca(a[1]) + sca(a[2])
            elif op == "s_addc_u32":
                continue
            elif op == "s_sub_u32":
                x, y = sca(a[1]), sca(a[2])
                scc = 1 if x < y else 0
                sreg[a[0]] = (x - y) & 0xFFFFFFFF
            elif op == "s_and_b32":
                sreg[a[0]] = sca(a[1]) & sca(a[2])
            elif op == "s_mul_i32":
                sreg[a[0]] = sca(a[1]) * sca(a[2])
            elif op == "s_lshl_b32":
                sreg[a[0]] = sca(a[1]) << sca(a[2])
            elif op in ("s_cbranch_scc0", "s_cbranch_scc1"):
                if scc == (1 if op.endswith("1") else 0):
                    assert a[0].endswith("f")
                    idx = code.index(a[0][:-1] + ":", idx)
            elif op == "s_setpc_b64":
                target = sreg["s" + a[0][2:a[0].index(":")]]
                assert isinstance(target, int) and target % self.stride == 0, target
                if here[0] == "sec":
                    trace.append((here[1], fm))
                fm = []
                here = ("sec", target // self.stride)
                assert here[1] < len(self.secs), here
                code, idx = self.secs[here[1]], 0
            elif op == "s_branch":
                assert a[0] == "8f"
                trace.append((here[1], fm))
                fm = []
                here = ("sec", len(self.secs) - 1)
                code, idx = self.secs[-1], 0
            else:
                raise AssertionError("instruction the model does not know: " + l)


@pytest.mark.parametrize("kind", ["one_column", "one_column_rows8", "four_column"])
def test_entry_loops_run_every_entry_once_and_stop(kind):
    """The emitted loops, executed on a model: for entry lists of several lengths from 1 to the chunk size — with the
    header pair and the end marker the kernel writes (one-column loop), or the packer's header and a count
    (four-column loop) — the sections visited are the entries' patterns in order (sets A and B alternating in the
    one-column loop), every multiply-add of entry i takes its weight from entry i's slot and its activation from
    entry i's channel, whatever stands behind the last entry is never used as a jump target, and the loop leaves
    through slot 255."""
    import random
    rnd = random.Random(5)
    ms = gen.masks()
    n = len(ms)
    quad = kind == "four_column"
    for nf, slot in [(1, 0), (2, 1)]:
        lines = gen.quad_entry_loop(nf, slot) if quad else gen.entry_loop(nf, slot, kind.endswith("rows8"))
        align = gen.QUAD_ALIGN_LOG2 if quad else gen.LEAF_ALIGN_LOG2
        ch_bytes = gen.QUAD_CH_BYTES if quad else gen.CH_BYTES
        m = _Machine(lines, align)
        vlane, ventry, cc = 7 * 48, 1 << 20, 16 if quad else 32
        for count in list(range(1, 6)) + [cc - 1, cc]:
            usable = [i for i, mk in enumerate(ms) if not (kind.endswith("rows8") and mk >> 6)]
            codes = [rnd.choice(usable) for _ in range(count)]
            chans = [rnd.randrange(cc) for _ in range(count)]
            lds = {}
            for i in range(count + 1):
                last = i == count
                if quad:      # the header as the packer stores it; the loop counts (nothing stands behind the last)
                    if not last:
                        lds[ventry + 32 * i + 16] = chans[i] | (codes[i] << 8)
                else:         # the header pair and the end marker the kernel writes when it stages the entries
                    lds[ventry + 32 * i + 16] = (n if last else codes[i]) << align
                    lds[ventry + 32 * i + 20] = 0 if last else chans[i] * ch_bytes
                for q in range(4):
                    lds[ventry + 32 * i + 4 * q] = ("w", i, q)
            trace = m.run(lds, vlane, ventry, cnt=count, ccmask=cc - 1)
            visited = [t[0] for t in trace]
            if quad:
                assert visited == codes + [n]
            else:
                want = [c + (n + 1) * (i % 2) for i, c in enumerate(codes)]
                # the exit slot of the table that was next, then (from table A's stub) the end of the block
                end = [n, 2 * n + 1] if count % 2 == 0 else [2 * n + 1]
                assert visited == want + end, (count, visited, want)
            for i, (sec, fm) in enumerate(trace[:count]):
                taps = bin(ms[codes[i]]).count("1")
                assert len(fm) == taps * (16 if quad else gen.R)
                for dst, wsrc, xsrc in fm:
                    assert ventry + 32 * i <= wsrc < ventry + 32 * i + 16
                    assert vlane + chans[i] * ch_bytes <= xsrc < vlane + (chans[i] + 1) * ch_bytes
            assert all(not fm for _, fm in trace[count:])


def test_every_four_tap_pattern_of_the_paper_has_a_section():
    ms = gen.masks()
    four = [m for m in ms if bin(m).count("1") == 4]
    assert len(four) == 126                       # C(9,4): every pattern a library can hold (section 4.1)
    assert len(set(ms)) == len(ms) == 255         # plus the fragments of stride-2 layers: 9 + 36 + 84
    # the rank of a mask among them is the section number the packer stores (mask_rank in pconv_host.cpp)
    assert [ms.index(m) for m in (1, 2, 3, 511 - 0b111110000)] == [0, 1, 2, ms.index(15)]
