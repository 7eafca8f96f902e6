#!/usr/bin/env python3
"""Generates pattern_leaves.inc: the inner loop of the tiled kernel as inline-assembly text for gfx950.

One block (macro PCONV_ENTRY_LOOP_NF<n>_S<slot>) runs all kept kernels ("entries") that one filter has in the staged
channel chunk.  It is threaded code, software-pipelined one entry deep over two register sets A and B: for each of
the 255 masks with one to four of nine taps (ascending mask value = pattern code 0..254) there are two 256-byte-aligned
sections, one per register set.  The section of entry i (set P, the other set is Q)

    waits for what the section before it requested: activations and weights of entry i (in P), header of entry i+1,
    requests from LDS the activations and weights of entry i+1 (into Q) and the header of entry i+2,
    does the 4*R multiply-adds of its pattern on P:   acc[kx][r] += w[q] * x[r + ky]   for every kept tap t = 3*ky + kx,
    and jumps straight to the section of entry i+1's pattern for set Q (s_setpc to table_Q + section offset).

So a kept kernel costs one jump and no branch tree, a wave never diverges, and the LDS latency of an entry is covered
by the multiply-adds of the entry before it: the per-pattern access code of the paper's section 6.2, emitted for
every possible pattern ahead of time.

Entries are read from LDS, where the wave put them when it staged the chunk; an entry is 8 dwords:
    w0 w1 w2 w3   the four kept weights, taps ascending (fp32)
    header        two words, ready to use: the byte offset of the pattern's section in a table (code * 256) and the
                  byte offset of the entry's channel in the staged chunk (the kernel derives both from the packed
                  header — channel index in bits 0..7, pattern code above — when it copies the entries to LDS)
    (two unused)
There is no counter: behind a filter's last entry the kernel writes a header whose section number is 255, one past
the last mask, and slot 255 of either table leaves the loop.  The section of the last entry has then already
requested "entry" 255's weights, patch (channel offset 0) and the header behind it; nothing uses them, and all of it
lies inside the LDS region the kernel reserves for a filter's entries (chunk size + 2 of them).

The four-column loop (further down) keeps the packed header (one word, decoded in the section) and a counter: there
the same change measured 2 % slower.

Registers.  Accumulators: 3*R registers per filter slot, fixed, ending at v127 (slot s of a kernel with NF slots
starts at v[128 - 3*R*(s+1)]); the kernel limits the compiler's own budget so that it never allocates them.  Scratch
registers of the loop (activations x0..x8 and weights of both sets, header pair, addresses) are fixed too, directly below
the accumulators of the last slot; they are listed as clobbered, so the compiler keeps nothing there across the
block.  Scalar scratch: s[58:66].
"""
import sys

TOP = 128   # one past the highest vector register of the kernel (four waves per SIMD on a 512-entry file)
R = 7
LEAF_ALIGN_LOG2 = 8
CH_BYTES = 64 * 12 * 4   # one staged channel in LDS: 64 lanes x 12 patch rows


def masks():
    """Every mask a kept kernel can have: one to four of the nine taps.  Four-tap masks are the paper's patterns;
    masks with fewer taps come from stride-2 layers, which run as stride-1 layers over the four row/column parity
    planes of the input, where a four-tap kernel falls apart into up to four kernels with fewer taps."""
    return [m for m in range(1, 512) if 1 <= bin(m).count("1") <= 4]


def acc_base(slot: int) -> int:
    return TOP - 3 * R * (slot + 1)


class Regs:
    """Fixed scratch registers of a kernel with nf filter slots."""

    def __init__(self, nf: int):
        low = acc_base(nf - 1)
        xa = (low - 10) & ~1            # register tuples start at even registers
        self.x = (xa, xa - 10)          # x0..x8 of each set; the tenth register of each block of ten holds an address
        self.va = xa + 9                # LDS address of the activations
        self.ve = xa - 1                # LDS address of the next entry
        self.w = (xa - 14, xa - 18)     # w0..w3 of each set
        self.m = xa - 20                # header of the entry after the next: section offset, channel offset (even pair)
        self.first = self.m
        self.count = low - self.first


def request_next(rg: Regs, q: int, rows8: bool = False) -> list:
    """The header of the next entry is in v[m:m+1] — the byte offset of its code section in a table and the byte
    offset of its channel in the LDS tile, as the kernel wrote them when it staged the entries: request that entry's
    activations and weights into set q and the header of the entry after it.  Leaves the next entry's section offset
    in s65.  rows8: the layer's kernels only have taps in their first two rows (a stride-2 layer over parity planes),
    so patch row 8 is never read and is not fetched."""
    x, w = rg.x[q], rg.w[q]
    lines = [
        f"v_readfirstlane_b32 s65, v{rg.m}",
        f"v_add_u32 v{rg.va}, v{rg.m + 1}, %[vlane]",
        f"ds_read_b128 v[{x}:{x + 3}], v{rg.va}",
        f"ds_read_b128 v[{x + 4}:{x + 7}], v{rg.va} offset:16",
        f"ds_read_b32 v{x + 8}, v{rg.va} offset:32",
        f"ds_read_b128 v[{w}:{w + 3}], v{rg.ve}",
        f"ds_read_b64 v[{rg.m}:{rg.m + 1}], v{rg.ve} offset:48",
        f"v_add_u32 v{rg.ve}, 32, v{rg.ve}",
    ]
    if rows8:
        lines = [l for l in lines if not l.startswith(f"ds_read_b32 v{x + 8},")]
    return lines


def jump(q: int) -> list:
    base = 60 if q == 0 else 58
    return [
        f"s_add_u32 s62, s{base}, s65",
        f"s_addc_u32 s63, s{base + 1}, 0",
        "s_setpc_b64 s[62:63]",
    ]


def entry_loop(nf: int, slot: int, rows8: bool = False) -> list:
    rg = Regs(nf)
    base = acc_base(slot)
    ms = masks()
    table_b = (len(ms) + 1) << LEAF_ALIGN_LOG2          # the exit stub sits between the two tables
    lines = [
        f"v_mov_b32 v{rg.ve}, %[ventry]",
        "s_getpc_b64 s[60:61]",
        "1:",
        "s_add_u32 s60, s60, 3f-1b",                   # s[60:61]: sections of set A
        "s_addc_u32 s61, s61, 0",
        f"s_add_u32 s58, s60, {table_b}",              # s[58:59]: sections of set B
        "s_addc_u32 s59, s61, 0",
        f"ds_read_b64 v[{rg.m}:{rg.m + 1}], v{rg.ve} offset:16",
        "s_waitcnt lgkmcnt(0)",
    ] + request_next(rg, 0, rows8) + jump(0)
    for p in (0, 1):
        for i, mask in enumerate(ms):
            lines.append(f".p2align {LEAF_ALIGN_LOG2}")
            if p == 0 and i == 0:
                lines.append("3:")
            lines.append("s_waitcnt lgkmcnt(0)")
            lines += request_next(rg, 1 - p, rows8)
            q = 0
            for t in range(9):
                if rows8 and t >= 6 and (mask >> t) & 1:
                    continue       # never packed for such a layer; the section stays as a placeholder of its slot
                if (mask >> t) & 1:
                    ky, kx = divmod(t, 3)
                    for r in range(R):
                        lines.append(f"v_fmac_f32 v{base + kx * R + r}, v{rg.w[p] + q}, v{rg.x[p] + r + ky}")
                    q += 1
            lines += jump(1 - p)
        if p == 0:
            # slot EXIT_CODE of table A: where the header behind a filter's last entry sends a section of set B
            lines += [f".p2align {LEAF_ALIGN_LOG2}", "s_waitcnt lgkmcnt(0)", "s_branch 8f"]
    # slot EXIT_CODE of table B is the end of the block (the fetches for the entry that is not there must land first)
    lines += [f".p2align {LEAF_ALIGN_LOG2}", "8:", "s_waitcnt lgkmcnt(0)"]
    return lines


# ---------------------------------------------------------------------------------------------------------------
# The "quad" kernel: a lane holds FOUR neighbouring input columns of RQ + 2 input rows (six 128-bit LDS reads) and
# accumulates RQ = 4 output rows of SIX output columns: a tap (ky,kx) on input column c (0..3) belongs to output
# column c + 1 - kx relative to the quad, i.e. to accumulator column j = c + 2 - kx (0..5); columns 0 and 5 are
# handed to the neighbouring lanes once, after the last channel.  16 multiply-adds per tap, 64 per kept kernel and
# jump instead of 28: the jump, whose instruction refetch is what the one-column kernel waits for most, is paid less
# than half as often.  One register set (the patch is 24 registers); sections are 512 bytes apart.
# ---------------------------------------------------------------------------------------------------------------
RQ = 4
QUAD_ALIGN_LOG2 = 9
QUAD_ROW_BYTES = 64 * 16          # one patch row of a channel in LDS: 64 lanes x four columns
QUAD_CH_BYTES = (RQ + 2) * QUAD_ROW_BYTES


def quad_acc_base(slot: int) -> int:
    return TOP - 6 * RQ * (slot + 1)


class QuadRegs:
    def __init__(self, nf: int):
        low = quad_acc_base(nf - 1)
        self.x = (low - 4 * (RQ + 2)) & ~1      # x[i][c] = x + 4*i + c
        self.w = self.x - 4
        self.m = self.w - 1
        self.va = self.w - 2
        self.ve = self.w - 3
        self.first = self.ve
        self.count = low - self.first


def quad_fetch(rg: QuadRegs) -> list:
    """The header of the next entry is in v[m]: fetch its patch and weights and the header after it; section offset
    of the next entry in s65."""
    lines = [
        f"v_readfirstlane_b32 s65, v{rg.m}",
        "s_and_b32 s64, s65, %[ccmask]",
        f"s_mul_i32 s64, s64, {QUAD_CH_BYTES}",
        f"v_add_u32 v{rg.va}, s64, %[vlane]",
    ]
    for i in range(RQ + 2):
        lines.append(f"ds_read_b128 v[{rg.x + 4 * i}:{rg.x + 4 * i + 3}], v{rg.va} offset:{i * QUAD_ROW_BYTES}")
    lines += [
        f"ds_read_b128 v[{rg.w}:{rg.w + 3}], v{rg.ve}",
        f"ds_read_b32 v{rg.m}, v{rg.ve} offset:48",
        f"v_add_u32 v{rg.ve}, 32, v{rg.ve}",
        "s_and_b32 s65, s65, 0xffffff00",
        "s_lshl_b32 s65, s65, 1",
        "s_add_u32 s62, s60, s65",
        "s_addc_u32 s63, s61, 0",
        "s_setpc_b64 s[62:63]",
    ]
    return lines


def quad_entry_loop(nf: int, slot: int) -> list:
    rg = QuadRegs(nf)
    base = quad_acc_base(slot)
    ms = masks()
    lines = [
        "s_sub_u32 s66, %[cnt], 1",
        f"v_mov_b32 v{rg.ve}, %[ventry]",
        "s_getpc_b64 s[60:61]",
        "1:",
        "s_add_u32 s60, s60, 3f-1b",                              # s[60:61]: the sections
        "s_addc_u32 s61, s61, 0",
        f"s_add_u32 s56, s60, {len(ms) << QUAD_ALIGN_LOG2}",       # s[56:57]: behind the last section
        "s_addc_u32 s57, s61, 0",
        f"ds_read_b32 v{rg.m}, v{rg.ve} offset:16",
        "s_waitcnt lgkmcnt(0)",
    ] + quad_fetch(rg)
    for i, mask in enumerate(ms):
        lines.append(f".p2align {QUAD_ALIGN_LOG2}")
        if i == 0:
            lines.append("3:")
        lines.append("s_waitcnt lgkmcnt(0)")
        q = 0
        for t in range(9):
            if (mask >> t) & 1:
                ky, kx = divmod(t, 3)
                for c in range(4):
                    for r in range(RQ):
                        lines.append(f"v_fmac_f32 v{base + 4 * (c + 2 - kx) + r}, v{rg.w + q}, v{rg.x + 4 * (r + ky) + c}")
                q += 1
        lines += [
            "s_sub_u32 s66, s66, 1",                               # borrow: this was the last entry
            "s_cbranch_scc0 2f",
            "s_setpc_b64 s[56:57]",
            "2:",
        ] + quad_fetch(rg)
    lines += [f".p2align {QUAD_ALIGN_LOG2}", "s_waitcnt lgkmcnt(0)"]
    return lines


def quad_clobbers(nf: int, slot: int) -> str:
    rg = QuadRegs(nf)
    regs = [f'"v{rg.first + i}"' for i in range(rg.count)] + [f'"v{quad_acc_base(slot) + i}"' for i in range(6 * RQ)]
    regs += [f'"s{i}"' for i in range(56, 67)] + ['"scc"']
    return ", ".join(regs)


def as_c_string(lines: list) -> str:
    return " \\\n    ".join('"' + l + '\\n"' for l in lines)


def clobbers(nf: int, slot: int) -> str:
    rg = Regs(nf)
    regs = [f'"v{rg.first + i}"' for i in range(rg.count)] + [f'"v{acc_base(slot) + i}"' for i in range(3 * R)]
    regs += [f'"s{i}"' for i in range(58, 66)] + ['"scc"']
    return ", ".join(regs)


def main(out_path: str):
    out = ["// Generated by gen_pattern_leaves.py -- do not edit.", "",
           f"#define PCONV_LEAF_STRIDE {1 << LEAF_ALIGN_LOG2}   // bytes between the code sections of two patterns",
           f"#define PCONV_EXIT_CODE {len(masks())}   // section slot behind the last mask: leaves the entry loop",
           f"#define PCONV_CH_BYTES {CH_BYTES}", ""]
    for s in range(3):
        b = acc_base(s)
        out.append(f"#define PCONV_ACC_BASE_S{s} {b}")
        out.append(f"#define PCONV_ACC_CLOBBERS_S{s} " + ", ".join(f'"v{b + i}"' for i in range(3 * R)))
        out.append(f"#define PCONV_ACC_ZERO_S{s} " + " ".join(f'"v_mov_b32 v{b + i}, 0\\n"' for i in range(3 * R)))
        out.append(f"#define PCONV_ACC_READ_S{s} " + " ".join(f'"v_mov_b32 %{i}, v{b + i}\\n"' for i in range(3 * R)))
        out.append("")
    for nf in (1, 2):
        out.append(f"#define PCONV_SCRATCH_FIRST_NF{nf} {Regs(nf).first}")
        for s in range(nf):
            out.append(f"#define PCONV_ENTRY_LOOP_NF{nf}_S{s} \\\n    {as_c_string(entry_loop(nf, s))}")
            out.append(f"#define PCONV_ENTRY_LOOP_ROWS8_NF{nf}_S{s} \\\n    {as_c_string(entry_loop(nf, s, True))}")
            out.append(f"#define PCONV_ENTRY_LOOP_CLOBBERS_NF{nf}_S{s} {clobbers(nf, s)}")
            out.append("")
    out.append(f"#define PCONV_QUAD_ROWS {RQ}")
    out.append(f"#define PCONV_QUAD_CH_BYTES {QUAD_CH_BYTES}")
    for s in range(2):
        b = quad_acc_base(s)
        n = 6 * RQ
        out.append(f"#define PCONV_QUAD_ACC_BASE_S{s} {b}")
        out.append(f"#define PCONV_QUAD_ACC_CLOBBERS_S{s} " + ", ".join(f'"v{b + i}"' for i in range(n)))
        out.append(f"#define PCONV_QUAD_ACC_ZERO_S{s} " + " ".join(f'"v_mov_b32 v{b + i}, 0\\n"' for i in range(n)))
        out.append(f"#define PCONV_QUAD_ACC_READ_S{s} " + " ".join(f'"v_mov_b32 %{i}, v{b + i}\\n"' for i in range(n)))
        for r in range(RQ):      # output row r of the six accumulator columns
            out.append(f"#define PCONV_QUAD_ACC_READ_ROW_S{s}_R{r} " +
                       " ".join(f'"v_mov_b32 %{j}, v{b + 4 * j + r}\\n"' for j in range(6)))
        out.append("")
    for nf in (1, 2):
        out.append(f"#define PCONV_QUAD_SCRATCH_FIRST_NF{nf} {QuadRegs(nf).first}")
        for s in range(nf):
            out.append(f"#define PCONV_QUAD_ENTRY_LOOP_NF{nf}_S{s} \\\n    {as_c_string(quad_entry_loop(nf, s))}")
            out.append(f"#define PCONV_QUAD_ENTRY_LOOP_CLOBBERS_NF{nf}_S{s} {quad_clobbers(nf, s)}")
            out.append("")
    with open(out_path, "w") as fh:
        fh.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "pattern_leaves.inc")
