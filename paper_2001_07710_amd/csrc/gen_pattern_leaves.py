#!/usr/bin/env python3
"""Generates pattern_leaves.inc: the inner loop of the tiled kernel as inline-assembly text for gfx950.

One block (macro PCONV_ENTRY_LOOP_NF<n>_S<slot>) runs all kept kernels ("entries") that one filter has in the staged
channel chunk.  It is threaded code: for each of the 126 masks with four of nine taps (ascending mask value =
pattern code 0..125) there is one 256-byte-aligned section that

    waits for the entry's activations and weights (LDS reads issued by the previous section),
    starts the LDS read of the next entry's header,
    does the 4*R multiply-adds of its pattern:   acc[kx][r] += w[q] * x[r + ky]   for every kept tap t = 3*ky + kx,
    then fetches the next entry's activations and weights and jumps straight to that entry's section
    (s_setpc to table + code*256), or leaves the loop after the last entry.

So a kept kernel costs one jump and no branch tree, and a wave never diverges: the per-pattern access code of the
paper's section 6.2, emitted for every possible pattern ahead of time.

Entries are read from LDS (the wave copied them there with the chunk); an entry is 8 dwords:
    w0 w1 w2 w3   the four kept weights, taps ascending (fp32)
    header        low half: byte offset of the entry's channel inside the staged chunk, divided by 16;
                  high half: pattern code
    (three unused)

Registers.  Accumulators: 3*R registers per filter slot, fixed, ending at v127 (slot s of a kernel with NF slots
starts at v[128 - 3*R*(s+1)]); the kernel limits the compiler's own budget so that it never allocates them.  Scratch
registers of the loop (activations x0..x11, weights, header, addresses) are fixed too, directly below the
accumulators of the last slot; they are listed as clobbered, so the compiler keeps nothing there across the block.
Scalar scratch: s[60:66].
"""
import sys

TOP = 128   # one past the highest vector register of the kernel (four waves per SIMD on a 512-entry file)
R = 7
LEAF_ALIGN_LOG2 = 8


def masks():
    return [m for m in range(512) if bin(m).count("1") == 4]


def acc_base(slot: int) -> int:
    return TOP - 3 * R * (slot + 1)


class Regs:
    """Fixed scratch registers of a kernel with nf filter slots."""

    def __init__(self, nf: int):
        low = acc_base(nf - 1)
        self.x = (low - 12) & ~1   # x0..x11 (x9..x11 are never read); register tuples start at even registers
        self.w = self.x - 4        # w0..w3
        self.m = self.w - 2        # header: lds_off, joff
        self.va = self.m - 1       # LDS address of the activations
        self.ve = self.m - 2       # LDS address of the next entry
        self.first = self.ve
        self.count = low - self.first


def fetch_next(rg: Regs) -> list:
    """Header of the next entry has arrived: fetch its activations and weights, advance, jump to its section."""
    x, w, m = rg.x, rg.w, rg.m
    return [
        f"v_readfirstlane_b32 s65, v{m}",
        "s_and_b32 s64, s65, 0xffff",
        "s_lshl_b32 s64, s64, 4",
        "s_lshr_b32 s65, s65, 16",
        "s_lshl_b32 s65, s65, 8",
        f"v_add_u32 v{rg.va}, s64, %[vlane]",
        f"ds_read_b128 v[{x}:{x + 3}], v{rg.va}",
        f"ds_read_b128 v[{x + 4}:{x + 7}], v{rg.va} offset:16",
        f"ds_read_b128 v[{x + 8}:{x + 11}], v{rg.va} offset:32",
        f"ds_read_b128 v[{w}:{w + 3}], v{rg.ve}",
        f"v_add_u32 v{rg.ve}, 32, v{rg.ve}",
        "s_add_u32 s62, s60, s65",
        "s_addc_u32 s63, s61, 0",
        "s_setpc_b64 s[62:63]",
    ]


def entry_loop(nf: int, slot: int) -> list:
    rg = Regs(nf)
    base = acc_base(slot)
    m = rg.m
    lines = [
        "s_mov_b32 s66, %[cnt]",
        f"v_mov_b32 v{rg.ve}, %[ventry]",
        "s_getpc_b64 s[60:61]",
        "1:",
        "s_add_u32 s60, s60, 3f-1b",
        "s_addc_u32 s61, s61, 0",
        f"ds_read_b32 v{m}, v{rg.ve} offset:16",
        "s_waitcnt lgkmcnt(0)",
    ] + fetch_next(rg)
    for i, mask in enumerate(masks()):
        lines.append(f".p2align {LEAF_ALIGN_LOG2}")
        if i == 0:
            lines.append("3:")
        lines += [
            "s_waitcnt lgkmcnt(0)",
            f"ds_read_b32 v{m}, v{rg.ve} offset:16",
        ]
        q = 0
        for t in range(9):
            if (mask >> t) & 1:
                ky, kx = divmod(t, 3)
                for r in range(R):
                    lines.append(f"v_fmac_f32 v{base + kx * R + r}, v{rg.w + q}, v{rg.x + r + ky}")
                q += 1
        lines += [
            "s_sub_u32 s66, s66, 1",
            "s_cmp_eq_u32 s66, 0",
            "s_cbranch_scc1 9f",
            "s_waitcnt lgkmcnt(0)",
        ] + fetch_next(rg)
    lines += [f".p2align {LEAF_ALIGN_LOG2}", "9:", "s_waitcnt lgkmcnt(0)"]
    return lines


def as_c_string(lines: list) -> str:
    return " \\\n    ".join('"' + l + '\\n"' for l in lines)


def clobbers(nf: int, slot: int) -> str:
    rg = Regs(nf)
    regs = [f'"v{rg.first + i}"' for i in range(rg.count)] + [f'"v{acc_base(slot) + i}"' for i in range(3 * R)]
    regs += [f'"s{i}"' for i in range(60, 67)] + ['"scc"']
    return ", ".join(regs)


def main(out_path: str):
    out = ["// Generated by gen_pattern_leaves.py -- do not edit.", "",
           f"#define PCONV_LEAF_STRIDE {1 << LEAF_ALIGN_LOG2}   // bytes between the code sections of two patterns", ""]
    for s in range(3):
        b = acc_base(s)
        out.append(f"#define PCONV_ACC_BASE_S{s} {b}")
        out.append(f"#define PCONV_ACC_CLOBBERS_S{s} " + ", ".join(f'"v{b + i}"' for i in range(3 * R)))
        out.append(f"#define PCONV_ACC_ZERO_S{s} " + " ".join(f'"v_mov_b32 v{b + i}, 0\\n"' for i in range(3 * R)))
        out.append(f"#define PCONV_ACC_READ_S{s} " + " ".join(f'"v_mov_b32 %{i}, v{b + i}\\n"' for i in range(3 * R)))
        out.append("")
    for nf in (1, 2, 3):
        out.append(f"#define PCONV_SCRATCH_FIRST_NF{nf} {Regs(nf).first}")
        for s in range(nf):
            out.append(f"#define PCONV_ENTRY_LOOP_NF{nf}_S{s} \\\n    {as_c_string(entry_loop(nf, s))}")
            out.append(f"#define PCONV_ENTRY_LOOP_CLOBBERS_NF{nf}_S{s} {clobbers(nf, s)}")
            out.append("")
    with open(out_path, "w") as fh:
        fh.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "pattern_leaves.inc")
