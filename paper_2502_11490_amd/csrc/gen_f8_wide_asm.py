#!/usr/bin/env python3
"""Writes mlp_mfma_f8_wide_asm.inc: the inline-assembly text of one chunk (64 hidden units) of the 8-bit
relevance kernel for 128-wide items, hidden 512 and 256 (mlp_mfma2_f8_wide_kernel in mlp_mfma_f8.hip).

A chunk is two statements: A = layer 1 of its two blocks and their conversion to e4m3 operands, B = layer 2.
Inside a statement nothing of the compiler's can come between an MFMA and the instruction that reads its
result (between two statements it may, say, copy an accumulator, and would read a result that is still on
its way), and the vector-ALU work of the conversion sits between MFMAs, which hide it.  Between A and B the
kernel's own code requests the next chunk's first-layer operands into the registers A has finished with;
they travel while B runs.

Fixed registers of a wave (the vector-ALU instructions name single registers of the tuples):

    v[64:79], v[80:95]      layer-1 accumulators of the even block (set P), pairs c = 0, 1
    v[96:111], v[112:127]   the same for the odd block (set Q)
    v[128:135], v[136:143]  the chunk's 64 hidden units as e4m3 B operands, c = 0, 1 (bytes 0..15: even block)
    v[144:175]              four layer-2 weight fragments in flight from LDS
    compiler's choice       item rows (4 operands), first-layer fragments (4), the 16 layer-2 accumulator
                            tiles (accumulation registers), the LDS address, the clamp constant 448.0

Order of a chunk (A up to "convert Q", then B):
    8 reads      the first four layer-2 fragments are requested at once (they depend on nothing); A ends
                 with a wait for them, long after they have arrived
    P1..P4       layer 1 of the even block: (step 0, c 0), (step 0, c 1), (step 1, c 0), (step 1, c 1)
    Q1, Q2       layer 1 of the odd block begins; two MFMAs have now issued behind P4, so its result is there
    convert P    ReLU, clamp, e4m3 of set P, spread behind Q2, Q3, Q4
    idle         until Q4's result is there (a 16-pass MFMA writes it 64 cycles after issue)
    convert Q    exposed
    layer 2      8 fragments x 2 MFMAs; a fragment's registers are requested again (four fragments ahead)
                 one slot after its MFMAs have issued; counted waits on the in-order LDS counter
The layer-2 accumulators are still being written when B ends: the next statement that touches them is the
next chunk's B (MFMA after MFMA, in order) or, after the last chunk, a statement of idle cycles.
"""
import os

ACC = {"P": (64, 80), "Q": (96, 112)}
H = (128, 136)
FR = 144
NB2 = 8
DRAIN = ["s_nop 15"] * 5


def vr(lo, n):
    return f"v[{lo}:{lo + n - 1}]"


def mfma(dst, a, b):
    return f"v_mfma_f32_32x32x64_f8f6f4 {dst}, {a}, {b}, {dst}"


def l1(s, ks, c):
    return mfma(vr(ACC[s][c], 16), f"%[w{s}{ks}]", f"%[x{c}{ks}]")


def convert(s):
    """ReLU + clamp in place (v_med3_f32 x, 0, 448), then two values per v_cvt_pk_fp8_f32: word w of the
    block's half of the operand takes values 4w .. 4w+3 of the accumulator."""
    half = 0 if s == "P" else 4
    ops = []
    for c in (0, 1):
        a = ACC[s][c]
        for w in range(4):
            ops += [f"v_med3_f32 v{a + 4 * w + e}, v{a + 4 * w + e}, 0, %[fmax]" for e in range(4)]
            d = H[c] + half + w
            ops.append(f"v_cvt_pk_fp8_f32 v{d}, v{a + 4 * w}, v{a + 4 * w + 1}")
            ops.append(f"v_cvt_pk_fp8_f32 v{d}, v{a + 4 * w + 2}, v{a + 4 * w + 3} op_sel:[0,0,1]")
    return ops


def frag_reads(k):
    r = FR + 8 * (k % 4)
    return [f"ds_read_b128 {vr(r, 4)}, %[wc] offset:{k * 2048}", f"ds_read_b128 {vr(r + 4, 4)}, %[wc] offset:{k * 2048 + 1024}"]


def part_a():
    """Layer 1 of both blocks and their conversion; the first four layer-2 fragments are requested first
    and have arrived when the statement ends."""
    out = []
    for k in range(4):
        out += frag_reads(k)
    out.append("s_nop 1")
    out += [l1("P", 0, 0), l1("P", 0, 1), l1("P", 1, 0), l1("P", 1, 1)]
    out += [l1("Q", 0, 0), l1("Q", 0, 1)]
    cp = convert("P")
    third = -(-len(cp) // 3)
    out += cp[:third]
    out.append(l1("Q", 1, 0))
    out += cp[third:2 * third]
    out.append(l1("Q", 1, 1))
    out += cp[2 * third:]
    out += DRAIN
    out += convert("Q")
    out.append("s_waitcnt lgkmcnt(0)")
    return out


def part_b():
    """Layer 2 over the chunk's 64 hidden units.  LDS reads complete in order: fragment k's two reads are
    followed by those of at most two more fragments."""
    out = ["s_nop 1"]
    outstanding = []
    for n2 in range(NB2):
        if n2 >= 4:
            idx = max(i for i, (k, _) in enumerate(outstanding) if k == n2)
            out.append(f"s_waitcnt lgkmcnt({len(outstanding) - 1 - idx})")
            del outstanding[:idx + 1]
        f = vr(FR + 8 * (n2 % 4), 8)
        out.append(mfma(f"%[a{n2}0]", f, vr(H[0], 8)))
        out.append(mfma(f"%[a{n2}1]", f, vr(H[1], 8)))
        # the registers of fragment n2-1 are free once this slot's MFMAs have issued behind its own
        k = n2 - 1 + 4
        if n2 >= 1 and k < NB2:
            out += frag_reads(k)
            outstanding += [(k, 0), (k, 1)]
    return out


def c_string(lines):
    return " \\\n    ".join('"' + l + '\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// Generated by gen_f8_wide_asm.py -- do not edit; see that script for the register plan.", ""]
    out.append(f"#define F8W_ASM_A \\\n    {c_string(part_a())}")
    out.append("")
    out.append(f"#define F8W_ASM_B \\\n    {c_string(part_b())}")
    out.append("")
    for s in "PQ":
        out.append(f'#define F8W_ACC_{s}(v0, v1) [acc{s}0] "+{{{vr(ACC[s][0], 16)}}}"(v0), [acc{s}1] "+{{{vr(ACC[s][1], 16)}}}"(v1)')
    out.append(f'#define F8W_H_OUT(h0, h1) [h0] "=&{{{vr(H[0], 8)}}}"(h0), [h1] "=&{{{vr(H[1], 8)}}}"(h1)')
    out.append(f'#define F8W_H_IN(h0, h1) [h0] "{{{vr(H[0], 8)}}}"(h0), [h1] "{{{vr(H[1], 8)}}}"(h1)')
    for kind, con in (("OUT", "=&"), ("IO", "+")):
        frs = ", ".join(f'[f{k}] "{con}{{{vr(FR + 8 * k, 8)}}}"(f{k})' for k in range(4))
        out.append(f"#define F8W_FRAGS_{kind}(f0, f1, f2, f3) {frs}")
    acc2 = ", ".join(f'[a{n2}{c}] "+a"(acc2[{n2}][{c}])' for n2 in range(NB2) for c in (0, 1))
    out.append(f"#define F8W_ACC2 {acc2}")
    out.append("")
    with open(os.path.join(here, "mlp_mfma_f8_wide_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
