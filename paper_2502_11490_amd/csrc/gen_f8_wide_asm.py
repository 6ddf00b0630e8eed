#!/usr/bin/env python3
"""Writes mlp_mfma_f8_wide_asm.inc: the inline-assembly text of one chunk (64 hidden units) of the 8-bit
relevance kernel for 128-wide items, hidden 512 and 256 (mlp_mfma2_f8_wide_kernel in mlp_mfma_f8.hip).

A chunk is two statements: A = layer 1 of its two blocks and their conversion to e4m3 operands, B = layer 2.
Two more frame a batch: INIT loads the layer-2 bias into the accumulators, HEAD converts the finished layer-2
tiles and runs the head layer.
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
    a[0:255]                the 16 layer-2 accumulator tiles, tile (n2, c) at a[16 (2 n2 + c) ...]: named
                            outright and listed as clobbered, not operands (HEAD reads single registers of a
                            tile, which an operand cannot express; the kernel's own code between the statements
                            has no use for accumulation registers, which a test checks on the compiled kernel)
    compiler's choice       item rows (4 operands), first-layer fragments (4), the head accumulators (2),
                            the LDS addresses, the clamp constant 448.0

Order of a chunk (A up to "convert Q", then B):
    8 reads      the first four layer-2 fragments are requested at once (they depend on nothing); A ends
                 with a wait for them, long after they have arrived
    P1..P4       layer 1 of the even block: (step 0, c 0), (step 0, c 1), (step 1, c 0), (step 1, c 1)
    Q1, Q2       layer 1 of the odd block begins; two MFMAs have now issued behind P4, so its result is there
    convert P    ReLU, clamp, e4m3 of set P, spread behind Q2, Q3, Q4
    convert Q    exposed.  No idle cycles are needed in front of it: an instruction slot of a wave is four
                 clocks (s_nop n takes 4 (n + 1)), a 16-pass MFMA has written its result 19 slots after it
                 issued, and 33 slots lie between Q3 and the first instruction that reads its result (a third
                 of convert P, Q4, another third), 40 between Q4 and the first that reads its (the rest of
                 convert P and the conversion of pair 0)
    layer 2      8 fragments x 2 MFMAs; a fragment's registers are requested again (four fragments ahead)
                 one slot after its MFMAs have issued; counted waits on the in-order LDS counter
The layer-2 accumulators are still being written when B ends: the next statement that touches them is the
next chunk's B (MFMA after MFMA, in order) or, after the last chunk, HEAD, which starts with idle cycles.

INIT: 64 LDS reads straight into the accumulation registers (register 4 t4 + e of a tile is unit
32 n2 + 8 t4 + 4 g + e, so a lane reads 16 bytes at %[b2] (= bias copy + 16 g) + 128 n2 + 32 t4, for both
column blocks); the first A of the batch ends with a full wait on the in-order LDS counter, before any B.

HEAD (after the last chunk; the registers of the hidden units and of the layer-2 fragments are free then):
    v[128:143]              one tile out of the accumulation registers
    v[144:151], v[152:159]  64 layer-2 units as e4m3 B operands, c = 0, 1 (bytes 0..15: the even tile)
    v[160:167], v[168:175]  two head fragments in flight from LDS
per pair p of tiles: four tiles (c, half) x (16 reads, 16 clamps, 8 conversions), then the fragment's two
MFMAs.  The conversion of the next pair starts with 32 instructions that do not write the operands, so they
are rewritten long after the MFMAs that read them have taken them.
"""
import os

NP = 4                  # head fragments: one per 64 layer-2 units
ACC = {"P": (64, 80), "Q": (96, 112)}
H = (128, 136)
FR = 144
NB2 = 8
DRAIN = ["s_nop 15", "s_nop 7"]     # 24 instruction slots: a 16-pass MFMA has written its result after 19


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
    cq = convert("Q")
    # slots between the last MFMA on an accumulator and the first instruction that reads it (see above)
    assert len(cp[third:2 * third]) + 1 + len(cp[2 * third:]) >= 19 and len(cp[2 * third:]) + len(cq) // 2 >= 19
    out += cq
    out.append("s_waitcnt lgkmcnt(0)")
    return out


def acc2_lo(n2, c):
    return 16 * (2 * n2 + c)


def acc2(n2, c):
    return f"a[{acc2_lo(n2, c)}:{acc2_lo(n2, c) + 15}]"


def init_acc2():
    return [f"ds_read_b128 a[{acc2_lo(n2, c) + 4 * t4}:{acc2_lo(n2, c) + 4 * t4 + 3}], %[b2] offset:{n2 * 128 + t4 * 32}"
            for n2 in range(NB2) for c in (0, 1) for t4 in range(4)]


RT, T, HF = 128, (144, 152), (160, 168)


def head():
    # The last chunk's layer 2 is still running: its MFMAs went tile 0 .. 7, and tile n2 is read here
    # 160 n2 / 2 instruction slots in, which is 19 slots behind its last MFMA for every tile.
    out = []
    def frag(p):
        return [f"ds_read_b128 {vr(HF[p % 2], 4)}, %[w3] offset:{p * 2048}",
                f"ds_read_b128 {vr(HF[p % 2] + 4, 4)}, %[w3] offset:{p * 2048 + 1024}"]
    out += frag(0) + frag(1)
    for p in range(NP):
        for c in (0, 1):
            for half in (0, 1):
                lo = acc2_lo(2 * p + half, c)
                out += [f"v_accvgpr_read_b32 v{RT + i}, a{lo + i}" for i in range(16)]
                out += [f"v_med3_f32 v{RT + i}, v{RT + i}, 0, %[fmax]" for i in range(16)]
                for w in range(4):
                    d = T[c] + 4 * half + w
                    out.append(f"v_cvt_pk_fp8_f32 v{d}, v{RT + 4 * w}, v{RT + 4 * w + 1}")
                    out.append(f"v_cvt_pk_fp8_f32 v{d}, v{RT + 4 * w + 2}, v{RT + 4 * w + 3} op_sel:[0,0,1]")
        out.append(f"s_waitcnt lgkmcnt({2 if p + 1 < NP else 0})")   # fragment p is there (p + 1 may be on its way)
        out.append("s_nop 1")
        for c in (0, 1):
            out.append(f"v_mfma_f32_32x32x64_f8f6f4 %[q3{c}], {vr(HF[p % 2], 8)}, {vr(T[c], 8)}, "
                       + ("0" if p == 0 else f"%[q3{c}]"))
        if p + 2 < NP:
            out += frag(p + 2)
    return out + DRAIN


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
        out.append(mfma(acc2(n2, 0), f, vr(H[0], 8)))
        out.append(mfma(acc2(n2, 1), f, vr(H[1], 8)))
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
    out.append(f"#define F8W_ASM_INIT \\\n    {c_string(init_acc2())}")
    out.append("")
    out.append(f"#define F8W_ASM_HEAD \\\n    {c_string(head())}")
    out.append("")
    out.append("#define F8W_ACC2_CLOBBERS " + ", ".join(f'"a{r}"' for r in range(256)))
    out.append("#define F8W_HEAD_CLOBBERS " + ", ".join(f'"v{r}"' for r in range(RT, HF[1] + 8)))
    out.append("")
    with open(os.path.join(here, "mlp_mfma_f8_wide_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
