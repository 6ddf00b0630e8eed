#!/usr/bin/env python3
"""Writes mlp_mfma_stream_asm.inc: the inline-assembly text of one pipeline step of the streaming
MFMA relevance kernel (mlp_mfma_stream.hip), for item width 128 (8 layer-1 fragments per step) and
second hidden width 256 (16 layer-2 fragments per step), 64 pairs per wave.

Register plan of a wave (fixed physical registers, so that the vector-ALU instructions that turn
fresh layer-1 accumulators into bf16 B operands can be interleaved with the MFMAs of layer 2 and
so that every variant of the step agrees on where the long-lived values are):

    256 AGPRs           layer-2 accumulators, 16 tiles (n2, c), constraint "a" (the allocator's choice)
    v[64:95], v[96:127] layer-1 accumulators, sets A and B (pairs c = 0, 1), alternating by step
    v[128:143]          hidden units produced from set A, tuple (c, half) at v[128 + 8c + 4half ...]
    v[144:159]          hidden units produced from set B
    compiler's choice   the 16 item-row operands, four weight fragments, the LDS address

Step variants:  FIRST  layer 1 only (set A), conversion exposed
                MID_A  layer 1 into set A, layer 2 with the hidden units of set B, conversion of
                       set A interleaved with the layer-2 MFMAs;  MID_B the mirror image
                LAST   layer 2 only, with the hidden units of set B

Global loads of a step and their waits are part of the assembly too, because the compiler cannot
count them: next to global-to-LDS loads any other vector-memory load makes it fall back to waiting
for ALL outstanding loads, the weight chunks included (and it treats every LDS access it sees as
depending on them).  A block therefore
    - first issues the N_DMA global-to-LDS loads of the weight chunk two steps ahead (scalar base
      %[sb<t>] + lane offset %[vo]; LDS base in M0, 4 KB further per load);
    - then loads the user term of the NEXT layer-1 block straight into the accumulator set that
      is idle during this step (8 loads), then one 16-byte piece of the next batch's item rows;
    - before its first layer-1 MFMA waits for its own user term, loaded one step earlier: the
      counter is in order, and younger than that term are the piece fetched after it and this
      step's own loads;
    - at the end waits until only this step's own loads are outstanding (then the chunk the next
      step reads has landed, and so has the piece fetched one step ago), stores that piece to the
      wave's LDS area, waits for the store and joins the workgroup barrier.

Run this script after changing it; the .inc file is committed next to it.
"""
import os

ACC = {"A": (64, 80), "B": (96, 112)}       # first register of the c = 0 / c = 1 accumulator
HF = {"A": 128, "B": 144}                   # first register of the four (c, half) tuples
N_DMA = 6                                   # global-to-LDS loads per step: 6 x 256 lanes x 16 B = one chunk


def vr(lo, n):
    return f"v[{lo}:{lo + n - 1}]"


def acc_reg(s, c):
    return vr(ACC[s][c], 16)


def hf_reg(s, c, half):
    return vr(HF[s] + 8 * c + 4 * half, 4)


def acc2_reg(n2, c):
    return f"%[a{n2}{c}]"  # layer-2 accumulators: any AGPR tuple, the allocator keeps them in place


def ld(buf, frag):
    return f"ds_read_b128 %[{buf}], %[wc] offset:{frag * 1024}"


def wt(n):
    return f"s_waitcnt lgkmcnt({n})"


def m1(s, buf, k):
    return [f"v_mfma_f32_32x32x16_bf16 {acc_reg(s, c)}, %[{buf}], %[x{c}{k}], {acc_reg(s, c)}" for c in (0, 1)]


def m2(hs, buf, n2, s2):
    return [f"v_mfma_f32_32x32x16_bf16 {acc2_reg(n2, c)}, %[{buf}], {hf_reg(hs, c, s2)}, {acc2_reg(n2, c)}"
            for c in (0, 1)]


def convert_ops(s):
    """ReLU + bf16 rounding of accumulator set s into its hidden-unit tuples: per packed word one
    v_cvt_pk_bf16_f32 and one signed 16-bit max with 0 (bf16 bit patterns: negative = sign bit)."""
    ops = []
    for c in (0, 1):
        for half in (0, 1):
            cv, mx = [], []
            for j in range(4):
                dst = HF[s] + 8 * c + 4 * half + j
                src = ACC[s][c] + 8 * half + 2 * j
                cv.append(f"v_cvt_pk_bf16_f32 v{dst}, v{src}, v{src + 1}")
                mx.append(f"v_pk_max_i16 v{dst}, v{dst}, 0")
            ops += cv + mx
    return ops


def schedule(frags, first_frag, compute, extra=None, before_first=None):
    """Four fragments in flight: preload 4, then per fragment: wait until it has arrived (the LDS
    counter is in order), issue its MFMAs, reload its register with the fragment 4 ahead.
    extra[t] = vector-ALU lines issued after the MFMAs of fragment t; before_first = lines
    placed right before the first MFMA."""
    n = len(frags)
    out = [wt(0)] + [ld(f"f{i}", first_frag + i) for i in range(min(4, n))]
    for t in range(n):
        issued = min(n, t + 4)
        out.append(wt(issued - t - 1))
        if t == 0 and before_first:
            out += before_first
        out += compute(t, f"f{t % 4}")
        if t + 4 < n:
            out.append(ld(f"f{t % 4}", first_frag + t + 4))
        if extra and t in extra:
            out += extra[t]
    return out


def dma_loads():
    out = ["s_mov_b32 m0, %[lb]"]
    for t in range(N_DMA):
        if t:
            out.append("s_add_u32 m0, m0, 0x1000")
        out += ["s_nop 0", f"global_load_lds_dwordx4 %[vo], %[sb{t}]"]  # one wait state between the M0 write and its use
    return out


def user_loads(into):
    """User term of the next layer-1 block into accumulator set `into`: register 4*t4 + e of pair
    c takes float 8*t4 + e of the 32 the lane's pointer %[upn<c>] addresses."""
    return [f"global_load_dwordx4 {vr(ACC[into][c] + 4 * t4, 4)}, %[upn{c}], off offset:{32 * t4}"
            for t4 in range(4) for c in (0, 1)]


def step(kind, s=None, load_user=True, load_xp=True, store_xp=True, wait_user=True):
    other = "B" if s == "A" else "A"
    own = N_DMA + (8 if load_user else 0) + (1 if load_xp else 0)
    head = dma_loads() + (user_loads(other) if load_user else []) + (["global_load_dwordx4 %[xpn], %[xpsrc], off"] if load_xp else [])
    # own user term: younger are the piece fetched after it (one load) and this step's loads
    before = [f"s_waitcnt vmcnt({own + 1})"] if wait_user else None
    tail = [f"s_waitcnt vmcnt({own})"]
    if store_xp:
        tail += ["ds_write_b128 %[xwst], %[xpo]"]
    tail += ["s_waitcnt lgkmcnt(0)", "s_barrier"]
    if kind == "FIRST":
        lines = schedule(range(8), 0, lambda t, b: m1("A", b, t), before_first=before)
        lines += ["s_nop 15"] + convert_ops("A")
    elif kind == "LAST":
        lines = schedule(range(16), 8, lambda t, b: m2("B", b, t // 2, t % 2))
        lines += ["s_nop 15"]
    else:
        ops = convert_ops(s)
        # the last layer-1 MFMA is fragment 7; conversions start after fragment 9's layer-2 MFMAs
        # (four more MFMAs in between: far beyond the MFMA-to-VALU hazard window) and are spread
        # over the remaining fragments
        slots = list(range(10, 24))
        per = -(-len(ops) // len(slots))
        extra = {}
        for i, t in enumerate(slots):
            chunk = ops[i * per:(i + 1) * per]
            if chunk:
                extra[t] = chunk

        def compute(t, b):
            return m1(s, b, t) if t < 8 else m2(other, b, (t - 8) // 2, (t - 8) % 2)

        lines = schedule(range(24), 0, compute, extra, before_first=before)
    return head + lines + tail


def c_string(lines):
    return " \\\n    ".join('"' + l + '\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// Generated by gen_stream_asm.py -- do not edit; see that script for the register plan.", ""]
    # FIRST: its user term was fetched by the last MID_B of the batch before and waited for by LAST
    variants = (("FIRST", step("FIRST", "A", store_xp=False, wait_user=False)),
                ("MID_A", step("MID", "A")), ("MID_B", step("MID", "B")),
                ("LAST", step("LAST", load_user=False, load_xp=False, wait_user=False)))
    for name, lines in variants:
        out.append(f"#define STREAM_ASM_{name} \\\n    {c_string(lines)}")
        out.append("")
    # operand lists
    for s in "AB":
        out.append(f'#define STREAM_ACC_{s}(v0, v1) [p{s}0] "+{{{acc_reg(s, 0)}}}"(v0), [p{s}1] "+{{{acc_reg(s, 1)}}}"(v1)')
        out.append(f'#define STREAM_ACC_OUT_{s}(v0, v1) [q{s}0] "=&{{{acc_reg(s, 0)}}}"(v0), [q{s}1] "=&{{{acc_reg(s, 1)}}}"(v1)')
        names = [(c, h) for c in (0, 1) for h in (0, 1)]
        outs = ", ".join(f'[h{s}{c}{h}] "=&{{{hf_reg(s, c, h)}}}"(h{c}{h})' for c, h in names)
        ins = ", ".join(f'[h{s}{c}{h}] "{{{hf_reg(s, c, h)}}}"(h{c}{h})' for c, h in names)
        out.append(f"#define STREAM_HF_OUT_{s}(h00, h01, h10, h11) {outs}")
        out.append(f"#define STREAM_HF_IN_{s}(h00, h01, h10, h11) {ins}")
    acc2 = ", ".join(f'[a{n2}{c}] "+a"(acc2[{n2}][{c}])' for n2 in range(8) for c in (0, 1))
    out.append(f"#define STREAM_ACC2 {acc2}")
    out.append("")
    with open(os.path.join(here, "mlp_mfma_stream_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
