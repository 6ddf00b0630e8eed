#!/usr/bin/env python3
"""Writes mlp_mfma_stream_asm.inc: the inline-assembly text of the NB1 + 1 = 17 pipeline steps of
the streaming MFMA relevance kernel (mlp_mfma_stream.hip), for item width 128 (8 layer-1
fragments per step), first hidden width 512 (16 blocks of 32 units) and second hidden width 256
(16 layer-2 fragments per step), 64 pairs per wave.  Every step has its own text, so that all
per-step addresses are immediates and nothing but one scalar add is left between two steps.

Register plan of a wave (fixed physical registers, so that the vector-ALU instructions that turn
fresh layer-1 accumulators into bf16 B operands can be interleaved with the MFMAs of layer 2 and
so that every step agrees on where the long-lived values are):

    256 AGPRs           layer-2 accumulators, 16 tiles (n2, c), constraint "a" (the allocator's choice)
    v[64:95], v[96:127] layer-1 accumulators, sets A and B (pairs c = 0, 1), alternating by step
    v[128:143]          hidden units produced from set A, tuple (c, half) at v[128 + 8c + 4half ...]
    v[144:159]          hidden units produced from set B
    v[160:175]          four weight fragments in flight from LDS (requested across step boundaries)
    compiler's choice   the 16 item-row operands, LDS read addresses, pointers

Step i (0 .. 16):
    layer 1   (i < 16)  hidden block i into set A (i even) or B (i odd); fragments 0..7 of chunk i
    layer 2   (i > 0)   over the hidden units of block i-1 (the other set); fragments 8..23
    convert   (i < 16)  ReLU + bf16 rounding of the fresh set, interleaved with the layer-2 MFMAs
                        (exposed in step 0, which has none)

Global loads of a step and their waits are part of the assembly too, because the compiler cannot
count them: next to global-to-LDS loads any other vector-memory load makes it fall back to
waiting for ALL outstanding loads, the weight chunks included (and it treats every LDS access it
sees as depending on them).  Loads are spread over the step, one after the MFMAs of a fragment:
issuing a vector-memory instruction holds the wave for some tens of cycles, which an MFMA in
flight hides.  In issue order a step has
    8   user term of hidden block i+1 (i < 15), straight into the accumulator set that is idle
        during this step (block 0 is fetched by the kernel's own code before step 0)
    1   one 16-byte piece of the next batch's item rows (i < 16)
    6   weight chunk (i+2) mod 17 into the LDS buffer that step i-1 read: scalar base in
        s[100:101] + lane offset %[vo]; LDS base in M0; both 4 KB further per load, so that the
        scalar base ends a step at the next chunk (the kernel resets it where the chunks wrap)
and waits (the counter is in order)
    - before its first layer-1 MFMA for its own user term, issued first in step i-1: younger are
      that step's item piece and chunk loads, 7 in all;
    - once its loads are issued, for the item piece fetched one step ago, which then goes to the
      wave's LDS area;
    - three fragments before its end until only this step's own loads are outstanding: then the
      chunk the next step reads has landed; the LDS store is waited for and the wave joins the
      workgroup barrier.  By then every read of this step's buffer has completed too: behind the barrier
      the next step may refill it, and this step may already request the next step's first
      fragments.

Run this script after changing it; the .inc file is committed next to it.
"""
import os

ACC = {"A": (64, 80), "B": (96, 112)}       # first register of the c = 0 / c = 1 accumulator
HF = {"A": 128, "B": 144}                   # first register of the four (c, half) tuples
NB1 = 16                                    # layer-1 blocks of 32 hidden units
SB, SB_LO, SB_HI = "s[100:101]", "s100", "s101"   # scalar base of the weight chunk being fetched
N_DMA = 6                                   # global-to-LDS loads per step: 6 x 256 lanes x 16 B = one chunk


def vr(lo, n):
    return f"v[{lo}:{lo + n - 1}]"


def acc_reg(s, c):
    return vr(ACC[s][c], 16)


def hf_reg(s, c, half):
    return vr(HF[s] + 8 * c + 4 * half, 4)


def acc2_reg(n2, c):
    return f"%[a{n2}{c}]"  # layer-2 accumulators: any AGPR tuple, the allocator keeps them in place


def wt(n):
    return f"s_waitcnt lgkmcnt({n})"


def m1(s, buf, k):
    return [f"v_mfma_f32_32x32x16_bf16 {acc_reg(s, c)}, {buf}, %[x{c}{k}], {acc_reg(s, c)}" for c in (0, 1)]


def m2(hs, buf, n2, s2):
    return [f"v_mfma_f32_32x32x16_bf16 {acc2_reg(n2, c)}, {buf}, {hf_reg(hs, c, s2)}, {acc2_reg(n2, c)}"
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


FRAG = 160                                  # first register of the four weight fragments in flight


def freg(k):
    return vr(FRAG + 4 * (k % 4), 4)


def ld(k, frag, addr="wc"):
    return f"ds_read_b128 {freg(k)}, %[{addr}] offset:{frag * 1024}"


def sync_slot(n):
    """Slot after whose MFMAs the wave synchronises with the workgroup: all reads of this step's
    buffer were issued two slots earlier, and three slots of MFMAs are left to cover the first
    reads of the next step's buffer."""
    return n - 3


def schedule(n, first_frag, compute, extra, before_first, sync, preloaded, next_first, store):
    """Fragment k of the step lives in register set k % 4; four are in flight.  Per slot t: wait
    until fragment t has arrived (the LDS counter is in order: allow as many outstanding
    operations as were issued after its read), issue its MFMAs, then re-use its registers for the
    fragment four ahead.  The last four slots have nothing of this step left to read: after slot
    n-3 comes `sync` (ending in the barrier), after which the next step's first fragments are
    requested (from %[wcn], the buffer the next step reads; next_first = its first fragment, None =
    no next step), so that the next block starts with its reads in flight (preloaded).
    store = (slot, wait line, LDS store line) or None: an LDS store issued after that slot."""
    out, queue = [], []          # queue: LDS operations issued and not known complete, in order

    def issue(tag, line):
        queue.append(tag)
        out.append(line)

    def wait_for(tag):
        if tag not in queue:     # completed by an earlier full wait
            return
        younger = len(queue) - queue.index(tag) - 1
        out.append(wt(younger))
        del queue[:queue.index(tag) + 1]

    if preloaded:
        queue += [("f", k) for k in range(4)]
    else:
        out.append(wt(0))
        for k in range(min(4, n)):
            issue(("f", k), ld(k, first_frag + k))
    for t in range(n):
        wait_for(("f", t))
        if t == 0:
            out.extend(before_first)
        # an MFMA occupies the matrix pipe for 32 cycles during which the wave can issue other
        # instructions: half of the slot's side work goes behind each of the two MFMAs (the
        # fragment's registers can only be re-used after the second)
        first, second = compute(t, freg(t))
        units = extra.get(t, [])
        half = (len(units) + 1) // 2
        out.append(first)
        for u in units[:half]:
            out.extend(u)
        out.append(second)
        if t + 4 < n:
            issue(("f", t + 4), ld(t + 4, first_frag + t + 4))
        for u in units[half:]:
            out.extend(u)
        if store and t == store[0]:
            out.append(store[1])
            issue(("w",), store[2])
        if t == sync_slot(n):
            out.extend(sync)     # ends with lgkmcnt(0): nothing outstanding
            queue.clear()
        if next_first is not None and t >= sync_slot(n):
            for k in ([0, 1] if t == sync_slot(n) else [t - sync_slot(n) + 1]):
                issue(("n", k), ld(k, next_first + k, "wcn"))
    return out


def vmem_ops(i, idle):
    """The step's global loads in issue order, each a list of lines."""
    ops = []
    if i + 1 < NB1:
        # register 4*t4 + e of pair c takes float 8*t4 + e of the 32 floats of block i+1
        ops += [[f"global_load_dwordx4 {vr(ACC[idle][c] + 4 * t4, 4)}, %[up{c}], off offset:{(i + 1) * 128 + 32 * t4}"]
                for t4 in range(4) for c in (0, 1)]
    if i < NB1:
        ops.append([f"global_load_dwordx4 %[xpn], %[xs], off offset:{32 * (i % 8)}"])  # %[xs]: row of pair c = i / 8
    for t in range(N_DMA):
        # the M0 write sits right after the previous load: far more than the one wait state it needs
        ops.append([f"global_load_lds_dwordx4 %[vo], {SB}", f"s_add_u32 {SB_LO}, {SB_LO}, 0x1000",
                    f"s_addc_u32 {SB_HI}, {SB_HI}, 0"] + (["s_add_u32 m0, m0, 0x1000"] if t + 1 < N_DMA else []))
    return ops


def step(i):
    fresh = "A" if i % 2 == 0 else "B"      # set that layer 1 of this step fills
    other = "B" if fresh == "A" else "A"    # its hidden units feed layer 2; its accumulators are idle
    has_l1, has_l2 = i < NB1, i > 0
    vm = vmem_ops(i, other)
    own = len(vm)
    before = [f"s_waitcnt vmcnt({1 + N_DMA})"] if 0 < i < NB1 else []   # step 0: the compiler's load and wait
    n_frag = (8 if has_l1 else 0) + (16 if has_l2 else 0)
    first_frag = 0 if has_l1 else 8

    def compute(t, b):
        f = first_frag + t
        return m1(fresh, b, f) if f < 8 else m2(other, b, (f - 8) // 2, (f - 8) % 2)

    extra = {t: [] for t in range(n_frag)}
    # vector-memory loads: from the first fragment on, as evenly as they fit before the synchronisation
    per = -(-own // (sync_slot(n_frag) + 1))
    for k, op in enumerate(vm):
        extra[k // per].append(op)
    tail = []
    if has_l1 and has_l2:
        # the last layer-1 MFMA is fragment 7; conversions start after fragment 9's layer-2 MFMAs
        # (four more MFMAs in between: far beyond the MFMA-to-VALU hazard window) and are spread
        # over the remaining fragments
        ops = convert_ops(fresh)
        slots = list(range(10, 24))
        cper = -(-len(ops) // len(slots))
        for j, t in enumerate(slots):
            extra[t] += [[op] for op in ops[j * cper:(j + 1) * cper]]
    elif has_l1:
        tail += ["s_nop 15"] + convert_ops(fresh)
    else:
        tail += ["s_nop 15"]    # the compiler's code reads the layer-2 accumulators next
    sync = [f"s_waitcnt vmcnt({own})", "s_waitcnt lgkmcnt(0)", "s_barrier"]
    store = None
    if i > 0:
        # the item piece fetched one step ago goes to the wave's LDS area once all of this step's
        # loads are issued (younger than it: the 6 chunk loads behind it and this step's own),
        # a few slots ahead of the synchronisation, which waits for the store
        last_vm = (own - 1) // per
        store = (max(last_vm + 1, sync_slot(n_frag) - 3), f"s_waitcnt vmcnt({N_DMA + own})",
                 f"ds_write_b128 %[xw], %[xpo] offset:{(i - 1) * 1024}")
        assert last_vm < store[0] < sync_slot(n_frag)
    # LDS read addresses of the lane, this step's buffer and the next step's: buffer base (scalar)
    # + 16 * lane, the latter from the lane offset of the chunk loads (16 * thread index, 64 lanes per wave)
    setup = ["s_mov_b32 m0, %[lb]", "v_and_b32 %[wcn], 0x3ff, %[vo]", "v_add_u32 %[wc], %[wcs], %[wcn]",
             "v_add_u32 %[wcn], %[wcsn], %[wcn]"]
    next_first = None if i == NB1 else (0 if i + 1 < NB1 else 8)
    return setup + schedule(n_frag, first_frag, compute, extra, before, sync, preloaded=i > 0, next_first=next_first, store=store) + tail


def c_string(lines):
    return " \\\n    ".join('"' + l + '\\n\\t"' for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// Generated by gen_stream_asm.py -- do not edit; see that script for the register plan.", ""]
    for i in range(NB1 + 1):
        out.append(f"#define STREAM_ASM_STEP_{i} \\\n    {c_string(step(i))}")
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
    out.append(f'#define STREAM_SB(p) [sb] "+{{{SB}}}"(p)')
    frs = ", ".join(f'[f{k}] "+{{{freg(k)}}}"(f{k})' for k in range(4))
    out.append(f"#define STREAM_FRAGS(f0, f1, f2, f3) {frs}")
    out.append("")
    with open(os.path.join(here, "mlp_mfma_stream_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
