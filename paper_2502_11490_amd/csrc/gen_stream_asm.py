#!/usr/bin/env python3
"""Writes mlp_mfma_stream_asm.inc: the inline-assembly text of the NB1 + 1 = 17 pipeline steps of
the streaming MFMA relevance kernel (mlp_mfma_stream.hip), for item width 128 (8 layer-1
fragments per step), first hidden width 512 (16 blocks of 32 units) and second hidden width 256
(16 layer-2 fragments per step), 64 pairs per wave.  Every step has its own text, so that all
per-step addresses are immediates and nothing but one scalar add is left between two steps.

Register plan of a wave (fixed physical registers, so that the vector-ALU instructions that turn
fresh layer-1 accumulators into bf16 B operands can be interleaved with the MFMAs of layer 2 and
so that every step agrees on where the long-lived values are):

    a[0:255]            layer-2 accumulators, tile (n2, c) at a[16 (2 n2 + c) ...]
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
    head      (i = 16)  the last step runs layer 2 tile by tile and, behind every finished tile, its
                        conversion to bf16 head operands and the head layer's MFMAs (see step16_head)

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


def acc2_lo(n2, c):
    return 16 * (2 * n2 + c)


def acc2_reg(n2, c):
    """Layer-2 accumulator tile (n2, c).  The 256 accumulation registers are named outright and are not
    operands: the head conversion reads single registers of a tile, which an operand cannot express, and
    tiles pinned as operands make the allocator shuffle them between the statements.  Every statement lists
    them as clobbered; the kernel's own code between the statements has no use for accumulation registers
    (a test compiles the kernel and checks that none appears outside the statements)."""
    return f"a[{acc2_lo(n2, c)}:{acc2_lo(n2, c) + 15}]"


def init_acc2():
    """The accumulators start from the layer-2 bias, read from LDS straight into the accumulation registers:
    register 4 t4 + e of a tile holds unit 32 n2 + 8 t4 + 4 g + e, so a lane reads 16 bytes at
    %[b2] (= bias base + 16 g) + 128 n2 + 32 t4 for both column blocks.  Step 0 starts with a full wait."""
    return [f"ds_read_b128 a[{acc2_lo(n2, c) + 4 * t4}:{acc2_lo(n2, c) + 4 * t4 + 3}], %[b2] offset:{n2 * 128 + t4 * 32}"
            for n2 in range(8) for c in (0, 1) for t4 in range(4)]


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


# ---- the last step: layer 2 of hidden block 15 with the head layer folded in ----
ACC3 = (96, 112)        # head accumulators of pairs c = 0, 1: set B's registers, idle since step 15's conversion
RT = 64                 # 16 registers that receive one tile from the accumulation registers (set A's, idle)
TSET = (80, 128)        # a tile's four bf16 head operands (c, s2) at TSET[n2 % 2] + 8 c + 4 s2: tiles alternate
                        # between the rest of set A's registers and set A's hidden units (consumed by step 15)
N_HEAD = 16             # head fragments [2 n2 + s2]


def head_convert(n2, c):
    """Tile (n2, c) of the layer-2 accumulators -> ReLU + bf16, the B operands of head fragments 2 n2 and
    2 n2 + 1 for pair c: 16 reads out of the accumulation registers, 8 conversions, 8 signed 16-bit max."""
    lo, t = acc2_lo(n2, c), TSET[n2 % 2] + 8 * c
    ops = [f"v_accvgpr_read_b32 v{RT + j}, a{lo + j}" for j in range(16)]
    ops += [f"v_cvt_pk_bf16_f32 v{t + j}, v{RT + 2 * j}, v{RT + 2 * j + 1}" for j in range(8)]
    ops += [f"v_pk_max_i16 v{t + j}, v{t + j}, 0" for j in range(8)]
    return ops


def head_pair(u):
    """Head fragment u against both column blocks; the first pair starts from zero."""
    n2, s2 = divmod(u, 2)
    out = []
    for c in (0, 1):
        acc = vr(ACC3[c], 16)
        out.append(f"v_mfma_f32_32x32x16_bf16 {acc}, %[w3{u % 4}], {vr(TSET[n2 % 2] + 8 * c + 4 * s2, 4)}, "
                   + ("0" if u == 0 else acc))
    return out


def step16_head():
    """Step 16 issues layer 2 tile by tile (fragment t = (n2, s2) = (t / 2, t % 2)), so tile n2 has its
    final value once slot 2 n2 + 1 has issued and two more MFMAs behind it.  From slot 4 on every slot
    also converts one (tile, c) for the head layer, and from slot 6 on it also issues one head fragment's
    pair of MFMAs (fragment u = t - 6: its operands were converted in slots 2 n2 + 4 and 2 n2 + 5); five
    more slots after layer 2 finish the last two tiles and the last six head fragments.  Per slot 32
    vector-ALU instructions stand against four MFMAs, 128 cycles each.  Head fragments come from LDS
    through four compiler-chosen tuples %[w30..w33], re-requested like the weight fragments."""
    n = 16
    vm = vmem_ops(NB1, "B")
    own = len(vm)
    assert own == N_DMA
    out = ["s_mov_b32 m0, %[lb]", "v_and_b32 %[wcn], 0x3ff, %[vo]", "v_add_u32 %[wc], %[wcs], %[wcn]",
           "v_add_u32 %[wcn], %[wcsn], %[wcn]"]
    queue = [("f", k) for k in range(4)]       # requested by step 15 after its barrier

    def issue(tag, line):
        queue.append(tag)
        out.append(line)

    def wait_for(tag):
        if tag not in queue:
            return
        younger = len(queue) - queue.index(tag) - 1
        out.append(wt(younger))
        del queue[:queue.index(tag) + 1]

    def w3_read(u):
        issue(("h", u), f"ds_read_b128 %[w3{u % 4}], %[w3] offset:{u * 1024}")

    for u in range(4):
        w3_read(u)
    convs = [(n2, c) for n2 in range(8) for c in (0, 1)]     # conversion k runs in slot k + 4
    store_slot, sync_at = 10, sync_slot(n)
    for t in range(n + 5):
        side = head_convert(*convs[t - 4]) if 0 <= t - 4 < len(convs) else []
        if t < own:
            side = vm[t] + side
        mf = []                                              # the slot's MFMAs, each with what it waits for
        if t < n:
            mf += [(("f", t), m) for m in m2("B", freg(t), t // 2, t % 2)]
        heads = [t - 6] if 6 <= t < n + 4 else ([N_HEAD - 2, N_HEAD - 1] if t == n + 4 else [])
        for u in heads:
            mf += [(("h", u), m) for m in head_pair(u)]
        per = -(-len(side) // max(len(mf), 1))
        if t == n + 4:
            out.append("s_nop 1")                            # the operands of fragment 14 were just written
        for j, (tag, m) in enumerate(mf):
            wait_for(tag)
            out.append(m)
            if j % 2 == 1:                                   # a fragment's registers are free behind its second MFMA
                if tag[0] == "f" and tag[1] + 4 < n:
                    issue(("f", tag[1] + 4), ld(tag[1] + 4, 8 + tag[1] + 4))
                if tag[0] == "h" and tag[1] + 4 < N_HEAD:
                    w3_read(tag[1] + 4)
            out.extend(side[j * per:(j + 1) * per])
        out.extend(side[len(mf) * per:])
        if t == store_slot:
            out.append(f"s_waitcnt vmcnt({N_DMA + own})")
            issue(("w",), f"ds_write_b128 %[xw], %[xpo] offset:{(NB1 - 1) * 1024}")
        if t == sync_at:
            out += [f"s_waitcnt vmcnt({own})", "s_waitcnt lgkmcnt(0)", "s_barrier"]
            queue.clear()
    out += ["s_nop 15", "s_nop 7"]                           # the head accumulators are read next
    return out


def c_string(lines):
    """The lines as adjacent C string literals; the 16-bit format's name in the two mnemonics that carry it
    (the MFMA and the packed conversion) is the macro argument T, "bf16" or "f16"."""
    def lit(l):
        for name in ("v_mfma_f32_32x32x16_bf16", "v_cvt_pk_bf16_f32"):
            l = l.replace(name, name.replace("bf16", '" T "'))
        return '"' + l + '\\n\\t"'
    return " \\\n    ".join(lit(l) for l in lines)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    out = ["// Generated by gen_stream_asm.py -- do not edit; see that script for the register plan.", ""]
    for i in range(NB1 + 1):
        out.append(f"#define STREAM_ASM_STEP_{i}(T) \\\n    {c_string(step16_head() if i == NB1 else step(i))}")
        out.append("")
    out.append(f"#define STREAM_ASM_INIT_ACC2 \\\n    {c_string(init_acc2())}")
    out.append("")
    out.append("#define STREAM_ACC2_CLOBBERS " + ", ".join(f'"a{r}"' for r in range(256)))
    out.append(f'#define STREAM_ACC3(v0, v1) [q30] "=&{{{vr(ACC3[0], 16)}}}"(v0), [q31] "=&{{{vr(ACC3[1], 16)}}}"(v1)')
    scratch = list(range(RT, RT + 16)) + [r for t in TSET for r in range(t, t + 16)]
    out.append("#define STREAM_HEAD_CLOBBERS " + ", ".join(f'"v{r}"' for r in sorted(scratch)))
    # operand lists
    for s in "AB":
        out.append(f'#define STREAM_ACC_{s}(v0, v1) [p{s}0] "+{{{acc_reg(s, 0)}}}"(v0), [p{s}1] "+{{{acc_reg(s, 1)}}}"(v1)')
        out.append(f'#define STREAM_ACC_OUT_{s}(v0, v1) [q{s}0] "=&{{{acc_reg(s, 0)}}}"(v0), [q{s}1] "=&{{{acc_reg(s, 1)}}}"(v1)')
        names = [(c, h) for c in (0, 1) for h in (0, 1)]
        outs = ", ".join(f'[h{s}{c}{h}] "=&{{{hf_reg(s, c, h)}}}"(h{c}{h})' for c, h in names)
        ins = ", ".join(f'[h{s}{c}{h}] "{{{hf_reg(s, c, h)}}}"(h{c}{h})' for c, h in names)
        out.append(f"#define STREAM_HF_OUT_{s}(h00, h01, h10, h11) {outs}")
        out.append(f"#define STREAM_HF_IN_{s}(h00, h01, h10, h11) {ins}")
    out.append(f'#define STREAM_SB(p) [sb] "+{{{SB}}}"(p)')
    frs = ", ".join(f'[f{k}] "+{{{freg(k)}}}"(f{k})' for k in range(4))
    out.append(f"#define STREAM_FRAGS(f0, f1, f2, f3) {frs}")
    out.append("")
    with open(os.path.join(here, "mlp_mfma_stream_asm.inc"), "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    main()
