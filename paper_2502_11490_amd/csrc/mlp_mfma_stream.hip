// Fused bf16 MFMA relevance kernel for the widest metric (item width 128, hidden 512 and 256):
// Sec. 3.1 (1), Eq. 5-8, over the dense pair list of Algorithm 2.
//
// Same formulation as mlp_mfma.hip (activations transposed and register resident, weights as
// the A operand in fragment order, user half of layer 1 pre-computed per query), but with the
// per-wave register file planned by hand, because at this size it is full:
//     256 AGPRs  layer-2 accumulators of 64 pairs x 256 units (16 MFMA tiles)
//      64 VGPRs  the 64 item rows as layer-1 B operands
//      64 VGPRs  layer-1 accumulators of this step and the pre-loaded user term of the next
//      16 VGPRs  the 32 hidden units of the previous step as layer-2 B operands (bf16)
//      16 VGPRs  four weight fragments in flight from LDS
//       8 VGPRs  staging of the next batch's item rows
// The compiler's register allocator does not find this plan, so one step of the pipeline is a
// single inline-assembly block with the register classes pinned by constraints.  The 256
// accumulation registers are not operands at all: the statements name them outright and list them
// as clobbered (tiles pinned as operands make the allocator shuffle them between the statements, and
// the head layer reads single registers of a tile, which an operand cannot express); the code between
// the statements has no use for accumulation registers, which a test checks on the compiled kernel.
//
// Pipeline.  Step i (0..NB1) contracts layer 1 for hidden units 32i..32i+31 and, skewed by one
// step, layer 2 over the hidden units of step i-1; chunk i of the weights holds exactly those
// fragments (8 of W1_item, then 16 of W2) and streams L2 -> LDS directly (global_load_lds, no
// registers in between) TWO steps ahead of its use into one of three 24 KB buffers: every CU of
// the chip asks for the same 24 KB at about the same time, so the L2 delivers them slowly, and
// a chunk gets two whole steps to arrive.  One barrier per step; before it each wave waits
// (counted, the vector-memory counter is in order) for everything it issued before this step,
// which includes its share of the chunk the next step reads.  Fragments are read from LDS four
// ahead of use.  A step issues its global loads first, weights before the user term before one
// piece of the next batch's item rows, so that the in-order counter never makes a
// short-latency consumer wait for the long-latency gather.
// ReLU + bf16 rounding of the fresh hidden units is the only vector-ALU work of a step.  The last
// step runs layer 2 tile by tile and carries the head layer: behind every finished tile its ReLU +
// bf16 conversion (out of the accumulation registers) and the head MFMAs over it, so that the 512
// vector-ALU instructions of that conversion run under MFMAs instead of behind them.  The
// item rows of the workgroup's NEXT batch are fetched one 16-byte piece per lane and step into
// a wave-private LDS area, so the HBM gather latency is hidden behind a whole batch of MFMAs.
//
// Hazards handled by hand inside the assembly (the compiler cannot see into it):
//   - the ReLU + bf16 conversion of a step's fresh layer-1 accumulators is interleaved with the
//     layer-2 MFMAs of the same block and starts six MFMAs after the last layer-1 MFMA;
//   - every block starts with s_waitcnt lgkmcnt(0): afterwards only its own LDS reads are in
//     flight and the counted waits (lgkmcnt(3..0)) are exact;
//   - an accumulator is never the target of two consecutive MFMAs (pairs 0 and 1 alternate);
//   - results read by the vector ALU right after a block (layer-1 accumulators after the
//     first step, head accumulators after the last) are waited for with s_nop; a layer-2 tile is
//     read at least four MFMAs after the last one that wrote it;
//   - a weight-fragment register is reloaded from LDS only after the MFMAs reading it have
//     issued (MFMA operands are read at issue).
#include <type_traits>
#include <vector>

#include "common.h"

namespace gmpgr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

constexpr int ST_BLOCK = 256;

// LDS accesses made while weight chunks are in flight towards the LDS go through assembly: for an
// LDS access it can see, the compiler first waits until every outstanding global-to-LDS load
// has landed (it cannot tell that the addresses differ), which would undo the pipelining.
__device__ __forceinline__ void lds_store_b128(uint32_t addr, const u32x4 &v) {
    asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
// f(integral_constant<int, I>) for I = 0 .. N-1: loop indices usable as template arguments
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// four 16-byte reads at addr + BASE + {0, 1, 2, 3} * STRIDE (immediates: no address registers), complete on return
template <int BASE, int STRIDE>
__device__ __forceinline__ void lds_load4_b128(uint32_t addr, u32x4 &r0, u32x4 &r1, u32x4 &r2, u32x4 &r3) {
    static_assert(BASE >= 0 && BASE + 3 * STRIDE < 65536, "offsets are 16-bit immediates");
    asm volatile("ds_read_b128 %0, %4 offset:%5\n\t"
                 "ds_read_b128 %1, %4 offset:%6\n\t"
                 "ds_read_b128 %2, %4 offset:%7\n\t"
                 "ds_read_b128 %3, %4 offset:%8\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
                 : "v"(addr), "n"(BASE), "n"(BASE + STRIDE), "n"(BASE + 2 * STRIDE), "n"(BASE + 3 * STRIDE)
                 : "memory");
}

#include "mlp_mfma_stream_asm.inc"  // STREAM_ASM_FIRST / MID_A / MID_B / LAST and their operand lists

#define FRAG_TEMPS STREAM_FRAGS(f0, f1, f2, f3), [wc] "=&v"(wct), [wcn] "=&v"(wcnt)
#define X_OPERANDS                                                                                  \
    [x00] "v"(xf[0][0]), [x01] "v"(xf[0][1]), [x02] "v"(xf[0][2]), [x03] "v"(xf[0][3]),             \
    [x04] "v"(xf[0][4]), [x05] "v"(xf[0][5]), [x06] "v"(xf[0][6]), [x07] "v"(xf[0][7]),             \
    [x10] "v"(xf[1][0]), [x11] "v"(xf[1][1]), [x12] "v"(xf[1][2]), [x13] "v"(xf[1][3]),             \
    [x14] "v"(xf[1][4]), [x15] "v"(xf[1][5]), [x16] "v"(xf[1][6]), [x17] "v"(xf[1][7])

// Weight fragments, bf16, 1 KB each (lane l at byte 16*l), NB1 + 1 chunks of 24 fragments:
//   chunk i, fragment s < 8       lane (m,g): W1_item[32i+m][16s + 8g + j]                      (zero for i = NB1)
//   chunk i, fragment 8+2*n2+s2   lane (m,g): W2[32*n2+m][32(i-1) + 16*s2 + 8*(j/4) + 4g + j%4] (zero for i = 0)
// then 16 head fragments [2*n2+s2], lane (m,g): W3[m][32*n2 + 16*s2 + 8*(j/4) + 4g + j%4], rows m >= J zero.
// F16: items, weights and hidden units are IEEE binary16 instead of bf16 (the operands travel as the same
// 16-byte tuples; the two mnemonics that name the format are a parameter of the step texts).
template <int H1, bool F16>
__global__ void __launch_bounds__(ST_BLOCK)
mlp_mfma2_stream_kernel(const uint16_t *__restrict__ emb, int64_t N, const float *__restrict__ upre,
                        const uint4 *__restrict__ frag, const float *__restrict__ b2, const float *__restrict__ b3,
                        const float *__restrict__ head_w, int J, const int32_t *__restrict__ pair_q,
                        const int32_t *__restrict__ pair_id, const int32_t *__restrict__ M_dev, int64_t M_max,
                        int32_t Q, float *__restrict__ scores) {
    constexpr int D = 128, KS1 = 8, NB1 = H1 / 32, NB2 = 8, CB = 2;
    constexpr int NSTEP = NB1 + 1;
    constexpr int CHUNK_U4 = 24 * 64;
    constexpr int W3_U4 = 16 * 64;
    constexpr int TILE = 64 * 4;
    constexpr int NBUF = 3;
    extern __shared__ __align__(16) uint4 lds[];
    uint4 *wbuf = lds;                       // [NBUF][CHUNK_U4]
    uint4 *w3buf = lds + NBUF * CHUNK_U4;    // [W3_U4]
    uint4 *xbuf = w3buf + W3_U4;             // [4 waves][CB*KS1][64 lanes]
    float *b2buf = (float *)(xbuf + 4 * CB * KS1 * 64);  // [NB2 * 32] layer-2 bias, [8] head weights, [8] head bias

    int64_t M = (int64_t)*M_dev;
    if (M > M_max) M = M_max;
    const int64_t n_tiles = (M + TILE - 1) / TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, col = lane & 31;
    uint4 *xw = xbuf + (size_t)wave * (CB * KS1 * 64) + lane;
    const uint32_t xw_addr = (uint32_t)(uintptr_t)xw;

    // Item rows are gathered one batch ahead of the arithmetic (into the wave's LDS area), so the
    // item ids run two batches ahead; query ids and validity are read again one batch ahead rather
    // than kept in registers through a batch.  Rows past the end read the last pair (never stored).
    struct Ids {
        int32_t id[CB], q[CB];
        bool bad[CB];
    };
    // Requesting a batch's ids and looking at them are two calls, so that a whole step can lie between them.
    // Both are tied to their place among the assembly statements (which keep their order): the row index of
    // request_ids passes through an empty statement, or the compiler would hoist these loads from read-only
    // arrays above earlier steps, whose counted waits then make them wait for younger loads; check_ids passes
    // the raw values through one, which keeps every use of them behind the statement written before it.
    struct RawIds {
        int32_t id[CB], q[CB];
    };
    auto request_ids = [&](int64_t tile) {
        RawIds r;
        int32_t here = 0;
        asm volatile("" : "+s"(here));
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            int64_t row = tile * TILE + (int64_t)wave * 64 + c * 32 + col + here;
            row = row < M ? row : M - 1;
            r.id[c] = pair_id[row];
            r.q[c] = pair_q[row];
        }
        return r;
    };
    auto check_ids = [&](RawIds raw) {
        Ids r;
        static_assert(CB == 2, "the statement below names two pairs");
        asm volatile("" : "+v"(raw.id[0]), "+v"(raw.id[1]), "+v"(raw.q[0]), "+v"(raw.q[1]));
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const int32_t v = raw.id[c], q = raw.q[c];
            r.bad[c] = ((uint64_t)(int64_t)v >= (uint64_t)N) | ((uint32_t)q >= (uint32_t)Q);
            r.id[c] = r.bad[c] ? 0 : v;
            r.q[c] = r.bad[c] ? 0 : q;
        }
        return r;
    };
    // The launch's fixed cost is a chain of trips to memory (pair count, ids, item rows, user term); the copies
    // of the head fragments, of weight chunks 0 and 1 and of the constants into LDS go between its links.
    const RawIds raw_c = request_ids(blockIdx.x), raw_n = request_ids((int64_t)blockIdx.x + gridDim.x);
    for (int i = threadIdx.x; i < W3_U4; i += ST_BLOCK) w3buf[i] = frag[(size_t)NSTEP * CHUNK_U4 + i];
    for (int i = threadIdx.x; i < 2 * CHUNK_U4; i += ST_BLOCK) wbuf[i] = frag[i];  // chunks 0 and 1
    Ids idc = check_ids(raw_c), idn = check_ids(raw_n);
    {
        uint4 rows[CB][KS1];
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const uint4 *src = (const uint4 *)(emb + (size_t)idc.id[c] * D) + g;
#pragma unroll
            for (int s = 0; s < KS1; ++s) rows[c][s] = src[2 * s];
        }
        for (int i = threadIdx.x; i < NB2 * 32; i += ST_BLOCK) b2buf[i] = b2[i];
        if (threadIdx.x < 8) {  // head weights and head bias, zero beyond J
            b2buf[NB2 * 32 + threadIdx.x] = (int)threadIdx.x < J ? head_w[threadIdx.x] : 0.f;
            b2buf[NB2 * 32 + 8 + threadIdx.x] = (int)threadIdx.x < J ? b3[threadIdx.x] : 0.f;
        }
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int s = 0; s < KS1; ++s) xw[(c * KS1 + s) * 64] = rows[c][s];
    }
    __syncthreads();

    const uint32_t tid16 = threadIdx.x * 16;
    // Set A of the layer-1 accumulators enters every batch holding the user term of hidden block
    // 0: loaded here for the first batch, at the end of the batch before otherwise.
    f32x16 accA0, accA1;
    const float *up[CB];
    bool bad[CB];
    auto load_user_term0 = [&]() {
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
            f32x4 pv0 = *(const f32x4 *)(up[0] + 8 * t4);
            f32x4 pv1 = *(const f32x4 *)(up[1] + 8 * t4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                accA0[4 * t4 + e] = pv0[e];
                accA1[4 * t4 + e] = pv1[e];
            }
        }
    };
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        up[c] = upre + (size_t)idc.q[c] * H1 + 4 * g;
        bad[c] = idc.bad[c];
    }
    load_user_term0();
    // LDS address and global-to-LDS base (the wave's quarter) of the buffers that steps
    // 0, 1, 2 (mod 3) of the current batch read
    uint32_t wsv[NBUF], lbv[NBUF];
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
        wsv[b] = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(wbuf + (size_t)b * CHUNK_U4));
        lbv[b] = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(wbuf + (size_t)b * CHUNK_U4 + wave * 64));
    }

#pragma unroll 1
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t row0 = tile * TILE + (int64_t)wave * 64;
        bf16x8 xf[CB][KS1];
        size_t nxt_off[CB];  // element offsets of this lane's pieces of the next batch's rows
        // The layer-2 accumulators (the 256 accumulation registers, which only the assembly statements of this
        // loop touch: see gen_stream_asm.py) start from the bias, read from LDS straight into them: requested first, so that the
        // item rows' reads queue up behind them and one wait covers both.
        {
            uint32_t t16 = tid16;  // small addresses are rebuilt where they are used rather than kept across the steps
            asm volatile("" : "+v"(t16));
            const uint32_t b2_addr = (uint32_t)(uintptr_t)b2buf + ((t16 >> 5) & 16);  // 16 bytes * g
            asm volatile(STREAM_ASM_INIT_ACC2 : : [b2] "v"(b2_addr) : "memory", STREAM_ACC2_CLOBBERS);
        }

        {   // the batch's 64 item rows out of the wave's LDS area: sixteen reads, one wait
            static_assert(CB * KS1 == 16, "sixteen 16-byte pieces per lane");
            u32x4 r[16];
#define RD(k) "ds_read_b128 %" #k ", %16 offset:" #k "*1024\n\t"
            asm volatile(RD(0) RD(1) RD(2) RD(3) RD(4) RD(5) RD(6) RD(7) RD(8) RD(9) RD(10) RD(11) RD(12) RD(13) RD(14) RD(15)
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]),
                           "=&v"(r[7]), "=&v"(r[8]), "=&v"(r[9]), "=&v"(r[10]), "=&v"(r[11]), "=&v"(r[12]), "=&v"(r[13]),
                           "=&v"(r[14]), "=&v"(r[15])
                         : "v"(xw_addr)
                         : "memory");
#undef RD
#pragma unroll
            for (int c = 0; c < CB; ++c)
#pragma unroll
                for (int k = 0; k < KS1; ++k) xf[c][k] = __builtin_bit_cast(bf16x8, r[c * KS1 + k]);
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) nxt_off[c] = (size_t)idn.id[c] * D + 8 * g;

        // Two sets of layer-1 accumulators (A, B) and of converted hidden units alternate by step;
        // all of them, and the layer-2 accumulators, sit in fixed physical registers (see
        // gen_stream_asm.py), so every variant of the step agrees on where they are.
        f32x16 accB0, accB1;
        u32x4 hA00, hA01, hA10, hA11, hB00, hB01, hB10, hB11;
        // Operands of step i (see gen_stream_asm.py for the text).  Weight chunk i+2 goes straight
        // to the buffer that step i-1 read: per load instruction the workgroup moves 4 KB, wave w
        // the 1 KB at +1024 w (the LDS base of such a load is wave-uniform, lane l lands at +16 l);
        // the global side is the chunk's scalar base plus one lane offset per instruction.
        u32x4 xpA, xpB;
        bf16x8 f0 = {}, f1 = {}, f2 = {}, f3 = {};  // in flight from LDS across the step boundaries: never touched in between
        uint32_t wct, wcnt;
        static_assert(NB1 == 16 && NB1 == CB * KS1 && NSTEP % NBUF == 2, "the generated steps assume these");
        const char *sbv = (const char *)frag + 2 * (CHUNK_U4 * 16);   // chunk 2; every step leaves it at the next chunk
        const uint16_t *xs = emb + nxt_off[0];                        // next batch's row of pair c = 0 (steps 0..7)
#define STEP_COMMON(i) \
    [wcs] "s"(wsv[(i) % NBUF]), [wcsn] "s"(wsv[((i) + 1) % NBUF]), [lb] "s"(lbv[((i) + 2) % NBUF]), [vo] "v"(tid16)
#define STEP_LOADS [up0] "v"(up[0]), [up1] "v"(up[1]), [xs] "v"(xs)
        // odd step: layer 1 into set B, layer 2 over the hidden units of set A; fetches into set A
#define STREAM_STMT(TEXT, ...)                                \
    do {                                                      \
        if constexpr (F16) asm volatile(TEXT("f16") __VA_ARGS__); \
        else asm volatile(TEXT("bf16") __VA_ARGS__);          \
    } while (0)
#define STEP_ODD(i)                                                                                   \
    STREAM_STMT(STREAM_ASM_STEP_##i,                                                                  \
                 : STREAM_ACC_B(accB0, accB1), STREAM_ACC_OUT_A(accA0, accA1), STREAM_SB(sbv),        \
                   STREAM_HF_OUT_B(hB00, hB01, hB10, hB11), FRAG_TEMPS, [xpn] "=&v"(xpB)              \
                 : STEP_COMMON(i), X_OPERANDS, STREAM_HF_IN_A(hA00, hA01, hA10, hA11), STEP_LOADS, \
                   [xpo] "v"(xpA), [xw] "v"(xw_addr)                                                  \
                 : "memory", "scc", STREAM_ACC2_CLOBBERS);
#define STEP_EVEN(i)                                                                                  \
    STREAM_STMT(STREAM_ASM_STEP_##i,                                                                  \
                 : STREAM_ACC_A(accA0, accA1), STREAM_ACC_OUT_B(accB0, accB1), STREAM_SB(sbv),        \
                   STREAM_HF_OUT_A(hA00, hA01, hA10, hA11), FRAG_TEMPS, [xpn] "=&v"(xpA)              \
                 : STEP_COMMON(i), X_OPERANDS, STREAM_HF_IN_B(hB00, hB01, hB10, hB11), STEP_LOADS, \
                   [xpo] "v"(xpB), [xw] "v"(xw_addr)                                                  \
                 : "memory", "scc", STREAM_ACC2_CLOBBERS);
        // step 0: layer 1 only
        STREAM_STMT(STREAM_ASM_STEP_0,
                     : STREAM_ACC_A(accA0, accA1), STREAM_ACC_OUT_B(accB0, accB1), STREAM_SB(sbv),
                       STREAM_HF_OUT_A(hA00, hA01, hA10, hA11), FRAG_TEMPS, [xpn] "=&v"(xpA)
                     : STEP_COMMON(0), X_OPERANDS, STEP_LOADS
                     : "memory", "scc", STREAM_ACC2_CLOBBERS);
        STEP_ODD(1) STEP_EVEN(2) STEP_ODD(3) STEP_EVEN(4) STEP_ODD(5) STEP_EVEN(6) STEP_ODD(7)
        xs = emb + nxt_off[1];  // steps 8..15 fetch the row of pair c = 1
        STEP_EVEN(8) STEP_ODD(9) STEP_EVEN(10) STEP_ODD(11) STEP_EVEN(12) STEP_ODD(13) STEP_EVEN(14)
        sbv = (const char *)frag;  // steps 15 and 16 fetch chunks 0 and 1 again
        STREAM_STMT(STREAM_ASM_STEP_15,   // the last layer-1 block: no user term to fetch
                     : STREAM_ACC_B(accB0, accB1), STREAM_SB(sbv), STREAM_HF_OUT_B(hB00, hB01, hB10, hB11),
                       FRAG_TEMPS, [xpn] "=&v"(xpB)
                     : STEP_COMMON(15), X_OPERANDS, STREAM_HF_IN_A(hA00, hA01, hA10, hA11), [xs] "v"(xs),
                       [xpo] "v"(xpA), [xw] "v"(xw_addr)
                     : "memory", "scc", STREAM_ACC2_CLOBBERS);
        // ids of the next batch (again) and of the one after it: requested ahead of the last step, which hides
        // their latency
        const RawIds raw_c = request_ids(tile + gridDim.x), raw_n = request_ids(tile + 2 * (int64_t)gridDim.x);
        // step 16: layer 2 of the last hidden block tile by tile, and behind each finished tile its ReLU + bf16
        // conversion and the head layer's MFMAs over it (fragment rows >= J are zero)
        f32x16 acc3[CB];
        {
            uint32_t h16 = tid16;
            asm volatile("" : "+v"(h16));
            const uint32_t w3_addr = (uint32_t)(uintptr_t)w3buf + (h16 & 1023);  // 16 bytes * lane
            u32x4 w30, w31, w32, w33;  // head fragments in flight from LDS
            STREAM_STMT(STREAM_ASM_STEP_16,
                         : FRAG_TEMPS, STREAM_SB(sbv), STREAM_ACC3(acc3[0], acc3[1]),
                           [w30] "=&v"(w30), [w31] "=&v"(w31), [w32] "=&v"(w32), [w33] "=&v"(w33)
                         : STEP_COMMON(16), STREAM_HF_IN_B(hB00, hB01, hB10, hB11), [xpo] "v"(xpB), [xw] "v"(xw_addr),
                           [w3] "v"(w3_addr)
                         : "memory", "scc", STREAM_HEAD_CLOBBERS, STREAM_ACC2_CLOBBERS);
        }
#undef STEP_ODD
#undef STREAM_STMT
#undef STEP_EVEN
#undef STEP_LOADS
#undef STEP_COMMON
        {   // the buffers of steps 0, 1, 2 of the next batch: chunks 0 and 1 went where steps 15 and 16 sent them
            uint32_t w = wsv[2], l = lbv[2];
            wsv[2] = wsv[1], lbv[2] = lbv[1];
            wsv[1] = wsv[0], lbv[1] = lbv[0];
            wsv[0] = w, lbv[0] = l;
        }
        idc = check_ids(raw_c);
        idn = check_ids(raw_n);
        // Eq. 8 over the head accumulators
        uint32_t h16 = tid16;
        asm volatile("" : "+v"(h16));
        const uint32_t hb_addr = (uint32_t)(uintptr_t)b2buf + ((h16 >> 5) & 16);  // 16 bytes * g
        float hw[4], bb3[4];
        {
            u32x4 r0, r1, r2, r3;
            lds_load4_b128<NB2 * 128, 32>(hb_addr, r0, r1, r2, r3);  // [4g..] of the weights, +32 bytes: of the bias
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hw[e] = __uint_as_float(r0[e]);
                bb3[e] = __uint_as_float(r1[e]);
            }
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) part = fmaf(hw[e], sigmoid_hw(acc3[c][e] + bb3[e]), part);
            float other = __shfl_xor(part, 32);
            int64_t row = row0 + c * 32 + col;
            if (g == 0 && row < M) scores[row] = bad[c] ? __uint_as_float(0x7fc00000u) : part + other;
        }
        // the next batch's user pointers, validity, and its user term of hidden block 0 (the
        // start of the next batch hides that latency)
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            up[c] = upre + (size_t)idc.q[c] * H1 + 4 * g;
            bad[c] = idc.bad[c];
        }
        load_user_term0();
    }
    // the last two steps streamed chunks nobody reads; they must have landed before the LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

bool mfma_stream_supported(int D, int H1, int H2) { return D == 128 && H2 == 256 && H1 == 512; }

static inline uint16_t w_at(const uint16_t *W, int n_in, int row, int colm) { return W[(size_t)row * n_in + colm]; }

int build_stream_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream) {
    const int D = m->d_item, H1 = m->dims[1], H2 = m->dims[2], J = m->J, du = m->d_user;
    const int KS1 = D / 16, NB1 = H1 / 32, NB2 = H2 / 32;
    const int CHUNK_FR = KS1 + 2 * NB2;
    const size_t n_frag = (size_t)(NB1 + 1) * CHUNK_FR + 2 * NB2;
    std::vector<uint16_t> buf(n_frag * 512, 0);
    const uint16_t *W1 = (const uint16_t *)W_host[0], *W2 = (const uint16_t *)W_host[1],
                   *W3 = (const uint16_t *)W_host[2];
    for (int i = 0; i <= NB1; ++i) {
        uint16_t *chunk = buf.data() + (size_t)i * CHUNK_FR * 512;
        if (i < NB1)
            for (int s = 0; s < KS1; ++s)
                for (int l = 0; l < 64; ++l)
                    for (int j = 0; j < 8; ++j)
                        chunk[(size_t)s * 512 + l * 8 + j] =
                            w_at(W1, du + D, i * 32 + (l & 31), du + 16 * s + 8 * (l >> 5) + j);
        if (i > 0)
            for (int n2 = 0; n2 < NB2; ++n2)
                for (int s2 = 0; s2 < 2; ++s2)
                    for (int l = 0; l < 64; ++l)
                        for (int j = 0; j < 8; ++j)
                            chunk[(size_t)(KS1 + 2 * n2 + s2) * 512 + l * 8 + j] = w_at(
                                W2, H1, n2 * 32 + (l & 31), (i - 1) * 32 + 16 * s2 + 8 * (j / 4) + 4 * (l >> 5) + j % 4);
    }
    uint16_t *head = buf.data() + (size_t)(NB1 + 1) * CHUNK_FR * 512;
    for (int n2 = 0; n2 < NB2; ++n2)
        for (int s2 = 0; s2 < 2; ++s2)
            for (int l = 0; l < 64; ++l)
                for (int j = 0; j < 8; ++j)
                    if ((l & 31) < J)
                        head[(size_t)(2 * n2 + s2) * 512 + l * 8 + j] =
                            w_at(W3, H2, l & 31, n2 * 32 + 16 * s2 + 8 * (j / 4) + 4 * (l >> 5) + j % 4);
    m->frag_bytes = (int64_t)buf.size() * 2;
    ANN_HIP_TRY(hipMalloc(&m->frag_dev, (size_t)m->frag_bytes));
    ANN_HIP_TRY(hipMemcpyAsync(m->frag_dev, buf.data(), (size_t)m->frag_bytes, hipMemcpyHostToDevice, stream));
    ANN_HIP_TRY(hipStreamSynchronize(stream));
    return ANN_OK;
}

int launch_mlp_mfma_stream(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                           const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                           hipStream_t stream) {
    constexpr int H1 = 512;
    constexpr size_t smem = ((size_t)3 * 24 * 64 + 16 * 64 + 4 * 16 * 64) * 16 + (256 + 32) * 4;  // 72 + 16 + 64 + 1 KB (+ head constants)
    constexpr int TILE = 256;
    const bool f16 = m->dtype == ANN_F16;
    auto fn = f16 ? mlp_mfma2_stream_kernel<H1, true> : mlp_mfma2_stream_kernel<H1, false>;
    static std::atomic<uint32_t> raised[2];
    if (int rc = raise_lds_limit((const void *)fn, smem, m->device, raised[f16 ? 1 : 0]); rc != ANN_OK) return rc;
    int64_t tiles = (M_max + TILE - 1) / TILE;
    int grid = (int)(tiles < 256 ? tiles : 256);
    const float *b2 = m->b_dev + m->b_off[1], *b3 = m->b_dev + m->b_off[2];
    hipLaunchKernelGGL(fn, dim3(grid), dim3(ST_BLOCK), smem, stream, (const uint16_t *)g->emb, g->N, upre,
                       (const uint4 *)m->frag_dev, b2, b3, m->head_w_dev, m->J, pair_q, pair_id, M_dev, M_max, Q,
                       scores);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

}  // namespace gmpgr
