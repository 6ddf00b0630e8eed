// The relevance metric of Sec. 3.1 (1), Eq. 5-8, with 8-bit operands (the quantised deployment of
// Sec. 4.3 taken one step further than 16 bits): e4m3 item vectors, weights and hidden activations on
// v_mfma_f32_32x32x64_f8f6f4, fp32 accumulation.  Shapes served: 64-wide items with hidden 256 and 128 (all
// weights resident in LDS), 128-wide items with hidden 512 and 256 (see mlp_mfma2_f8_wide_kernel).
//
// Same transposed formulation as the bf16 kernels (H_out^T = W * H_in^T, weights are the A operand,
// the activations of 32 pairs the B operand), with a contraction of 64 per instruction: lane (m, g)
// of an operand holds 32 bytes, the contraction indices 32g .. 32g+31, and A's byte b meets B's byte b.
// The D layout is the one of every 32x32 MFMA: lane (pair, g) holds output units
// 8*(i/4) + 4g + i%4, i = 0..15.  Two consecutive 32-unit blocks therefore give a lane the 32 values
// that ARE its share of the next layer's B operand, once its weights are stored in the matching
// order ("fragment order", written by build_f8_fragments).
//
// Scales (all powers of two, so they only move exponents): every weight matrix is stored as
// e4m3(4 w); hidden layer 1 is held as e4m3(4 h), hidden layer 2 as e4m3(16 h).  With the user term
// and the biases pre-multiplied (4 * (W1_user u + b1), 16 * b2) the accumulators of a layer are
// already its activations at their scale: ReLU and the clamp to the largest e4m3 value are one
// v_med3_f32, the rounding one v_cvt_pk_fp8_f32 per two values.  The head accumulators are 64 x the
// logits.
//
// Narrow shape: all weights (52 KB) stay in LDS; a workgroup of eight waves, 64 pairs per wave.
#include <math.h>
#include <string.h>

#include <vector>

#include "common.h"

namespace gmpgr {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float E4M3_MAX = 448.f;
constexpr float F8_W_SCALE = 4.f;    // weights; hidden layer 1 is therefore held at 4 x its value, layer 2 at 16 x,
constexpr float F8_LOGIT_SCALE = 64.f;  // and the head's sums at 64 x

__device__ __forceinline__ f32x16 mfma_f8(const i32x8 &a, const i32x8 &b, const f32x16 &c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

// relu, clamp, round: 16 accumulator values -> half (bytes 16 * half .. + 15) of the lane's next B operand
__device__ __forceinline__ void quantize_half(const f32x16 &src, i32x8 &dst, int half) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int i = 4 * w;
        int v = 0;
        v = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(src[i], 0.f, E4M3_MAX),
                                            __builtin_amdgcn_fmed3f(src[i + 1], 0.f, E4M3_MAX), v, false);
        v = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(src[i + 2], 0.f, E4M3_MAX),
                                            __builtin_amdgcn_fmed3f(src[i + 3], 0.f, E4M3_MAX), v, true);
        dst[4 * half + w] = v;
    }
}

// Fragments, 2 KB each, stored as two 1 KB halves (lane l's bytes 0..15 at 16*l of the first half,
// bytes 16..31 at 16*l of the second):
//   [blk < H1/32]                       lane (m,g) byte b: e4m3(4 W1_item[32 blk + m][32g + b])
//   [H1/32 + (H2/32) c + n2], c < H1/64 lane (m,g) byte b: e4m3(4 W2[32 n2 + m][unit(c, g, b)])
//   [H1/32 + (H1/64)(H2/32) + p], p < H2/64              : e4m3(4 W3[m][unit(p, g, b)]), rows m >= J zero
//   unit(c, g, b) = 64c + 32 (b / 16) + 8 ((b % 16) / 4) + 4g + b % 4
template <int D, int H1, int H2, int CB, int WAVES>
__global__ void __launch_bounds__(64 * WAVES)
mlp_mfma2_f8_kernel(const uint8_t *__restrict__ emb, int64_t N, const float *__restrict__ upre,
                    const uint4 *__restrict__ frag, const float *__restrict__ b2s, const float *__restrict__ b3,
                    const float *__restrict__ head_w, int J, const int32_t *__restrict__ pair_q,
                    const int32_t *__restrict__ pair_id, const int32_t *__restrict__ M_dev, int64_t M_max, int32_t Q,
                    float *__restrict__ scores) {
    static_assert(D == 64, "one contraction step of 64 covers the item vector");
    constexpr int NB1 = H1 / 32, NC = H1 / 64, NB2 = H2 / 32, NP = H2 / 64;
    constexpr int N_FRAG = NB1 + NC * NB2 + NP;
    constexpr int BLOCK_T = 64 * WAVES;
    constexpr int RW = 32 * CB, TILE = RW * WAVES;
    extern __shared__ __align__(16) uint4 lds[];  // [N_FRAG][2][64]

    int64_t M = (int64_t)*M_dev;
    if (M > M_max) M = M_max;
    const int64_t n_tiles = (M + TILE - 1) / TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, col = lane & 31;
    for (int i = threadIdx.x; i < N_FRAG * 128; i += BLOCK_T) lds[i] = frag[i];
    __syncthreads();

    auto fragment = [&](int f) {
        const uint4 lo = lds[f * 128 + lane], hi = lds[f * 128 + 64 + lane];
        i32x8 a;
        a[0] = lo.x, a[1] = lo.y, a[2] = lo.z, a[3] = lo.w, a[4] = hi.x, a[5] = hi.y, a[6] = hi.z, a[7] = hi.w;
        return a;
    };

    float hw[4], bb3[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int j = 4 * g + i;
        hw[i] = j < J ? head_w[j] : 0.f;
        bb3[i] = j < J ? b3[j] : 0.f;
    }

    // Item rows are fetched one batch ahead (the head layer of the current batch hides the latency), the pair
    // ids two batches ahead.  Rows past the end read the last pair and are not stored.
    struct Ids {
        int32_t id[CB], q[CB];
        bool bad[CB];
    };
    auto load_ids = [&](int64_t tile) {
        Ids r;
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            int64_t row = tile * TILE + (int64_t)wave * RW + c * 32 + col;
            row = row < M ? row : M - 1;
            const int32_t v = pair_id[row], q = pair_q[row];
            r.bad[c] = ((uint64_t)(int64_t)v >= (uint64_t)N) | ((uint32_t)q >= (uint32_t)Q);
            r.id[c] = r.bad[c] ? 0 : v;
            r.q[c] = r.bad[c] ? 0 : q;
        }
        return r;
    };
    i32x8 x[CB];
    auto gather = [&](const Ids &ids) {
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const uint4 *src = (const uint4 *)(emb + (size_t)ids.id[c] * D + 32 * g);
            const uint4 lo = src[0], hi = src[1];
            x[c][0] = lo.x, x[c][1] = lo.y, x[c][2] = lo.z, x[c][3] = lo.w;
            x[c][4] = hi.x, x[c][5] = hi.y, x[c][6] = hi.z, x[c][7] = hi.w;
        }
    };
    Ids idc = load_ids(blockIdx.x), idn = load_ids((int64_t)blockIdx.x + gridDim.x);
    gather(idc);

#pragma unroll 1
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t row0 = tile * TILE + (int64_t)wave * RW;
        const float *up[CB];
        bool bad[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            up[c] = upre + (size_t)idc.q[c] * H1 + 4 * g;
            bad[c] = idc.bad[c];
        }
        idc = idn;                                      // the next batch ...
        idn = load_ids(tile + 2 * (int64_t)gridDim.x);  // ... and the one after it
        f32x16 acc2[NB2][CB];
        // the bias pointer is laundered once per batch: otherwise its loads are hoisted out of the batch
        // loop and their values carried (spilled) across it
        int opaque_zero = 0;
        asm volatile("" : "+s"(opaque_zero));
        const float *b2t = b2s + opaque_zero;
#pragma unroll
        for (int n2 = 0; n2 < NB2; ++n2) {
            f32x16 init;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                f32x4 bv = *(const f32x4 *)(b2t + n2 * 32 + 8 * t4 + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) init[4 * t4 + e] = bv[e];
            }
#pragma unroll
            for (int c = 0; c < CB; ++c) acc2[n2][c] = init;
        }
#pragma unroll 1
        for (int ch = 0; ch < NC; ++ch) {
            // layer 1, units 64 ch .. 64 ch + 63, one block of 32 at a time: accumulators start from the
            // (scaled) user term, their rounded ReLU is one half of the layer-2 operand
            i32x8 h1q[CB];
#pragma unroll
            for (int hb = 0; hb < 2; ++hb) {
                const i32x8 a = fragment(2 * ch + hb);
#pragma unroll
                for (int c = 0; c < CB; ++c) {
                    f32x16 acc1;
#pragma unroll
                    for (int t4 = 0; t4 < 4; ++t4) {
                        f32x4 pv = *(const f32x4 *)(up[c] + (2 * ch + hb) * 32 + 8 * t4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc1[4 * t4 + e] = pv[e];
                    }
                    acc1 = mfma_f8(a, x[c], acc1);
                    quantize_half(acc1, h1q[c], hb);
                }
            }
            // layer 2: every output unit consumes these 64 hidden units
#pragma unroll
            for (int n2 = 0; n2 < NB2; ++n2) {
                const i32x8 a = fragment(NB1 + NB2 * ch + n2);
#pragma unroll
                for (int c = 0; c < CB; ++c) acc2[n2][c] = mfma_f8(a, h1q[c], acc2[n2][c]);
            }
        }
        gather(idc);  // the item rows of the next batch: layer 1 of this one is done with the registers

        // head layer (rows >= J of its fragments are zero), then Eq. 8
        f32x16 acc3[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc3[c][i] = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const i32x8 a = fragment(NB1 + NC * NB2 + p);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                i32x8 h2q;
                quantize_half(acc2[2 * p][c], h2q, 0);
                quantize_half(acc2[2 * p + 1][c], h2q, 1);
                acc3[c] = mfma_f8(a, h2q, acc3[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float part = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float logit = acc3[c][i] * (1.0f / F8_LOGIT_SCALE) + bb3[i];
                part = fmaf(hw[i], sigmoid_hw(logit), part);
            }
            float other = __shfl_xor(part, 32);
            int64_t row = row0 + c * 32 + col;
            if (g == 0 && row < M) scores[row] = bad[c] ? __uint_as_float(0x7fc00000u) : part + other;
        }
    }
}

// The wide shape (128-wide items, hidden 512 and 256): 200 KB of e4m3 weights do not fit the LDS.  The
// second layer's (128 KB) and the head's fragments stay resident; the first layer's 64 KB are read by every
// wave straight from global memory (they are hot in L2: every wave of the chip reads the same 64 KB per batch),
// one block of 32 hidden units ahead of its use, so the main loop has no barrier and no staging.
// A batch is a handful of inline-assembly statements (text from gen_f8_wide_asm.py): the bias into the layer-2
// accumulators, per chunk of 64 hidden units layer 1 + conversion and layer 2, and the head layer.  The 256
// layer-2 accumulators of a wave fill the accumulation registers, which the statements name outright and list as
// clobbered (the head layer reads single registers of a tile, which an operand cannot express; the code between
// the statements has no use for accumulation registers, which a test checks on the compiled kernel).  The
// short-lived layer-1 accumulators and operands are pinned to fixed ordinary registers.  Hazards the compiler
// would otherwise handle are kept by hand inside the statements:
//   - a register written by a vector-ALU instruction is not read by an MFMA in the next two issue slots
//     (s_nop 1 in front of every such MFMA);
//   - an accumulator is not the target of two consecutive MFMAs (pairs 0 and 1 alternate);
//   - the vector ALU reads an MFMA result only after the MFMA has written it: 19 instruction slots after a
//     16-pass MFMA issued (a slot of a wave is four clocks, s_nop n takes n + 1 slots), which the statements
//     fill with other work wherever they can.
// MFMAs and the idle cycles that let the last of them finish are ONE statement: between two statements the
// compiler may copy a register tuple (it does, to free one for the next block's user term), and such a copy
// right behind an MFMA reads a result that is not there yet.
#include "mlp_mfma_f8_wide_asm.inc"  // F8W_ASM_INIT / _A / _B / _HEAD and their operand and clobber lists

// Fragments as above with two contraction steps in layer 1: fragment KS*blk + ks holds W1_item[32 blk + m][64 ks + 32g + b].
template <int D, int H1, int H2>
__global__ void __launch_bounds__(256)
mlp_mfma2_f8_wide_kernel(const uint8_t *__restrict__ emb, int64_t N, const float *__restrict__ upre,
                         const uint4 *__restrict__ frag, const float *__restrict__ b2s, const float *__restrict__ b3,
                         const float *__restrict__ head_w, int J, const int32_t *__restrict__ pair_q,
                         const int32_t *__restrict__ pair_id, const int32_t *__restrict__ M_dev, int64_t M_max,
                         int32_t Q, float *__restrict__ scores) {
    constexpr int CB = 2, WAVES = 4;
    constexpr int KS = D / 64, NB1 = H1 / 32, NC = H1 / 64, NB2 = H2 / 32, NP = H2 / 64;
    static_assert(KS == 2 && NB2 == 8, "the generated chunk statements assume these");
    constexpr int N_W1 = NB1 * KS;                 // fragments that stay in global memory
    constexpr int N_LDS = NC * NB2 + NP;           // fragments resident in LDS
    constexpr int BLOCK_T = 64 * WAVES;
    constexpr int RW = 32 * CB, TILE = RW * WAVES;
    extern __shared__ __align__(16) uint4 lds[];   // [N_LDS][2][64] fragments, then the H2 layer-2 biases

    int64_t M = (int64_t)*M_dev;
    if (M > M_max) M = M_max;
    const int64_t n_tiles = (M + TILE - 1) / TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, col = lane & 31;
    for (int i = threadIdx.x; i < N_LDS * 128; i += BLOCK_T) lds[i] = frag[(size_t)N_W1 * 128 + i];
    for (int i = threadIdx.x; i < H2 / 4; i += BLOCK_T) lds[N_LDS * 128 + i] = ((const uint4 *)b2s)[i];
    __syncthreads();

    auto w1_fragment = [&](int f) {  // straight from global memory
        const uint4 lo = frag[(size_t)f * 128 + lane], hi = frag[(size_t)f * 128 + 64 + lane];
        i32x8 a;
        a[0] = lo.x, a[1] = lo.y, a[2] = lo.z, a[3] = lo.w, a[4] = hi.x, a[5] = hi.y, a[6] = hi.z, a[7] = hi.w;
        return a;
    };

    float hw[4], bb3[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int j = 4 * g + i;
        hw[i] = j < J ? head_w[j] : 0.f;
        bb3[i] = j < J ? b3[j] : 0.f;
    }

    struct Ids {
        int32_t id[CB], q[CB];
        bool bad[CB];
    };
    auto load_ids = [&](int64_t tile) {
        Ids r;
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            int64_t row = tile * TILE + (int64_t)wave * RW + c * 32 + col;
            row = row < M ? row : M - 1;  // rows past the end read the last pair and are not stored
            const int32_t v = pair_id[row], q = pair_q[row];
            r.bad[c] = ((uint64_t)(int64_t)v >= (uint64_t)N) | ((uint32_t)q >= (uint32_t)Q);
            r.id[c] = r.bad[c] ? 0 : v;
            r.q[c] = r.bad[c] ? 0 : q;
        }
        return r;
    };
    i32x8 x[CB][KS];
    auto gather = [&](const Ids &ids) {
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 *src = (const uint4 *)(emb + (size_t)ids.id[c] * D + 64 * ks + 32 * g);
                const uint4 lo = src[0], hi = src[1];
                x[c][ks][0] = lo.x, x[c][ks][1] = lo.y, x[c][ks][2] = lo.z, x[c][ks][3] = lo.w;
                x[c][ks][4] = hi.x, x[c][ks][5] = hi.y, x[c][ks][6] = hi.z, x[c][ks][7] = hi.w;
            }
    };
    Ids idc = load_ids(blockIdx.x), idn = load_ids((int64_t)blockIdx.x + gridDim.x);
    gather(idc);
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds + 16u * (uint32_t)lane;
    const uint32_t w3_addr = lds_addr + (uint32_t)(NC * NB2) * 2048u;                           // head fragments
    const uint32_t b2_addr = (uint32_t)(uintptr_t)lds + (uint32_t)N_LDS * 2048u + 16u * (uint32_t)g;  // bias copy
    // Two sets (P: even blocks, Q: odd blocks) of first-layer fragments and of layer-1 accumulators: once both
    // blocks of a chunk are contracted, the sets receive the next chunk's fragments and user term, which travel
    // while layer 2 of this chunk runs.  An empty memory-clobbering statement keeps the compiler from moving
    // loads across it: requests are issued where they are written.
#define F8_FENCE asm volatile("" ::: "memory")
    i32x8 w1P[KS], w1Q[KS];
    f32x16 accP[CB], accQ[CB];
    auto load_user_term = [&](f32x16 (&acc)[CB], const float *const (&upc)[CB], int blk) {
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                f32x4 pv = *(const f32x4 *)(upc[c] + blk * 32 + 8 * t4);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[c][4 * t4 + e] = pv[e];
            }
    };
    const float *up[CB];
    bool bad[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        up[c] = upre + (size_t)idc.q[c] * H1 + 4 * g;
        bad[c] = idc.bad[c];
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        w1P[ks] = w1_fragment(ks);
        w1Q[ks] = w1_fragment(KS + ks);
    }
    load_user_term(accP, up, 0);
    load_user_term(accQ, up, 1);

#pragma unroll 1
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t row0 = tile * TILE + (int64_t)wave * RW;
        bool bad_now[CB];
        const float *upn[CB];   // the next batch's user rows: its block 0 is requested during this batch's last block
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            bad_now[c] = bad[c];
            upn[c] = upre + (size_t)idn.q[c] * H1 + 4 * g;
        }
        // The 16 layer-2 accumulator tiles live in the accumulation registers, which only the assembly statements
        // of this loop touch (see gen_f8_wide_asm.py).  They start from the bias, read from its LDS copy straight
        // into them; the first chunk's statement A ends with a full wait for LDS reads.
        asm volatile(F8W_ASM_INIT : : [b2] "v"(b2_addr) : "memory", F8W_ACC2_CLOBBERS);
        uint32_t wc = lds_addr;  // this lane's 16 bytes of the chunk's first layer-2 fragment
#pragma unroll 1
        for (int ch = 0; ch < NC; ++ch) {
            // statement A: layer 1 of hidden units 64 ch .. 64 ch + 63 (even block from set P, odd block from set Q)
            // and their conversion; statement B: layer 2 over them.  See gen_f8_wide_asm.py.
            i32x8 h0, h1, f0, f1, f2, f3;
            asm volatile(F8W_ASM_A
                         : F8W_ACC_P(accP[0], accP[1]), F8W_ACC_Q(accQ[0], accQ[1]), F8W_H_OUT(h0, h1),
                           F8W_FRAGS_OUT(f0, f1, f2, f3)
                         : [wP0] "v"(w1P[0]), [wP1] "v"(w1P[1]), [wQ0] "v"(w1Q[0]), [wQ1] "v"(w1Q[1]),
                           [x00] "v"(x[0][0]), [x01] "v"(x[0][1]), [x10] "v"(x[1][0]), [x11] "v"(x[1][1]),
                           [wc] "v"(wc), [fmax] "s"(E4M3_MAX)
                         : "memory");
            // both sets are free now: they receive the next chunk's fragments and user term (after the last
            // chunk: those of the next batch's first chunk), which travel while layer 2 runs
            const bool wrap = (ch + 1 == NC);
            const int nb = wrap ? 0 : 2 * ch + 2;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                w1P[ks] = w1_fragment(nb * KS + ks);
                w1Q[ks] = w1_fragment((nb + 1) * KS + ks);
            }
            if (wrap) {
                load_user_term(accP, upn, 0);
                load_user_term(accQ, upn, 1);
            } else {
                load_user_term(accP, up, nb);
                load_user_term(accQ, up, nb + 1);
            }
            asm volatile(F8W_ASM_B
                         : F8W_FRAGS_IO(f0, f1, f2, f3)
                         : F8W_H_IN(h0, h1), [wc] "v"(wc)
                         : "memory", F8W_ACC2_CLOBBERS);
            wc += NB2 * 2048;
        }
        // ids: the next batch becomes the current one, the one after it is requested
        idc = idn;
        idn = load_ids(tile + 2 * (int64_t)gridDim.x);
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            up[c] = upn[c];
            bad[c] = idc.bad[c];
        }
        gather(idc);  // the item rows of the next batch: layer 1 of this one is done with the registers
        F8_FENCE;

        // head layer: the finished layer-2 tiles leave the accumulation registers through ReLU, clamp and e4m3
        // rounding, pair of tiles by pair of tiles, each followed by its head fragment's two MFMAs
        f32x16 acc3[CB];
        asm volatile(F8W_ASM_HEAD
                     : [q30] "=&v"(acc3[0]), [q31] "=&v"(acc3[1])
                     : [w3] "v"(w3_addr), [fmax] "s"(E4M3_MAX)
                     : "memory", F8W_HEAD_CLOBBERS, F8W_ACC2_CLOBBERS);
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float part = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float logit = acc3[c][i] * (1.0f / F8_LOGIT_SCALE) + bb3[i];
                part = fmaf(hw[i], sigmoid_hw(logit), part);
            }
            float other = __shfl_xor(part, 32);
            int64_t row = row0 + c * 32 + col;
            if (g == 0 && row < M) scores[row] = bad_now[c] ? __uint_as_float(0x7fc00000u) : part + other;
        }
    }
}

// ---- host side: e4m3 encoding of the weights (nearest even; the format: sign, 4 exponent bits with
// bias 7, 3 mantissa bits, subnormals below 2^-6, largest value 448) ----
static bool encode_e4m3(float v, uint8_t *code) {
    const uint8_t sign = signbit(v) ? 0x80 : 0;
    const float a = fabsf(v);
    if (!(a <= E4M3_MAX)) return false;
    if (a < 0.015625f) {  // subnormal spacing 2^-9; 8 steps carry into the first normal code by themselves
        *code = (uint8_t)(sign | (uint8_t)nearbyintf(a * 512.f));
        return true;
    }
    int e;
    const float f = frexpf(a, &e);                       // a = f 2^e, f in [0.5, 1)
    int mant = (int)nearbyintf((2.f * f - 1.f) * 8.f);   // 0..8
    int ex = e - 1 + 7;
    if (mant == 8) mant = 0, ++ex;
    *code = (uint8_t)(sign | (ex << 3) | mant);
    return true;
}

static inline float bf16_value(uint16_t bits) {
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

bool f8_supported(const int32_t *dims, int32_t n_layers, int32_t d_user) {
    if (n_layers != 3 || d_user < 1) return false;
    const int J = dims[3];
    if (J < 1 || J > MAX_HEADS) return false;
    const int D = dims[0] - d_user;
    return (D == 64 && dims[1] == 256 && dims[2] == 128) || (D == 128 && dims[1] == 512 && dims[2] == 256);
}

static inline int f8_unit(int c, int g, int b) { return 64 * c + 32 * (b / 16) + 8 * ((b % 16) / 4) + 4 * g + b % 4; }

// W_host: bf16 matrices as for the bf16 metric.  Fails (ANN_EINVAL) if a weight times 4 exceeds 448.
int build_f8_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream) {
    const int D = m->d_item, H1 = m->dims[1], H2 = m->dims[2], J = m->J, du = m->d_user;
    const int KS = D / 64, NB1 = H1 / 32, NC = H1 / 64, NB2 = H2 / 32, NP = H2 / 64;
    const int n_w1 = NB1 * KS;
    const int n_frag = n_w1 + NC * NB2 + NP;
    std::vector<uint8_t> buf((size_t)n_frag * 2048, 0);
    const uint16_t *W1 = (const uint16_t *)W_host[0], *W2 = (const uint16_t *)W_host[1],
                   *W3 = (const uint16_t *)W_host[2];
    bool ok = true;
    auto put = [&](int f, int l, int b, uint16_t w) {
        uint8_t code = 0;
        ok &= encode_e4m3(F8_W_SCALE * bf16_value(w), &code);
        buf[(size_t)f * 2048 + (size_t)(b / 16) * 1024 + (size_t)l * 16 + b % 16] = code;
    };
    for (int l = 0; l < 64; ++l) {
        const int mrow = l & 31, g = l >> 5;
        for (int b = 0; b < 32; ++b) {
            for (int blk = 0; blk < NB1; ++blk)
                for (int ks = 0; ks < KS; ++ks)
                    put(blk * KS + ks, l, b, W1[(size_t)(32 * blk + mrow) * (du + D) + du + 64 * ks + 32 * g + b]);
            for (int c = 0; c < NC; ++c)
                for (int n2 = 0; n2 < NB2; ++n2)
                    put(n_w1 + NB2 * c + n2, l, b, W2[(size_t)(32 * n2 + mrow) * H1 + f8_unit(c, g, b)]);
            if (mrow < J)
                for (int p = 0; p < NP; ++p) put(n_w1 + NC * NB2 + p, l, b, W3[(size_t)mrow * H2 + f8_unit(p, g, b)]);
        }
    }
    if (!ok) {
        set_error("a weight is too large for the 8-bit metric (|4 w| must not exceed 448)");
        return ANN_EINVAL;
    }
    m->frag_bytes = (int64_t)buf.size();
    ANN_HIP_TRY(hipMalloc(&m->frag_dev, (size_t)m->frag_bytes));
    ANN_HIP_TRY(hipMemcpyAsync(m->frag_dev, buf.data(), (size_t)m->frag_bytes, hipMemcpyHostToDevice, stream));
    ANN_HIP_TRY(hipStreamSynchronize(stream));  // buf is freed on return
    return ANN_OK;
}

int launch_mlp_mfma_f8(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                       const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                       hipStream_t stream) {
    if (M_max <= 0) return ANN_OK;
    if (m->d_item == 128) {
        constexpr int D = 128, H1 = 512, H2 = 256, TILE = 256;
        constexpr size_t smem = (size_t)((H1 / 64) * (H2 / 32) + H2 / 64) * 2048 + (size_t)H2 * 4;  // 136 + 1 KB
        auto fn = mlp_mfma2_f8_wide_kernel<D, H1, H2>;
        static std::atomic<uint32_t> raised;
        if (int rc = raise_lds_limit((const void *)fn, smem, m->device, raised); rc != ANN_OK) return rc;
        int64_t tiles = (M_max + TILE - 1) / TILE;
        int grid = (int)(tiles < 256 ? tiles : 256);
        hipLaunchKernelGGL(fn, dim3(grid), dim3(256), smem, stream, (const uint8_t *)g->emb, g->N, upre,
                           (const uint4 *)m->frag_dev, m->b_dev + m->b_off[1], m->b_dev + m->b_off[2], m->head_w_dev,
                           m->J, pair_q, pair_id, M_dev, M_max, Q, scores);
        ANN_HIP_TRY(hipGetLastError());
        return ANN_OK;
    }
    constexpr int D = 64, H1 = 256, H2 = 128, CB = 2, WAVES = 8;
    constexpr int N_FRAG = H1 / 32 + (H1 / 64) * (H2 / 32) + H2 / 64;
    constexpr size_t smem = (size_t)N_FRAG * 2048;  // 52 KB
    constexpr int TILE = 32 * CB * WAVES;
    auto fn = mlp_mfma2_f8_kernel<D, H1, H2, CB, WAVES>;
    static std::atomic<uint32_t> raised;
    if (int rc = raise_lds_limit((const void *)fn, smem, m->device, raised); rc != ANN_OK) return rc;
    int64_t tiles = (M_max + TILE - 1) / TILE;
    int grid = (int)(tiles < 256 ? tiles : 256);
    hipLaunchKernelGGL(fn, dim3(grid), dim3(64 * WAVES), smem, stream, (const uint8_t *)g->emb, g->N, upre,
                       (const uint4 *)m->frag_dev, m->b_dev + m->b_off[1], m->b_dev + m->b_off[2], m->head_w_dev, m->J,
                       pair_q, pair_id, M_dev, M_max, Q, scores);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

// out[i] = e4m3(scale * in[i]), magnitudes above 448 clamped (the conversion instruction would give NaN)
template <bool BF16>
__global__ void __launch_bounds__(256)
quantize_e4m3_kernel(const void *__restrict__ in, uint8_t *__restrict__ out, int64_t n, float scale) {
    const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i0 >= n) return;
    float v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int64_t i = i0 + t < n ? i0 + t : n - 1;
        const float f = BF16 ? __uint_as_float((uint32_t)((const uint16_t *)in)[i] << 16) : ((const float *)in)[i];
        v[t] = __builtin_amdgcn_fmed3f(f * scale, -E4M3_MAX, E4M3_MAX);
    }
    int r = 0;
    r = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], r, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], r, true);
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (i0 + t < n) out[i0 + t] = (uint8_t)((uint32_t)r >> (8 * t));
}

int launch_quantize_e4m3(const void *in, int dtype, int64_t n, float scale, uint8_t *out, hipStream_t stream) {
    if (n == 0) return ANN_OK;
    const int64_t groups = (n + 3) / 4;
    const unsigned grid = (unsigned)((groups + 255) / 256);
    if (dtype == ANN_BF16)
        hipLaunchKernelGGL(quantize_e4m3_kernel<true>, dim3(grid), dim3(256), 0, stream, in, out, n, scale);
    else
        hipLaunchKernelGGL(quantize_e4m3_kernel<false>, dim3(grid), dim3(256), 0, stream, in, out, n, scale);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

}  // namespace gmpgr
