// Relevance metric of Sec. 3.1 (1), Eq. 5-8, as fused bf16 MFMA GEMM chains on gfx950.
//
// The dense pair list produced by the packing step (Algorithm 2) is cut into batches of
// TILE pairs; a workgroup of four waves takes one batch, each wave owns RW = 32*CB pairs of
// it and carries them through ALL layers without the activations ever leaving registers.
//
// Transposed formulation.  Every layer is computed as  H_out^T = W * H_in^T  with
// v_mfma_f32_32x32x16_bf16: the weights are the A operand (32 output units x 16 inputs), the
// activations of 32 pairs are the B operand (16 inputs x 32 pairs).  In the D layout a lane
// holds, for ITS pair (lane % 32), output units  8*(i/4) + 4*(lane/32) + i%4  (i = 0..15).
// Since the contraction index of the next layer may be visited in any order, those 16 values
// (ReLU, rounded to bf16) ARE two B operands of the next layer, provided its weights are
// stored in the matching input order.  ann_mlp_load writes the weights once in exactly the
// order the lanes read them ("fragment order": 1 KB = 64 lanes x 8 bf16 per MFMA operand).
//
// Layer 1 is split as  W1 [u ; v] + b1 = (W1_user u + b1) + W1_item v  (Eq. 5, 7): the first
// term depends on the query only and is computed once per search (user_pre_kernel, fp32);
// it initialises the layer-1 accumulators, so only the item half is contracted per pair.
//
// The weights of this kernel's shapes fill most of the LDS, so a CU runs one workgroup; it has
// eight waves (two per SIMD, 256 registers each) so that one wave's item-row gather and
// conversions overlap the other's MFMAs.
//
// Weights do not fit in registers and (for the largest metric) not in LDS either: they are
// streamed through LDS in chunks, chunk nb = the 32 layer-1 units nb*32.. and the slab of
// layer-2 weights that consumes exactly those units, double buffered; when all chunks fit
// they are loaded once and stay resident.
//
// Numerics (bf16 mode of the library): bf16 inputs and weights, fp32 accumulation inside the
// MFMA, hidden activations rounded to bf16 (nearest even) after ReLU, head logits, sigmoid
// and the weighted sum (Eq. 8) in fp32.
#include <vector>

#include "common.h"

namespace gmpgr {

// Eight 16-bit operands of an MFMA.  The two 16-bit formats (bf16, and IEEE binary16 when the template flag
// F16 is set) share every kernel: an operand is carried as bf16x8 whatever it holds, and only the three places
// that look inside differ -- the MFMA instruction, the rounding of fresh hidden units, the widening of the
// user vector and its weights for the per-query term.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MF_BLOCK = 256;
constexpr int MF_WAVES = 4;

// Register plan.  The layer-2 accumulators of a wave fill all 256 accumulation registers
// (AGPRs) for the whole batch; the compiler keeps the destination of every MFMA it selects
// itself in AGPRs, which is right for layer 2 but leaves no room for the short-lived layer-1
// and head accumulators.  Those two use mfma_vgpr_pair(): the same instruction written as inline
// assembly with the accumulator pinned to ordinary VGPRs.  The hazard rules the compiler
// would otherwise enforce are kept by hand there:
//   - a VGPR written by a vector-ALU instruction may not be read by an MFMA in the next two
//     issue slots: every mfma_vgpr_pair starts with s_nop 1;
//   - an accumulator is never used by two consecutive MFMAs: callers alternate two of them;
//   - the vector ALU may read an MFMA result only after the MFMA has drained: the last pair of a group
//     carries the idle cycles in its own statement.  (The compiler does not know that the result of such a
//     statement arrives later: a register copy of an accumulator placed between the last MFMA and a
//     separate statement of idle cycles would read too early; it was seen to do that in the 8-bit kernel
//     for the wide metric.)
// One weight fragment against both column blocks of pairs.  LAST: the group ends here; the idle cycles that
// let its MFMAs finish are part of the same statement, so that nothing can come between them (an 8-pass MFMA
// has written its result 11 instruction slots after it issued; s_nop n takes n + 1 slots of four clocks).
#define MFMA_PAIR_TEXT(T) "s_nop 1\n\tv_mfma_f32_32x32x16_" T " %0, %2, %3, %0\n\tv_mfma_f32_32x32x16_" T " %1, %2, %4, %1"
template <bool LAST, bool F16>
__device__ __forceinline__ void mfma_vgpr_pair(f32x16 &acc0, f32x16 &acc1, const bf16x8 &a, const bf16x8 &b0,
                                               const bf16x8 &b1) {
    if (LAST && F16)
        asm volatile(MFMA_PAIR_TEXT("f16") "\n\ts_nop 13" : "+v"(acc0), "+v"(acc1) : "v"(a), "v"(b0), "v"(b1));
    else if (LAST)
        asm volatile(MFMA_PAIR_TEXT("bf16") "\n\ts_nop 13" : "+v"(acc0), "+v"(acc1) : "v"(a), "v"(b0), "v"(b1));
    else if (F16)
        asm volatile(MFMA_PAIR_TEXT("f16") : "+v"(acc0), "+v"(acc1) : "v"(a), "v"(b0), "v"(b1));
    else
        asm volatile(MFMA_PAIR_TEXT("bf16") : "+v"(acc0), "+v"(acc1) : "v"(a), "v"(b0), "v"(b1));
}
#undef MFMA_PAIR_TEXT

// acc += A * B with the accumulator where the compiler puts it (the accumulation registers)
template <bool F16>
__device__ __forceinline__ f32x16 mfma16(const bf16x8 &a, const bf16x8 &b, const f32x16 &acc) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}

// ReLU and rounding (nearest even) of half a tile of fresh hidden units to the metric's 16-bit format
template <bool F16>
__device__ __forceinline__ bf16x8 relu_pack(const f32x16 &acc, int half) {
    f32x8 v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = fmaxf(acc[half * 8 + j], 0.f);
    if constexpr (F16)
        return __builtin_bit_cast(bf16x8, __builtin_convertvector(v, f16x8));
    else
        return __builtin_convertvector(v, bf16x8);
}

template <bool F16>
__device__ __forceinline__ float widen16(uint16_t bits) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, bits);
    else return __uint_as_float(((uint32_t)bits) << 16);
}

// upre[q][n] = b1[n] + sum_{i < d_user} W1[n][i] * u_q[i]   (fp32 FMA chain in index order)
template <bool F16>
__global__ void __launch_bounds__(256)
user_pre_kernel(const uint16_t *__restrict__ W1, int n_in, int d_user, int H1, const float *__restrict__ b1,
                const uint16_t *__restrict__ users, int Q, float *__restrict__ upre, float out_scale) {
    extern __shared__ float u_s[];
    const int q = blockIdx.x;
    for (int i = threadIdx.x; i < d_user; i += blockDim.x)
        u_s[i] = widen16<F16>(users[(size_t)q * d_user + i]);
    __syncthreads();
    for (int n = threadIdx.x; n < H1; n += blockDim.x) {
        float acc = b1[n];
        const uint16_t *row = W1 + (size_t)n * n_in;
        for (int i = 0; i < d_user; ++i) acc = fmaf(widen16<F16>(row[i]), u_s[i], acc);
        upre[(size_t)q * H1 + n] = acc * out_scale;  // a power of two (1 for the bf16 kernels): exact
    }
}

// Fragment-ordered weights, all bf16, 1 KB per fragment (lane l at byte 16*l):
//   chunk nb (nb < H1/32), CHUNK = (D/16 + 2*H2/32) fragments:
//     [s < D/16]            lane (m,g): W1_item[nb*32+m][16s + 8g + j],                  j < 8
//     [D/16 + 2*n2 + s2]    lane (m,g): W2[n2*32+m][nb*32 + 16*s2 + 8*(j/4) + 4g + j%4], j < 8
//   then the head layer, H2/16 fragments, rows >= J are zero:
//     [2*n2 + s2]           lane (m,g): W3[m][n2*32 + 16*s2 + 8*(j/4) + 4g + j%4]
template <int D, int H1, int H2, int CB, bool RESIDENT, int WAVES, bool F16>
__global__ void __launch_bounds__(64 * WAVES)
mlp_mfma2_kernel(const uint16_t *__restrict__ emb, int64_t N, const float *__restrict__ upre,
                 const uint4 *__restrict__ frag, const float *__restrict__ b2, const float *__restrict__ b3,
                 const float *__restrict__ head_w, int J, const int32_t *__restrict__ pair_q,
                 const int32_t *__restrict__ pair_id, const int32_t *__restrict__ M_dev, int64_t M_max, int32_t Q,
                 float *__restrict__ scores) {
    constexpr int KS1 = D / 16, NB1 = H1 / 32, NB2 = H2 / 32;
    constexpr int CHUNK_FR = KS1 + 2 * NB2;          // fragments per chunk
    constexpr int CHUNK_U4 = CHUNK_FR * 64;          // uint4 per chunk
    constexpr int W3_FR = 2 * NB2;
    constexpr int BLOCK_T = 64 * WAVES;
    constexpr int RW = 32 * CB, TILE = RW * WAVES;
    constexpr int NBUF = RESIDENT ? NB1 : 2;
    constexpr int ST = (CHUNK_U4 + BLOCK_T - 1) / BLOCK_T;  // staged uint4 per thread and chunk
    extern __shared__ __align__(16) uint4 lds[];
    uint4 *wbuf = lds;                                // [NBUF][CHUNK_U4]
    uint4 *w3buf = lds + (size_t)NBUF * CHUNK_U4;     // [W3_FR * 64]

    int64_t M = (int64_t)*M_dev;
    if (M > M_max) M = M_max;
    const int64_t n_tiles = (M + TILE - 1) / TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, col = lane & 31;

    // head-layer fragments, and either every chunk (resident) or chunk 0
    for (int i = threadIdx.x; i < W3_FR * 64; i += BLOCK_T) w3buf[i] = frag[(size_t)NB1 * CHUNK_U4 + i];
    {
        const int n_pre = RESIDENT ? NB1 * CHUNK_U4 : CHUNK_U4;
        for (int i = threadIdx.x; i < n_pre; i += BLOCK_T) wbuf[i] = frag[i];
    }
    __syncthreads();

    float hw[4], bb3[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int j = 4 * g + i;
        hw[i] = j < J ? head_w[j] : 0.f;
        bb3[i] = j < J ? b3[j] : 0.f;
    }

    // Item rows are fetched one batch ahead, into the registers the layer-1 MFMAs of the current
    // batch have finished with (its last layer-2 block and the head layer hide the latency); the
    // pair ids run two batches ahead.  Rows past the end read the last pair and are not stored.
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
    bf16x8 xf[CB][KS1];
    auto gather = [&](const Ids &ids) {
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const bf16x8 *src = (const bf16x8 *)(emb + (size_t)ids.id[c] * D) + g;
#pragma unroll
            for (int s = 0; s < KS1; ++s) xf[c][s] = src[2 * s];
        }
    };
    Ids idc = load_ids(blockIdx.x), idn = load_ids((int64_t)blockIdx.x + gridDim.x);
    gather(idc);

    int cur = 0;
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
        idc = idn;                                             // the next batch ...
        idn = load_ids(tile + 2 * (int64_t)gridDim.x);         // ... and the one after it
        f32x16 acc2[NB2][CB];
        // the bias pointer is laundered once per batch: otherwise the loads below are hoisted
        // out of the batch loop and their 16*NB2 values are carried (spilled) across it
        int opaque_zero = 0;
        asm volatile("" : "+s"(opaque_zero));
        const float *b2t = b2 + opaque_zero;
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
        for (int nb = 0; nb < NB1; ++nb) {
            const uint4 *wc = wbuf + (size_t)(RESIDENT ? nb : cur) * CHUNK_U4;
            uint4 stage[ST];
            if (!RESIDENT) {
                const int nxt = (nb + 1 == NB1) ? 0 : nb + 1;
                const uint4 *srcw = frag + (size_t)nxt * CHUNK_U4;
#pragma unroll
                for (int t = 0; t < ST; ++t) {
                    int i = threadIdx.x + t * BLOCK_T;
                    if (i < CHUNK_U4) stage[t] = srcw[i];
                }
            }
            // layer 1, units nb*32 .. nb*32+31: accumulators start from the per-query user term
            f32x16 acc1[CB];
#pragma unroll
            for (int c = 0; c < CB; ++c) {
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4) {
                    f32x4 pv = *(const f32x4 *)(up[c] + nb * 32 + 8 * t4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc1[c][4 * t4 + e] = pv[e];
                }
            }
#pragma unroll
            for (int s = 0; s < KS1; ++s) {
                bf16x8 a = *(const bf16x8 *)(wc + s * 64 + lane);
                static_assert(CB == 2, "pairs 0 and 1 alternate");
                if (s == KS1 - 1) mfma_vgpr_pair<true, F16>(acc1[0], acc1[1], a, xf[0][s], xf[1][s]);
                else mfma_vgpr_pair<false, F16>(acc1[0], acc1[1], a, xf[0][s], xf[1][s]);
            }
            bf16x8 hf[CB][2];
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                hf[c][0] = relu_pack<F16>(acc1[c], 0);
                hf[c][1] = relu_pack<F16>(acc1[c], 1);
            }
            // layer 2: every output unit consumes these 32 hidden units
#pragma unroll
            for (int n2 = 0; n2 < NB2; ++n2) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    bf16x8 a = *(const bf16x8 *)(wc + (KS1 + 2 * n2 + s2) * 64 + lane);
#pragma unroll
                    for (int c = 0; c < CB; ++c)
                        acc2[n2][c] = mfma16<F16>(a, hf[c][s2], acc2[n2][c]);
                }
            }
            if (!RESIDENT) {
                uint4 *dst = wbuf + (size_t)(cur ^ 1) * CHUNK_U4;
#pragma unroll
                for (int t = 0; t < ST; ++t) {
                    int i = threadIdx.x + t * BLOCK_T;
                    if (i < CHUNK_U4) dst[i] = stage[t];
                }
                __syncthreads();
                cur ^= 1;
            }
        }

        gather(idc);  // the item rows of the next batch: layer 1 of this one is done with the registers

        // head layer (rows >= J of the fragments are zero), then Eq. 8
        static_assert(CB >= 2, "two accumulators must alternate");
        f32x16 acc3[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc3[c][i] = 0.f;
#pragma unroll
        for (int n2 = 0; n2 < NB2; ++n2) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                bf16x8 a = *(const bf16x8 *)(w3buf + (2 * n2 + s2) * 64 + lane);
                const bf16x8 h0 = relu_pack<F16>(acc2[n2][0], s2), h1 = relu_pack<F16>(acc2[n2][1], s2);
                if (n2 == NB2 - 1 && s2 == 1) mfma_vgpr_pair<true, F16>(acc3[0], acc3[1], a, h0, h1);
                else mfma_vgpr_pair<false, F16>(acc3[0], acc3[1], a, h0, h1);
            }
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float part = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) part = fmaf(hw[i], sigmoid_hw(acc3[c][i] + bb3[i]), part);
            float other = __shfl_xor(part, 32);
            int64_t row = row0 + c * 32 + col;
            if (g == 0 && row < M) scores[row] = bad[c] ? __uint_as_float(0x7fc00000u) : part + other;
        }
    }
}

// One hidden layer (the metric of the 10^8-item configuration, 128 -> 256 -> J): the same scheme
// without the middle layer.  Per block of 32 hidden units: layer 1 from the user term, ReLU,
// bf16, and at once the two head MFMAs that consume those units; nothing but 2 x 16 head
// accumulators lives across blocks.  All weights (D/16 + 2 fragments per block) stay in LDS.
// The kernel is bound by the item-row gather, not by the MFMAs (about 250 flop per gathered
// byte, below the ridge of the chip), so its few registers and 48 KB of LDS are what matter:
// three workgroups share a CU and hide each other's gather latency.
// Fragment order: block nb: [s < D/16] W1_item as above; [D/16 + s2] lane (m,g):
// W_head[m][nb*32 + 16*s2 + 8*(j/4) + 4g + j%4], rows >= J zero.
template <int D, int H1, int CB, bool F16>
__global__ void __launch_bounds__(MF_BLOCK)
mlp_mfma1_kernel(const uint16_t *__restrict__ emb, int64_t N, const float *__restrict__ upre,
                 const uint4 *__restrict__ frag, const float *__restrict__ b_head, const float *__restrict__ head_w,
                 int J, const int32_t *__restrict__ pair_q, const int32_t *__restrict__ pair_id,
                 const int32_t *__restrict__ M_dev, int64_t M_max, int32_t Q, float *__restrict__ scores) {
    constexpr int KS1 = D / 16, NB1 = H1 / 32;
    constexpr int BLK_FR = KS1 + 2;
    constexpr int RW = 32 * CB, TILE = RW * MF_WAVES;
    extern __shared__ __align__(16) uint4 lds[];  // [NB1][BLK_FR][64]

    int64_t M = (int64_t)*M_dev;
    if (M > M_max) M = M_max;
    const int64_t n_tiles = (M + TILE - 1) / TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, col = lane & 31;
    for (int i = threadIdx.x; i < NB1 * BLK_FR * 64; i += MF_BLOCK) lds[i] = frag[i];
    __syncthreads();

    float hw[4], bh[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int j = 4 * g + i;
        hw[i] = j < J ? head_w[j] : 0.f;
        bh[i] = j < J ? b_head[j] : 0.f;
    }

#pragma unroll 1
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t row0 = tile * TILE + (int64_t)wave * RW;
        bf16x8 xf[CB][KS1];
        const float *up[CB];
        bool bad[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            int64_t row = row0 + c * 32 + col;
            row = row < M ? row : M - 1;  // rows past the end read the last pair and are not stored
            int32_t v = pair_id[row], q = pair_q[row];
            bad[c] = ((uint64_t)(int64_t)v >= (uint64_t)N) | ((uint32_t)q >= (uint32_t)Q);
            if (bad[c]) v = 0, q = 0;
            const bf16x8 *src = (const bf16x8 *)(emb + (size_t)v * D) + g;
#pragma unroll
            for (int s = 0; s < KS1; ++s) xf[c][s] = src[2 * s];
            up[c] = upre + (size_t)q * H1 + 4 * g;
        }
        static_assert(CB >= 2, "two accumulators must alternate");
        f32x16 acc3[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc3[c][i] = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB1; ++nb) {
            const uint4 *wc = lds + (size_t)nb * BLK_FR * 64;
            f32x16 acc1[CB];
#pragma unroll
            for (int c = 0; c < CB; ++c) {
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4) {
                    f32x4 pv = *(const f32x4 *)(up[c] + nb * 32 + 8 * t4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc1[c][4 * t4 + e] = pv[e];
                }
            }
#pragma unroll
            for (int s = 0; s < KS1; ++s) {
                bf16x8 a = *(const bf16x8 *)(wc + s * 64 + lane);
                static_assert(CB == 2, "pairs 0 and 1 alternate");
                if (s == KS1 - 1) mfma_vgpr_pair<true, F16>(acc1[0], acc1[1], a, xf[0][s], xf[1][s]);
                else mfma_vgpr_pair<false, F16>(acc1[0], acc1[1], a, xf[0][s], xf[1][s]);
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                bf16x8 a = *(const bf16x8 *)(wc + (KS1 + s2) * 64 + lane);
                const bf16x8 h0 = relu_pack<F16>(acc1[0], s2), h1 = relu_pack<F16>(acc1[1], s2);
                if (nb == NB1 - 1 && s2 == 1) mfma_vgpr_pair<true, F16>(acc3[0], acc3[1], a, h0, h1);
                else mfma_vgpr_pair<false, F16>(acc3[0], acc3[1], a, h0, h1);
            }
        }
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float part = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) part = fmaf(hw[i], sigmoid_hw(acc3[c][i] + bh[i]), part);
            float other = __shfl_xor(part, 32);
            int64_t row = row0 + c * 32 + col;
            if (g == 0 && row < M) scores[row] = bad[c] ? __uint_as_float(0x7fc00000u) : part + other;
        }
    }
}


bool mfma_supported(const int32_t *dims, int32_t n_layers, int32_t d_user, int32_t dtype) {
    if ((dtype != ANN_BF16 && dtype != ANN_F16) || d_user < 1 || (n_layers != 2 && n_layers != 3)) return false;
    const int D = dims[0] - d_user, H1 = dims[1], J = dims[n_layers];
    if (J < 1 || J > MAX_HEADS) return false;
    if (n_layers == 2) return D == 64 && H1 == 256;
    const int H2 = dims[2];
    return (D == 128 && H1 == 512 && H2 == 256) || (D == 64 && H1 == 256 && H2 == 128);
}

static inline uint16_t w_at(const uint16_t *W, int n_in, int row, int colm) { return W[(size_t)row * n_in + colm]; }

static int upload_fragments(ann_mlp *m, const std::vector<uint16_t> &buf, hipStream_t stream) {
    m->frag_bytes = (int64_t)buf.size() * 2;
    ANN_HIP_TRY(hipMalloc(&m->frag_dev, (size_t)m->frag_bytes));
    ANN_HIP_TRY(hipMemcpyAsync(m->frag_dev, buf.data(), (size_t)m->frag_bytes, hipMemcpyHostToDevice, stream));
    ANN_HIP_TRY(hipStreamSynchronize(stream));  // buf is freed by the caller
    return ANN_OK;
}

static int build_fragments_one_hidden(ann_mlp *m, const void *const *W_host, hipStream_t stream) {
    const int D = m->d_item, H1 = m->dims[1], J = m->J, du = m->d_user;
    const int KS1 = D / 16, NB1 = H1 / 32, BLK_FR = KS1 + 2;
    std::vector<uint16_t> buf((size_t)NB1 * BLK_FR * 512, 0);
    const uint16_t *W1 = (const uint16_t *)W_host[0], *Wh = (const uint16_t *)W_host[1];
    for (int nb = 0; nb < NB1; ++nb) {
        uint16_t *blk = buf.data() + (size_t)nb * BLK_FR * 512;
        for (int s = 0; s < KS1; ++s)
            for (int l = 0; l < 64; ++l)
                for (int j = 0; j < 8; ++j)
                    blk[(size_t)s * 512 + l * 8 + j] = W1[(size_t)(nb * 32 + (l & 31)) * (du + D) + du + 16 * s + 8 * (l >> 5) + j];
        for (int s2 = 0; s2 < 2; ++s2)
            for (int l = 0; l < 64; ++l)
                for (int j = 0; j < 8; ++j)
                    if ((l & 31) < J)
                        blk[(size_t)(KS1 + s2) * 512 + l * 8 + j] =
                            Wh[(size_t)(l & 31) * H1 + nb * 32 + 16 * s2 + 8 * (j / 4) + 4 * (l >> 5) + j % 4];
    }
    return upload_fragments(m, buf, stream);
}

int build_mfma_fragments(ann_mlp *m, const void *const *W_host, hipStream_t stream) {
    if (m->n_layers == 2) return build_fragments_one_hidden(m, W_host, stream);
    if (mfma_stream_supported(m->d_item, m->dims[1], m->dims[2])) return build_stream_fragments(m, W_host, stream);
    const int D = m->d_item, H1 = m->dims[1], H2 = m->dims[2], J = m->J, du = m->d_user;
    const int KS1 = D / 16, NB1 = H1 / 32, NB2 = H2 / 32;
    const int CHUNK_FR = KS1 + 2 * NB2;
    const size_t n_frag = (size_t)NB1 * CHUNK_FR + 2 * NB2;
    std::vector<uint16_t> buf(n_frag * 512, 0);
    const uint16_t *W1 = (const uint16_t *)W_host[0], *W2 = (const uint16_t *)W_host[1],
                   *W3 = (const uint16_t *)W_host[2];
    for (int nb = 0; nb < NB1; ++nb) {
        uint16_t *chunk = buf.data() + (size_t)nb * CHUNK_FR * 512;
        for (int s = 0; s < KS1; ++s)
            for (int l = 0; l < 64; ++l)
                for (int j = 0; j < 8; ++j)
                    chunk[(size_t)s * 512 + l * 8 + j] =
                        w_at(W1, du + D, nb * 32 + (l & 31), du + 16 * s + 8 * (l >> 5) + j);
        for (int n2 = 0; n2 < NB2; ++n2)
            for (int s2 = 0; s2 < 2; ++s2)
                for (int l = 0; l < 64; ++l)
                    for (int j = 0; j < 8; ++j)
                        chunk[(size_t)(KS1 + 2 * n2 + s2) * 512 + l * 8 + j] =
                            w_at(W2, H1, n2 * 32 + (l & 31), nb * 32 + 16 * s2 + 8 * (j / 4) + 4 * (l >> 5) + j % 4);
    }
    uint16_t *head = buf.data() + (size_t)NB1 * CHUNK_FR * 512;
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
    ANN_HIP_TRY(hipStreamSynchronize(stream));  // buf is freed on return
    return ANN_OK;
}

int launch_user_pre(const ann_mlp *m, const void *queries, int32_t Q, float *upre, hipStream_t stream) {
    if (Q <= 0) return ANN_OK;
    auto fn = m->dtype == ANN_F16 ? user_pre_kernel<true> : user_pre_kernel<false>;
    hipLaunchKernelGGL(fn, dim3(Q), dim3(256), (size_t)m->d_user * sizeof(float), stream,
                       (const uint16_t *)m->W_dev, m->dims[0], m->d_user, m->dims[1], m->b_dev,
                       (const uint16_t *)queries, Q, upre, m->dtype == ANN_F8 ? 4.f : 1.f);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

template <int D, int H1, int H2, int CB, bool RESIDENT, int WAVES, bool F16>
static int launch_one(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                      const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                      hipStream_t stream) {
    constexpr int KS1 = D / 16, NB1 = H1 / 32, NB2 = H2 / 32;
    constexpr int CHUNK_U4 = (KS1 + 2 * NB2) * 64;
    constexpr int NBUF = RESIDENT ? NB1 : 2;
    constexpr size_t smem = ((size_t)NBUF * CHUNK_U4 + 2 * NB2 * 64) * 16;
    constexpr int TILE = 32 * CB * WAVES;
    static_assert(smem <= 160 * 1024, "LDS budget");
    auto fn = mlp_mfma2_kernel<D, H1, H2, CB, RESIDENT, WAVES, F16>;
    static std::atomic<uint32_t> raised;
    if (int rc = raise_lds_limit((const void *)fn, smem, m->device, raised); rc != ANN_OK) return rc;
    int64_t tiles = (M_max + TILE - 1) / TILE;
    int grid = (int)(tiles < 256 ? tiles : 256);
    const float *b2 = m->b_dev + m->b_off[1], *b3 = m->b_dev + m->b_off[2];
    hipLaunchKernelGGL(fn, dim3(grid), dim3(64 * WAVES), smem, stream, (const uint16_t *)g->emb, g->N, upre,
                       (const uint4 *)m->frag_dev, b2, b3, m->head_w_dev, m->J, pair_q, pair_id, M_dev, M_max, Q,
                       scores);
    ANN_HIP_TRY(hipGetLastError());
    return ANN_OK;
}

int launch_mlp_mfma(const ann_graph *g, const ann_mlp *m, const float *upre, const int32_t *pair_q,
                    const int32_t *pair_id, const int32_t *M_dev, int64_t M_max, int32_t Q, float *scores,
                    int32_t tile_rows, hipStream_t stream) {
    (void)tile_rows;
    if (M_max <= 0) return ANN_OK;
    if (m->dtype == ANN_F8) return launch_mlp_mfma_f8(g, m, upre, pair_q, pair_id, M_dev, M_max, Q, scores, stream);
    const int D = m->d_item, H1 = m->dims[1], H2 = m->dims[2];
    if (m->n_layers == 2 && D == 64 && H1 == 256) {
        constexpr int CB = 2, TILE = 32 * CB * MF_WAVES;
        constexpr size_t smem = (size_t)(256 / 32) * (64 / 16 + 2) * 64 * 16;  // 48 KB: three workgroups per CU
        const bool f16 = m->dtype == ANN_F16;
        auto fn = f16 ? mlp_mfma1_kernel<64, 256, CB, true> : mlp_mfma1_kernel<64, 256, CB, false>;
        static std::atomic<uint32_t> raised[2];
        if (int rc = raise_lds_limit((const void *)fn, smem, m->device, raised[f16 ? 1 : 0]); rc != ANN_OK) return rc;
        int64_t tiles = (M_max + TILE - 1) / TILE;
        int grid = (int)(tiles < 3 * 256 ? tiles : 3 * 256);
        hipLaunchKernelGGL(fn, dim3(grid), dim3(MF_BLOCK), smem, stream, (const uint16_t *)g->emb, g->N, upre,
                           (const uint4 *)m->frag_dev, m->b_dev + m->b_off[1], m->head_w_dev, m->J, pair_q, pair_id,
                           M_dev, M_max, Q, scores);
        ANN_HIP_TRY(hipGetLastError());
        return ANN_OK;
    }
    if (mfma_stream_supported(D, H1, H2))
        return launch_mlp_mfma_stream(g, m, upre, pair_q, pair_id, M_dev, M_max, Q, scores, stream);
    if (D == 64 && H1 == 256 && H2 == 128)
        return m->dtype == ANN_F16
                   ? launch_one<64, 256, 128, 2, true, 8, true>(g, m, upre, pair_q, pair_id, M_dev, M_max, Q, scores, stream)
                   : launch_one<64, 256, 128, 2, true, 8, false>(g, m, upre, pair_q, pair_id, M_dev, M_max, Q, scores, stream);
    set_error("no MFMA kernel for item width %d, hidden %d, %d", D, H1, H2);
    return ANN_ENOTIMPL;
}

}  // namespace gmpgr
