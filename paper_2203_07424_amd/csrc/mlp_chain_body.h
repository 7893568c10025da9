// Body of the kernel that runs a stack of fully connected layers on chip
// (csrc/mlp_chain.hip has the description), as a device function: the block
// that calls it may be one of that kernel's own, or a spare block of another
// launch that the stack rides along with.
#ifndef REC_MLP_CHAIN_BODY_H
#define REC_MLP_CHAIN_BODY_H
#include "rec_internal.h"

namespace rec {
namespace chain {

constexpr int CH_ROWS = 32;
constexpr int CH_WAVES = 8;
constexpr int CH_THREADS = CH_WAVES * 64;
constexpr int CH_PF = 8;      // k-steps (of 16) a weight fragment is requested ahead
static_assert(CH_PF == 8, "the tail of chunk_product assumes rounds of 8 and widths padded to 64");
constexpr int CH_LDS_PAD = 8; // elements added to an LDS row: consecutive rows start 4 banks apart

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Input rows -> LDS as bf16, zero for rows >= M and columns >= K.
template <bool A_F32>
__device__ inline void stage_input(const ChainProblem &a, int g, int row0, __bf16 *dst, int ld)
{
    const int Kpad = a.Kpad[0];
    const int tid = threadIdx.x;
    if (A_F32) {
        const float *A = static_cast<const float *>(a.A) + (long long)g * a.a_stride;
        if (a.a_vec) {  // four columns per thread
            const int per_row = Kpad / 4;
            for (int i = tid; i < CH_ROWS * per_row; i += CH_THREADS) {
                const int r = i / per_row, k = (i - r * per_row) * 4;
                f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (row0 + r < a.M && k < a.K)  // K is a multiple of 4 here
                    v = *reinterpret_cast<const f32x4 *>(A + (long long)(row0 + r) * a.lda + k);
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                *reinterpret_cast<bf16x4 *>(dst + r * ld + k) = o;
            }
        } else {
            for (int i = tid; i < CH_ROWS * Kpad; i += CH_THREADS) {
                const int r = i / Kpad, k = i - r * Kpad;
                const float v = (row0 + r < a.M && k < a.K) ? A[(long long)(row0 + r) * a.lda + k] : 0.0f;
                dst[r * ld + k] = (__bf16)v;
            }
        }
    } else {
        const __bf16 *A = static_cast<const __bf16 *>(a.A) + (long long)g * a.a_stride;
        if (a.a_vec) {  // eight columns per thread
            const int per_row = Kpad / 8;
            for (int i = tid; i < CH_ROWS * per_row; i += CH_THREADS) {
                const int r = i / per_row, k = (i - r * per_row) * 8;
                bf16x8 v;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.0f;
                if (row0 + r < a.M && k < a.K) {
                    v = *reinterpret_cast<const bf16x8 *>(A + (long long)(row0 + r) * a.lda + k);
                    if (k + 8 > a.K) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (k + e >= a.K) v[e] = (__bf16)0.0f;
                    }
                }
                *reinterpret_cast<bf16x8 *>(dst + r * ld + k) = v;
            }
        } else {
            for (int i = tid; i < CH_ROWS * Kpad; i += CH_THREADS) {
                const int r = i / Kpad, k = i - r * Kpad;
                dst[r * ld + k] = (row0 + r < a.M && k < a.K) ? A[(long long)(row0 + r) * a.lda + k] : (__bf16)0.0f;
            }
        }
    }
}

// acc_c += W_c X^T over all KS k-steps for NCH (1 or 2) chunks of 32 output
// columns.  Straight-line code: every weight fragment is requested CH_PF steps
// before its use, the requests past the end repeat the last fragment instead of
// branching (a branch would make the compiler wait for all loads at every step).
template <int NCH>
__device__ inline void chunk_product(const u32x4 *w0, const u32x4 *w1, const __bf16 *xrow, int KS,
                                     f32x16 &acc0, f32x16 &acc1)
{
    u32x4 q0[CH_PF], q1[CH_PF];
    const int lastk = KS - 1;
#pragma unroll
    for (int p = 0; p < CH_PF; ++p) {
        const int k = min(p, lastk);
        q0[p] = w0[k * 64];
        if (NCH == 2) q1[p] = w1[k * 64];
    }
    int ks = 0;
    for (; ks + CH_PF <= KS; ks += CH_PF) {
#pragma unroll
        for (int p = 0; p < CH_PF; ++p) {
            const bf16x8 x = *reinterpret_cast<const bf16x8 *>(xrow + (ks + p) * 16);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q0[p]), x, acc0, 0, 0, 0);
            if (NCH == 2)
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q1[p]), x, acc1, 0, 0, 0);
            const int k = min(ks + p + CH_PF, lastk);
            q0[p] = w0[k * 64];
            if (NCH == 2) q1[p] = w1[k * 64];
            __builtin_amdgcn_sched_barrier(0);  // keep each request where it is written: CH_PF steps ahead
        }
    }
    if (ks < KS) {  // KS is a multiple of 4: half a round is left, already in q[0..3]
#pragma unroll
        for (int p = 0; p < CH_PF / 2; ++p) {
            const bf16x8 x = *reinterpret_cast<const bf16x8 *>(xrow + (ks + p) * 16);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q0[p]), x, acc0, 0, 0, 0);
            if (NCH == 2)
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q1[p]), x, acc1, 0, 0, 0);
        }
    }
}

// One block's share of the run: samples bx * CH_ROWS ... of stack g, bx out of
// grid_x blocks.  `smem` is chain_lds_bytes(a.ld_lds) of dynamic LDS; all
// CH_THREADS threads of the block take part.
template <bool A_F32>
__device__ inline void mlp_chain_block(const ChainProblem &a, unsigned char *smem, int bx, int g, int grid_x)
{
    const int ld = a.ld_lds;
    // Two activation buffers of CH_ROWS rows; one base pointer and integer offsets,
    // so that every access is compiled as an LDS access.
    __bf16 *lds = reinterpret_cast<__bf16 *>(smem);
    float *red = reinterpret_cast<float *>(smem + 2 * (size_t)CH_ROWS * ld * sizeof(__bf16));  // [CH_WAVES][CH_ROWS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = bx * CH_ROWS;
    const int m = lane & 31, half = lane >> 5;  // sample of this lane, and which 8 of a step's 16 k

    // All blocks walk the weights in the same order at the same time, so a line
    // missing in the L2 is missing for every block that wants it.  Before anything
    // else the blocks that share an L2 (every eighth block, the XCDs taking blocks
    // round-robin) each touch their slice of every layer's weights: one load per
    // 128-byte line, all in flight together while the input rows are staged.
    unsigned touched = 0;
    {
        const int share = min(16, max(1, grid_x >> 3));
        const int mine = (bx >> 3) % share;
        for (int L = 0; L < a.n_layers; ++L) {
            const int lines = a.Kpad[L] * a.Npad[L] / 64;  // bf16: 64 elements per line
            const int per = (lines + share - 1) / share;
            const unsigned *w = static_cast<const unsigned *>(a.W[L][g]);
            for (int i = mine * per + tid; i < min(lines, (mine + 1) * per); i += CH_THREADS)
                touched |= w[(size_t)i * 32];
        }
    }
    stage_input<A_F32>(a, g, row0, lds, ld);
    asm volatile("" ::"v"(touched));  // the loads above are issued, their values unused
    __syncthreads();

    float dot_part = 0.0f;
    int cur = 0;
    for (int L = 0; L < a.n_layers; ++L) {
        const int KS = a.Kpad[L] / 16, NC = a.Npad[L] / 32;
        const bool last = L + 1 == a.n_layers;
        const bool relu = a.relu[L] != 0;
        const u32x4 *W = static_cast<const u32x4 *>(a.W[L][g]);  // fragment (nc, ks) at W[(nc * KS + ks) * 64 + lane]
        const float *bias = a.bias[L][g];
        const __bf16 *xrow = lds + cur * CH_ROWS * ld + m * ld + half * 8;
        __bf16 *yrow = lds + (cur ^ 1) * CH_ROWS * ld + m * ld;

        for (int nc0 = wave; nc0 < NC; nc0 += 2 * CH_WAVES) {
            const int nc1 = nc0 + CH_WAVES;
            const bool two = nc1 < NC;  // wave-uniform
            const u32x4 *w0 = W + (size_t)nc0 * KS * 64 + lane;
            const u32x4 *w1 = W + (size_t)(two ? nc1 : nc0) * KS * 64 + lane;
            f32x16 acc0, acc1;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.0f;
            if (two)
                chunk_product<2>(w0, w1, xrow, KS, acc0, acc1);
            else
                chunk_product<1>(w0, w1, xrow, KS, acc0, acc1);
            // acc[r] is output column n = 32 nc + 8 (r / 4) + 4 half + r % 4 of sample m.
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                if (c == 1 && !two) break;
                const f32x16 &acc = c == 0 ? acc0 : acc1;
                const int nbase = (c == 0 ? nc0 : nc1) * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = nbase + 8 * q;
                    const f32x4 bq = *reinterpret_cast<const f32x4 *>(bias + n);
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = acc[4 * q + e] + bq[e];
                        if (relu) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
                    }
                    if (!last) {
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                        *reinterpret_cast<bf16x4 *>(yrow + n) = o;
                    } else if (a.out_mode == CHAIN_OUT_DOT) {
                        const f32x4 wq = *reinterpret_cast<const f32x4 *>(a.dot_w[g] + n);
#pragma unroll
                        for (int e = 0; e < 4; ++e) dot_part += v[e] * wq[e];
                    } else if (row0 + m < a.M) {
                        const long long at = (long long)(row0 + m) * a.ldc + (long long)g * a.c_stride + n;
                        if (a.out_mode == CHAIN_OUT_F32) {
                            *reinterpret_cast<f32x4 *>(static_cast<float *>(a.C) + at) = v;
                        } else {
                            bf16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                            *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(a.C) + at) = o;
                        }
                    }
                }
            }
        }
        __syncthreads();
        cur ^= 1;
    }

    if (a.out_mode == CHAIN_OUT_DOT) {
        // Per sample: the two half-waves, then the waves in order.
        dot_part += __shfl_xor(dot_part, 32, 64);
        if (lane < 32) red[wave * CH_ROWS + m] = dot_part;
        __syncthreads();
        if (tid < CH_ROWS && row0 + tid < a.M) {
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < CH_WAVES; ++w) sum += red[w * CH_ROWS + tid];
            a.dot_out[(long long)(row0 + tid) * a.dot_ld + g] = sum + a.dot_bias[g][0];
        }
    }
}

inline size_t chain_lds_bytes(int ld) { return 2 * (size_t)CH_ROWS * ld * sizeof(__bf16) + sizeof(float) * CH_WAVES * CH_ROWS; }

}  // namespace chain
}  // namespace rec
#endif
