// S2 / S4 as one kernel per stack: a run of fully connected layers whose
// activations never leave the compute unit (the FC stacks of Sec. II-A and
// Table I are narrow: a few hundred to a thousand units per layer).
//
// A block owns CH_ROWS samples.  Their input row is brought into LDS as bf16
// once; every layer then reads its input from one LDS buffer and leaves its
// output (bias, ReLU, narrowed to bf16) in the other, so between the first
// read and the last write only weights move.  The weights come straight from
// global memory (they stay in L2 across blocks) into the MFMA operand
// registers: they are stored fragment by fragment, 64 lanes x 16 bytes each, so
// every load of a wave is one contiguous KiB.  The product is computed
// transposed, D[n][m] = sum_k W[n][k] X[m][k] on v_mfma_f32_32x32x16_bf16: a
// lane then holds four consecutive outputs of one sample and stores them with
// one instruction.
//
// Wave w of the eight takes the 32-column chunks w, w + 8, ... of a layer, two
// at a time, each weight fragment requested CH_PF k-steps before it is used.
//
// The run ends in fp32 or bf16 rows in global memory, or - the Predict-FC's
// one-output layer - in a dot product of the last activations (fp32, before
// any narrowing) with that layer's weights, summed in a fixed order.
#include "rec_internal.h"

namespace rec {

namespace {

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

template <bool A_F32>
__global__ __launch_bounds__(CH_THREADS) void mlp_chain_kernel(const ChainProblem a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int ld = a.ld_lds;
    // Two activation buffers of CH_ROWS rows; one base pointer and integer offsets,
    // so that every access is compiled as an LDS access.
    __bf16 *lds = reinterpret_cast<__bf16 *>(smem);
    float *red = reinterpret_cast<float *>(smem + 2 * (size_t)CH_ROWS * ld * sizeof(__bf16));  // [CH_WAVES][CH_ROWS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.y, row0 = blockIdx.x * CH_ROWS;
    const int m = lane & 31, half = lane >> 5;  // sample of this lane, and which 8 of a step's 16 k

    // All blocks walk the weights in the same order at the same time, so a line
    // missing in the L2 is missing for every block that wants it.  Before anything
    // else the blocks that share an L2 (every eighth block, the XCDs taking blocks
    // round-robin) each touch their slice of every layer's weights: one load per
    // 128-byte line, all in flight together while the input rows are staged.
    unsigned touched = 0;
    {
        const int share = min(16, max(1, (int)gridDim.x >> 3));
        const int mine = ((int)blockIdx.x >> 3) % share;
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

// fp32 [N][K] -> bf16 fragments: element e of lane l of fragment (nc, ks) is
// W[32 nc + l % 32][16 ks + 8 (l / 32) + e], zero outside the matrix.
__global__ __launch_bounds__(256) void pack_chain_kernel(const float *__restrict__ W, int N, int K, int Npad,
                                                         int Kpad, __bf16 *__restrict__ Wp)
{
    const long long total = (long long)Npad * Kpad;
    const int KS = Kpad / 16;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long frag = i >> 9;
        const int within = (int)(i & 511), lane = within >> 3, e = within & 7;
        const int nc = (int)(frag / KS), ks = (int)(frag % KS);
        const int n = nc * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8 + e;
        Wp[i] = (__bf16)((n < N && k < K) ? W[(long long)n * K + k] : 0.0f);
    }
}

size_t chain_lds_bytes(int ld) { return 2 * (size_t)CH_ROWS * ld * sizeof(__bf16) + sizeof(float) * CH_WAVES * CH_ROWS; }

}  // namespace

bool chain_layer_fits(int Kpad, int Npad) { return Kpad <= CHAIN_MAX_WIDTH && Npad <= CHAIN_MAX_WIDTH; }

hipError_t chain_prepare()
{
    const int most = (int)chain_lds_bytes(CHAIN_MAX_WIDTH + CH_LDS_PAD);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(mlp_chain_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, most);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(mlp_chain_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, most);
}

hipError_t launch_mlp_chain(const ChainProblem &p, hipStream_t s)
{
    if (p.M <= 0) return hipSuccess;
    if (p.n_layers < 1 || p.n_layers > CHAIN_MAX_LAYERS || p.groups < 1 || p.groups > MAX_GROUPS)
        return hipErrorInvalidValue;
    int widest = p.Kpad[0];
    for (int L = 0; L < p.n_layers; ++L) {
        if (p.Kpad[L] % PAD != 0 || p.Npad[L] % PAD != 0 || !chain_layer_fits(p.Kpad[L], p.Npad[L]))
            return hipErrorInvalidValue;
        if (L > 0 && p.Kpad[L] != p.Npad[L - 1]) return hipErrorInvalidValue;
        widest = widest > p.Npad[L] ? widest : p.Npad[L];
    }
    if (p.K > p.Kpad[0]) return hipErrorInvalidValue;
    ChainProblem a = p;
    a.ld_lds = widest + CH_LDS_PAD;
    // Wide loads of the input rows need aligned rows that end on a vector boundary.
    const int vec = p.a_f32 ? 4 : 8;
    const int esz = p.a_f32 ? 4 : 2;
    a.a_vec = reinterpret_cast<uintptr_t>(p.A) % 16 == 0 && p.lda % vec == 0 && p.a_stride % vec == 0 &&
              (p.a_f32 ? p.K % vec == 0 : true) && (long long)p.lda * esz % 16 == 0;
    if (p.out_mode != CHAIN_OUT_DOT) {
        const int ov = 4;
        if (reinterpret_cast<uintptr_t>(p.C) % 16 != 0 || p.ldc % ov != 0 || p.c_stride % ov != 0)
            return hipErrorInvalidValue;
    }
    const dim3 grid((p.M + CH_ROWS - 1) / CH_ROWS, p.groups), block(CH_THREADS);
    const size_t lds = chain_lds_bytes(a.ld_lds);
    if (p.a_f32)
        hipLaunchKernelGGL(mlp_chain_kernel<true>, grid, block, lds, s, a);
    else
        hipLaunchKernelGGL(mlp_chain_kernel<false>, grid, block, lds, s, a);
    return hipGetLastError();
}

hipError_t launch_pack_chain(const float *W, int N, int K, int Npad, int Kpad, void *W_packed, hipStream_t s)
{
    const long long total = (long long)Npad * Kpad;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(pack_chain_kernel, dim3(blocks), dim3(256), 0, s, W, N, K, Npad, Kpad,
                       static_cast<__bf16 *>(W_packed));
    return hipGetLastError();
}

}  // namespace rec
