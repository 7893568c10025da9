// S2 / S4: fully connected layers (Bottom-FC, Predict-FC; Table I) on the
// bf16 matrix cores, with the element-wise tail fused in (Sec. IV-A): bias,
// ReLU and the narrowing to bf16 happen in the epilogue, and the first layer
// narrows its fp32 input while staging it.
//
//   C[m][n] = act( sum_k A[m][k] * W[n][k] + bias[n] )
//
// Both operands are K-contiguous, which is what v_mfma_f32_32x32x16_bf16 wants:
// lane l feeds 8 consecutive k of row (l % 32), k-offset 8 * (l / 32).  The
// weight tile is the first MFMA operand and the activation tile the second, so
// that each lane ends up with 4 consecutive output features of one sample and
// can store them as one 8-byte (bf16) or 16-byte (fp32) word.
//
// A block of 4 waves computes a BM x BN tile; tiles of A and W go through one
// LDS buffer each, the next tile's global loads being in flight while the
// current one is multiplied.
//
// Several stacks of equal shape (the N task towers of Table I's MT-WnD row)
// run as one launch: the tile list is the tiles of stack 0, then stack 1, ...;
// a block picks its stack's weights from a table passed by value and offsets
// its activation pointers by the stack's column block.
#include "rec_internal.h"

namespace rec {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;            // k extent of one staged tile
constexpr int LDS_LD = BK + 8;    // row stride in LDS (elements); 144 B keeps 16-byte reads conflict-free
constexpr int FC_THREADS = 256;

// 8 consecutive k of one activation row as fetched: raw fp32 (narrowed only when
// it is stored to LDS, so that the load stays in flight) or bf16.
template <bool A_F32>
struct AChunk;
template <>
struct AChunk<true> {
    f32x4 lo, hi;
    __device__ inline bf16x8 narrow() const
    {
        bf16x8 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[i] = (__bf16)lo[i];
            o[i + 4] = (__bf16)hi[i];
        }
        return o;
    }
};
template <>
struct AChunk<false> {
    bf16x8 v;
    __device__ inline bf16x8 narrow() const { return v; }
};

__device__ inline void load_a_chunk(AChunk<true> &c, const void *A, long long row, int lda, int k,
                                    int K, bool vec_ok)
{
    const float *p = static_cast<const float *>(A) + row * lda + k;
    if (vec_ok && k + 8 <= K) {
        c.lo = *reinterpret_cast<const f32x4 *>(p);
        c.hi = *reinterpret_cast<const f32x4 *>(p + 4);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c.lo[i] = (k + i < K) ? p[i] : 0.0f;
            c.hi[i] = (k + 4 + i < K) ? p[4 + i] : 0.0f;
        }
    }
}

__device__ inline void load_a_chunk(AChunk<false> &c, const void *A, long long row, int lda, int k,
                                    int, bool)
{
    // bf16 activations live in buffers whose columns up to lda are valid (zero padded).
    c.v = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(A) + row * lda + k);
}

// BM x BN block tile, 4 waves laid out WAVES_M x (4 / WAVES_M), P k-tiles of
// global loads in flight.  FUSE_DOT (needs BN == Npad): instead of storing C,
// the epilogue contracts act(C) with a weight vector - the one-output last
// layer - and writes one fp32 logit per row.
//
// The small tiles with two k-tiles in flight, and the 128 x 128 tile with one,
// are the forms that run beside a pooling launch (FcProblem::corun): they are
// held to 128 registers, the part of a SIMD's register file that eight pooling
// waves leave free, so that a wave of theirs needs nothing but a wave slot.
template <int BM, int BN, int WAVES_M, int P, bool A_F32, bool OUT_F32, bool FUSE_DOT>
__global__ __launch_bounds__(FC_THREADS, ((P == 2 && BM * BN <= 4096) || P == 1) ? 4 : 1) void fc_kernel(const void *__restrict__ A0, int lda,
                                                        long long a_stride, int M, int K, int Kpad,
                                                        const FcGroups groups, int relu,
                                                        void *__restrict__ C0, int ldc,
                                                        long long c_stride, int vec_ok,
                                                        float *__restrict__ dot_out, int dot_ld,
                                                        int grid_n, int tiles_per_group)
{
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // per-wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // 32 x 32 MFMA tiles per wave
    constexpr int A_LOADS = BM / 32, W_LOADS = BN / 32;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be whole MFMA tiles");

    __shared__ __attribute__((aligned(16))) __bf16 sA[BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) __bf16 sW[BN * LDS_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    // Blocks are dealt to the 8 XCDs round-robin.  The 1-D grid is re-ordered so
    // that XCD x owns the x-th eighth of the tile list (n fastest): the tiles
    // that share a slab of activations then share an L2 and the slab comes from
    // HBM once instead of once per XCD.
    int v = blockIdx.x;
    if ((gridDim.x & 7) == 0) v = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int grp = v / tiles_per_group;
    v -= grp * tiles_per_group;
    const int bm = v / grid_n, bn = v - bm * grid_n;
    const int m0 = bm * BM, n0 = bn * BN;
    const void *A = static_cast<const char *>(A0) + grp * a_stride * (A_F32 ? 4 : 2);
    void *C = static_cast<char *>(C0) + grp * c_stride * (OUT_F32 ? 4 : 2);
    const __bf16 *__restrict__ W = static_cast<const __bf16 *>(groups.W[grp]);
    const float *__restrict__ bias = groups.bias[grp];
    const float *__restrict__ dot_w = groups.dot_w[grp];
    const float *__restrict__ dot_bias = groups.dot_bias[grp];

    // Staging role: 8 threads cover the 64 k of one row, 32 rows per pass.
    const int ld_row = tid >> 3, ld_chunk = tid & 7;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    AChunk<A_F32> ra[P][A_LOADS];
    bf16x8 rw[P][W_LOADS];
    const int nk = Kpad / BK;

#define REC_FC_FETCH(kt, slot)                                                              \
    do {                                                                                    \
        const int k_ = (kt) * BK + ld_chunk * 8;                                            \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i) {                               \
            int row_ = m0 + ld_row + 32 * i;                                                \
            row_ = row_ < M ? row_ : M - 1; /* rows past M are computed and dropped */      \
            load_a_chunk(ra[slot][i], A, row_, lda, k_, K, vec_ok);                         \
        }                                                                                   \
        _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i) {                               \
            const long long row_ = n0 + ld_row + 32 * i;                                    \
            rw[slot][i] = *reinterpret_cast<const bf16x8 *>(W + row_ * Kpad + k_);          \
        }                                                                                   \
    } while (0)

    // One k-tile out of register slot u: into LDS, multiply; the slot is refilled
    // with tile kt + P.  Fetches past the last tile repeat it instead of being
    // skipped: with a branch around them the compiler can no longer count the
    // loads in flight and waits for all of them before every LDS write.
#define REC_FC_TILE(kt, u)                                                                  \
    do {                                                                                    \
        __syncthreads();                                                                    \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                 \
            *reinterpret_cast<bf16x8 *>(&sA[(ld_row + 32 * i) * LDS_LD + ld_chunk * 8]) = ra[u][i].narrow(); \
        _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i)                                 \
            *reinterpret_cast<bf16x8 *>(&sW[(ld_row + 32 * i) * LDS_LD + ld_chunk * 8]) = rw[u][i]; \
        __syncthreads();                                                                    \
        REC_FC_FETCH(min((kt) + P, nk - 1), u);                                             \
        /* all operand fragments of the k-tile are requested before the first product: */   \
        /* read-wait-multiply per 16 k would expose the LDS latency four times */          \
        bf16x8 fw[BK / 16][TN], fa[BK / 16][TM];                                            \
        _Pragma("unroll") for (int kk = 0; kk < BK / 16; ++kk) {                            \
            const int kofs = kk * 16 + (lane >> 5) * 8;                                     \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                  \
                fw[kk][i] = *reinterpret_cast<const bf16x8 *>(&sW[(wn * WN + i * 32 + (lane & 31)) * LDS_LD + kofs]); \
            _Pragma("unroll") for (int j = 0; j < TM; ++j)                                  \
                fa[kk][j] = *reinterpret_cast<const bf16x8 *>(&sA[(wm * WM + j * 32 + (lane & 31)) * LDS_LD + kofs]); \
        }                                                                                   \
        _Pragma("unroll") for (int kk = 0; kk < BK / 16; ++kk)                              \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                  \
                _Pragma("unroll") for (int j = 0; j < TM; ++j)                              \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[kk][i], fa[kk][j], acc[i][j], 0, 0, 0); \
    } while (0)

#pragma unroll
    for (int p = 0; p < P; ++p) REC_FC_FETCH(min(p, nk - 1), p);

    int kt0 = 0;
    for (; kt0 + P <= nk; kt0 += P) {
#pragma unroll
        for (int u = 0; u < P; ++u) REC_FC_TILE(kt0 + u, u);
    }
#pragma unroll
    for (int u = 0; u < P - 1; ++u)
        if (kt0 + u < nk) REC_FC_TILE(kt0 + u, u);
#undef REC_FC_TILE
#undef REC_FC_FETCH

    // acc[i][j][r]: feature n = 8 * (r / 4) + 4 * (lane / 32) + r % 4, sample m = lane % 32.
    float dot[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) dot[j] = 0.0f;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m0 + wm * WM + j * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + i * 32 + 8 * q + 4 * (lane >> 5);
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + n);
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float x = acc[i][j][4 * q + r] + bv[r];
                    v[r] = (relu && x < 0.0f) ? 0.0f : x;
                }
                if (FUSE_DOT) {
                    const f32x4 wv = *reinterpret_cast<const f32x4 *>(dot_w + n);
#pragma unroll
                    for (int r = 0; r < 4; ++r) dot[j] += v[r] * wv[r];
                } else if (m < M) {
                    if (OUT_F32) {
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(C) + (long long)m * ldc + n) = v;
                    } else {
                        bf16x4 o;
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] = (__bf16)v[r];
                        *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(C) + (long long)m * ldc + n) = o;
                    }
                }
            }
        }
    }
    if (FUSE_DOT) {
        // Lanes l and l ^ 32 hold the two halves of a sample's features in this
        // wave; the WAVES_N waves of a row of waves hold the rest.
        float *red = reinterpret_cast<float *>(sA);  // [WAVES_N][BM], the tiles are done with
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const float d = dot[j] + __shfl_xor(dot[j], 32, 64);
            if (lane < 32) red[wn * BM + wm * WM + j * 32 + lane] = d;
        }
        __syncthreads();
        if (tid < BM && m0 + tid < M) {
            float d = dot_bias[0];
#pragma unroll
            for (int w = 0; w < WAVES_N; ++w) d += red[w * BM + tid];
            dot_out[(long long)(m0 + tid) * dot_ld + grp] = d;
        }
    }
}

template <int BM, int BN, int WAVES_M, int P>
hipError_t launch_tile(const FcProblem &a, hipStream_t s)
{
    const int grid_n = a.Npad / BN;
    const int tiles = grid_n * ((a.M + BM - 1) / BM);
    const dim3 grid(tiles * a.groups), block(FC_THREADS);
    // 16-byte loads of fp32 rows need lda and the stack stride % 4 == 0 and an aligned base.
    const int vec_ok = a.a_f32 && (a.lda % 4 == 0) && (a.a_stride % 4 == 0) &&
                       (reinterpret_cast<uintptr_t>(a.A) % 16 == 0);
    const int r = a.relu ? 1 : 0;
#define REC_FC_LAUNCH(AF, OF, FD)                                                                  \
    hipLaunchKernelGGL((fc_kernel<BM, BN, WAVES_M, P, AF, OF, FD>), grid, block, 0, s, a.A, a.lda, \
                       a.a_stride, a.M, a.K, a.Kpad, a.g, r, a.C, a.ldc, a.c_stride, vec_ok,       \
                       a.dot_out, a.dot_ld, grid_n, tiles)
    if (a.dot_out) {
        if (a.a_f32) REC_FC_LAUNCH(true, false, true);
        else REC_FC_LAUNCH(false, false, true);
    } else if (a.a_f32 && a.out_f32) REC_FC_LAUNCH(true, true, false);
    else if (a.a_f32) REC_FC_LAUNCH(true, false, false);
    else if (a.out_f32) REC_FC_LAUNCH(false, true, false);
    else REC_FC_LAUNCH(false, false, false);
#undef REC_FC_LAUNCH
    return hipGetLastError();
}

// Last Predict-FC layer (one output per sample): a plain fp32 dot product with
// fp32 weights; 8 lanes share a row.  The input is the previous layer's fp32
// output, or the bf16 interaction output when the stack has a single layer.
template <bool A_F32>
__global__ __launch_bounds__(256) void rowdot_kernel(const void *__restrict__ A0, int lda,
                                                     long long a_stride, int M, int Kpad,
                                                     const FcGroups groups,
                                                     float *__restrict__ logits, int ld)
{
    const int grp = blockIdx.y;
    const void *A = static_cast<const char *>(A0) + grp * a_stride * (A_F32 ? 4 : 2);
    const float *__restrict__ w = groups.dot_w[grp];
    const float *__restrict__ bias = groups.dot_bias[grp];
    const int sub = threadIdx.x & 7;
    const long long m = (long long)blockIdx.x * 32 + (threadIdx.x >> 3);
    const long long row = m < M ? m : M - 1;
    float acc = 0.0f;
    for (int k = sub * 8; k < Kpad; k += 64) {
        float a[8];
        if (A_F32) {
            const float *p = static_cast<const float *>(A) + row * lda + k;
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(p);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = lo[i]; a[i + 4] = hi[i]; }
        } else {
            const bf16x8 v = *reinterpret_cast<const bf16x8 *>(static_cast<const __bf16 *>(A) + row * lda + k);
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = (float)v[i];
        }
        const f32x4 w0 = *reinterpret_cast<const f32x4 *>(w + k);
        const f32x4 w1 = *reinterpret_cast<const f32x4 *>(w + k + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc += a[i] * w0[i];
            acc += a[i + 4] * w1[i];
        }
    }
    acc += __shfl_xor(acc, 1, 64);
    acc += __shfl_xor(acc, 2, 64);
    acc += __shfl_xor(acc, 4, 64);
    if (sub == 0 && m < M) logits[m * ld + grp] = acc + bias[0];
}

// One-output layer: fp32 weights [Kpad], zero padded, and its bias.
__global__ __launch_bounds__(256) void pack_dot_kernel(const float *__restrict__ W,
                                                       const float *__restrict__ b, int K, int Kpad,
                                                       float *__restrict__ Wp, float *__restrict__ bp)
{
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < Kpad; k += gridDim.x * blockDim.x)
        Wp[k] = k < K ? W[k] : 0.0f;
    if (blockIdx.x == 0 && threadIdx.x == 0) bp[0] = b[0];
}

__global__ __launch_bounds__(256) void pack_fc_kernel(const float *__restrict__ W,
                                                      const float *__restrict__ b, int N, int K,
                                                      int Npad, int Kpad, __bf16 *__restrict__ Wp,
                                                      float *__restrict__ bp)
{
    const long long total = (long long)Npad * Kpad;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const int n = (int)(i / Kpad), k = (int)(i % Kpad);
        Wp[i] = (__bf16)((n < N && k < K) ? W[(long long)n * K + k] : 0.0f);
        if (k == 0) bp[n] = n < N ? b[n] : 0.0f;
    }
}

}  // namespace

bool fc_can_fuse_dot(int Npad) { return Npad == 64 || Npad == 128 || Npad == 256; }

hipError_t launch_fc(const FcProblem &a, hipStream_t s)
{
    const int M = a.M, Npad = a.Npad;
    if (M <= 0) return hipSuccess;
    if (a.Kpad % BK != 0 || Npad % 64 != 0 || a.groups < 1 || a.groups > MAX_GROUPS)
        return hipErrorInvalidValue;
    // corun: the launch shares the device with a pooling launch, whose waves
    // (48 registers each, eight per SIMD) hold every wave slot; a wave of this
    // kernel gets in when one of them retires, and then finds 512 - 7 * 48 = 176
    // registers free.  With four k-tiles in flight these kernels need 184-214 and
    // would wait for a second slot on the same SIMD, which pooling refills first
    // (measured: 123 instead of 14 us); with three they need 130-150.
    if (a.dot_out) {
        // The block must own whole rows.
        if (Npad == 256) return launch_tile<64, 256, 1, 2>(a, s);
        if (Npad == 128) return a.corun ? launch_tile<32, 128, 1, 2>(a, s) : launch_tile<32, 128, 1, 4>(a, s);
        if (Npad == 64) return a.corun ? launch_tile<64, 64, 2, 2>(a, s) : launch_tile<64, 64, 2, 4>(a, s);
        return hipErrorInvalidValue;
    }
    if (a.num_cus > 0 && fc_big_applies(a, a.num_cus)) return launch_fc_big(a, a.num_cus, s);
    // Large tiles only where they still give every compute unit a block.
    const long long big_blocks = (long long)a.groups * (Npad / 128) * ((M + 127) / 128);
    // Beside pooling what a launch costs is the wave slots it holds and the lines
    // it pulls through the L1s, not its own duration: few large tiles, even if
    // they leave compute units without a block (rmc2's first Predict-FC layer:
    // 128 blocks instead of 512, 3 us less per pipelined step).
    // (bf16 input only: with fp32 staging registers the tile does not fit 128 registers.)
    if (a.corun && !a.a_f32 && Npad % 128 == 0 && big_blocks >= 64) return launch_tile<128, 128, 2, 1>(a, s);
    if (Npad % 128 == 0 && big_blocks >= 256) return launch_tile<128, 128, 2, 2>(a, s);
    const long long mid_blocks = (long long)a.groups * (Npad / 64) * ((M + 63) / 64);
    if (Npad % 128 == 0 && mid_blocks < 256)
        return a.corun ? launch_tile<32, 128, 1, 2>(a, s) : launch_tile<32, 128, 1, 4>(a, s);
    return a.corun ? launch_tile<64, 64, 2, 2>(a, s) : launch_tile<64, 64, 2, 4>(a, s);
}

hipError_t launch_rowdot(const void *A, bool a_f32, int lda, long long a_stride, int M, int Kpad,
                         const FcGroups &groups, int n_groups, float *logits, int ld, hipStream_t s)
{
    if (M <= 0) return hipSuccess;
    if (n_groups < 1 || n_groups > MAX_GROUPS) return hipErrorInvalidValue;
    const dim3 grid((M + 31) / 32, n_groups), block(256);
    if (a_f32)
        hipLaunchKernelGGL(rowdot_kernel<true>, grid, block, 0, s, A, lda, a_stride, M, Kpad, groups,
                           logits, ld);
    else
        hipLaunchKernelGGL(rowdot_kernel<false>, grid, block, 0, s, A, lda, a_stride, M, Kpad, groups,
                           logits, ld);
    return hipGetLastError();
}

hipError_t launch_pack_dot(const float *W, const float *b, int K, int Kpad, float *W_packed,
                           float *bias_packed, hipStream_t s)
{
    hipLaunchKernelGGL(pack_dot_kernel, dim3((Kpad + 255) / 256), dim3(256), 0, s, W, b, K, Kpad,
                       W_packed, bias_packed);
    return hipGetLastError();
}

hipError_t launch_pack_fc(const float *W, const float *b, int N, int K, int Npad, int Kpad,
                          void *W_packed, float *bias_packed, hipStream_t s)
{
    const long long total = (long long)Npad * Kpad;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(pack_fc_kernel, dim3(blocks), dim3(256), 0, s, W, b, N, K, Npad, Kpad,
                       static_cast<__bf16 *>(W_packed), bias_packed);
    return hipGetLastError();
}

}  // namespace rec
