// S2 / S4 for wide layers on large batches (Table I: the 2560-wide Bottom-FC of
// DLRM-RMC3, the N towers of 1024-512-256 of MT-WnD): the same
// C = act(A W^T + b)  as fc_kernel, with block tiles of 256 x 256, 256 x 128 or
// 128 x 128 and 8 waves per block.
//
// A BM x BN tile moves (BM + BN) * 2 bytes per k for 2 * BM * BN flops, so large
// tiles ask least of the caches; the L2 can feed a compute unit about 49 bytes
// per clock (measured with a read-only probe on an L2-resident footprint) and a
// 256 x 256 tile needs 32 at full MFMA rate.  The tile pairs are double
// buffered in LDS (one barrier per k-tile; 256 x 256 x 64: 2 x 72 KB of the
// 160 KB), so one block owns a compute unit, two waves per SIMD.
//
// Per k-tile: tile kt is multiplied out of one LDS buffer while the registers
// holding tile kt+1 (fetched one iteration earlier) go to the other buffer and
// are refilled with tile kt+2, a quarter of that staging work per 16-wide step
// of matrix instructions.  Measured and not kept: 4 waves with 128 x 128 wave
// tiles (accumulators in AGPRs), 16 waves, and global loads written straight
// into LDS (swizzled rows, no staging registers) - each within 5 % of this.
#include "rec_internal.h"

namespace rec {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;          // k extent of one staged tile
constexpr int LDS_LD = BK + 8;  // 144-byte row stride: 16-byte reads of 16 consecutive rows hit 16 different bank groups

template <int BM, int BN>
constexpr size_t big_lds_bytes() { return 2 * (size_t)(BM + BN) * LDS_LD * sizeof(__bf16); }

// 8 consecutive k of one activation row as fetched: bf16, or raw fp32 (the model's
// dense input) that is narrowed only when it is written to LDS.
template <bool A_F32>
struct AReg;
template <>
struct AReg<false> {
    bf16x8 v;
    __device__ inline void fetch(const char *p) { v = *reinterpret_cast<const bf16x8 *>(p); }
    __device__ inline bf16x8 narrow(bool) const { return v; }
};
template <>
struct AReg<true> {
    f32x4 lo, hi;
    __device__ inline void fetch(const char *p)
    {
        lo = *reinterpret_cast<const f32x4 *>(p);
        hi = *reinterpret_cast<const f32x4 *>(p + 16);
    }
    __device__ inline bf16x8 narrow(bool valid) const
    {
        bf16x8 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[i] = (__bf16)(valid ? lo[i] : 0.0f);
            o[i + 4] = (__bf16)(valid ? hi[i] : 0.0f);
        }
        return o;
    }
};

// A_F32: A is fp32 [M][lda] with only k < K valid (K a multiple of 8); chunks at
// k >= K are fetched from the row's last valid chunk and zeroed.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_F32, bool OUT_F32>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void fc_big_kernel(
    const void *__restrict__ A0, int lda, long long a_stride, int M, int K, int Kpad,
    const FcGroups groups, int relu, void *__restrict__ C0, int ldc, long long c_stride, int grid_m,
    int grid_n, int tiles_per_group)
{
    constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // per-wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // 32 x 32 MFMA tiles per wave
    constexpr int ROWS_PER_PASS = THREADS / 8;           // 8 threads fetch the 64 k of one row
    constexpr int A_LOADS = BM / ROWS_PER_PASS, W_LOADS = BN / ROWS_PER_PASS;
    constexpr int BUF = (BM + BN) * LDS_LD;              // elements of one tile pair
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be whole MFMA tiles");
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "staging passes must tile the block");

    extern __shared__ __attribute__((aligned(16))) __bf16 smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    // XCD x (blocks are dealt round-robin) takes the x-th eighth of the tile
    // list; the list runs over strips of 4 row-tiles, column-tiles next, so the
    // tiles resident on one XCD form a compact patch that shares its slabs of A
    // and W in that XCD's L2.
    int v = blockIdx.x;
    if ((gridDim.x & 7) == 0) v = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int grp = v / tiles_per_group;
    v -= grp * tiles_per_group;
    int bm, bn;
    if ((grid_m & 3) == 0) {
        const int strip = v / (4 * grid_n), w = v - strip * 4 * grid_n;
        bn = w >> 2;
        bm = strip * 4 + (w & 3);
    } else {
        bm = v / grid_n;
        bn = v - bm * grid_n;
    }
    const int m0 = bm * BM, n0 = bn * BN;
    constexpr int A_ELT = A_F32 ? 4 : 2;
    const char *__restrict__ A = static_cast<const char *>(A0) + grp * a_stride * A_ELT;
    const __bf16 *__restrict__ W = static_cast<const __bf16 *>(groups.W[grp]);
    const float *__restrict__ bias = groups.bias[grp];

    const int ld_row = tid >> 3, ld_chunk = tid & 7;
    const char *a_src[A_LOADS];  // this thread's chunk of k-tile 0 in each of its rows
    const __bf16 *w_src[W_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int row = m0 + ld_row + ROWS_PER_PASS * i;
        row = row < M ? row : M - 1;  // rows past M are computed and dropped
        a_src[i] = A + (long long)row * lda * A_ELT;
    }
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i)
        w_src[i] = W + (long long)(n0 + ld_row + ROWS_PER_PASS * i) * Kpad + ld_chunk * 8;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    AReg<A_F32> ra[A_LOADS];
    bf16x8 rw[W_LOADS];
    const int nk = Kpad / BK;

    // The staging work of a k-tile (BK / 16 = 4 steps of MFMAs) is cut into 4 parts,
    // one per step, so that LDS writes, global loads and LDS reads are issued in
    // the shadow of the matrix instructions instead of in a burst of their own.
    constexpr int KSTEPS = BK / 16;
    constexpr int A_PART = (A_LOADS + KSTEPS - 1) / KSTEPS, W_PART = (W_LOADS + KSTEPS - 1) / KSTEPS;
#define REC_BIG_FETCH_PART(kt, part)                                                       \
    do {                                                                                   \
        int k_ = (kt) * BK + ld_chunk * 8;                                                 \
        if (A_F32) k_ = k_ < K ? k_ : K - 8;                                               \
        _Pragma("unroll") for (int i = (part) * A_PART; i < ((part) + 1) * A_PART && i < A_LOADS; ++i) \
            ra[i].fetch(a_src[i] + (long long)k_ * A_ELT);                                 \
        _Pragma("unroll") for (int i = (part) * W_PART; i < ((part) + 1) * W_PART && i < W_LOADS; ++i) \
            rw[i] = *reinterpret_cast<const bf16x8 *>(w_src[i] + (kt) * BK);               \
    } while (0)
#define REC_BIG_STASH_PART(kt, buf, part)                                                  \
    do {                                                                                   \
        __bf16 *sa_ = smem + (buf) * BUF, *sw_ = sa_ + BM * LDS_LD;                        \
        const bool valid_ = !A_F32 || (kt) * BK + ld_chunk * 8 < K; /* the chunk held in ra lies below K */ \
        _Pragma("unroll") for (int i = (part) * A_PART; i < ((part) + 1) * A_PART && i < A_LOADS; ++i) \
            *reinterpret_cast<bf16x8 *>(&sa_[(ld_row + ROWS_PER_PASS * i) * LDS_LD + ld_chunk * 8]) = ra[i].narrow(valid_); \
        _Pragma("unroll") for (int i = (part) * W_PART; i < ((part) + 1) * W_PART && i < W_LOADS; ++i) \
            *reinterpret_cast<bf16x8 *>(&sw_[(ld_row + ROWS_PER_PASS * i) * LDS_LD + ld_chunk * 8]) = rw[i]; \
    } while (0)
    // One k-tile: multiply tile kt out of buffer kt & 1; meanwhile (STASH) put the
    // registers holding tile kt+1 into the other buffer, whose last readers passed
    // the previous barrier, and (FETCH) refill them with tile kt+2.
#define REC_BIG_ITERATION(kt, STASH, FETCH)                                                \
    do {                                                                                   \
        const int cur_ = (kt) & 1;                                                         \
        const __bf16 *sA = smem + cur_ * BUF, *sW = sA + BM * LDS_LD;                      \
        _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk) {                            \
            const int kofs = kk * 16 + (lane >> 5) * 8;                                    \
            bf16x8 fw[TN], fa[TM];                                                         \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                 \
                fw[i] = *reinterpret_cast<const bf16x8 *>(&sW[(wn * WN + i * 32 + (lane & 31)) * LDS_LD + kofs]); \
            _Pragma("unroll") for (int j = 0; j < TM; ++j)                                 \
                fa[j] = *reinterpret_cast<const bf16x8 *>(&sA[(wm * WM + j * 32 + (lane & 31)) * LDS_LD + kofs]); \
            if (STASH) REC_BIG_STASH_PART((kt) + 1, cur_ ^ 1, kk);                                   \
            if (FETCH) REC_BIG_FETCH_PART((kt) + 2, kk);                                   \
            __builtin_amdgcn_sched_barrier(0); /* else the compiler sinks all fetches to the end of the k-tile */ \
            _Pragma("unroll") for (int i = 0; i < TN; ++i)                                 \
                _Pragma("unroll") for (int j = 0; j < TM; ++j)                             \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0); \
        }                                                                                  \
        __syncthreads();                                                                   \
    } while (0)

#pragma unroll
    for (int part = 0; part < KSTEPS; ++part) REC_BIG_FETCH_PART(0, part);
#pragma unroll
    for (int part = 0; part < KSTEPS; ++part) REC_BIG_STASH_PART(0, 0, part);
    if (nk > 1) {
#pragma unroll
        for (int part = 0; part < KSTEPS; ++part) REC_BIG_FETCH_PART(1, part);
    }
    __syncthreads();

    int kt = 0;
    for (; kt + 2 < nk; ++kt) REC_BIG_ITERATION(kt, true, true);
    if (kt + 1 < nk) {
        REC_BIG_ITERATION(kt, true, false);
        ++kt;
    }
    REC_BIG_ITERATION(kt, false, false);
#undef REC_BIG_ITERATION
#undef REC_BIG_FETCH_PART
#undef REC_BIG_STASH_PART

    // acc[i][j][r]: feature n = 8 * (r / 4) + 4 * (lane / 32) + r % 4, sample m = lane % 32.
    // A lane therefore holds 4 consecutive features of 32 different rows: stored
    // as they are, every store instruction would touch 32 lines with 16 bytes
    // each.  bf16 output goes through LDS instead (the operand tiles are done
    // with after the loop's last barrier): each wave lays its WM x WN tile out
    // row-major in a region of its own and writes it back as whole 128-byte rows.
    void *C = static_cast<char *>(C0) + grp * c_stride * (OUT_F32 ? 4 : 2);
    constexpr int EP_LD = WN + 8;  // padded row pitch of the staged tile (elements)
    static_assert(OUT_F32 || (size_t)WAVES_M * WAVES_N * WM * EP_LD <= 2 * (size_t)BUF, "staged C tiles must fit the LDS");
    __bf16 *stage = smem + (size_t)wave * WM * EP_LD;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m0 + wm * WM + j * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nl = i * 32 + 8 * q + 4 * (lane >> 5);  // column inside the wave tile
                const int n = n0 + wn * WN + nl;
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + n);
                f32x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float x = acc[i][j][4 * q + r] + bv[r];
                    o[r] = (relu && x < 0.0f) ? 0.0f : x;
                }
                if (OUT_F32) {
                    if (m < M) *reinterpret_cast<f32x4 *>(static_cast<float *>(C) + (long long)m * ldc + n) = o;
                } else {
                    bf16x4 h;
#pragma unroll
                    for (int r = 0; r < 4; ++r) h[r] = (__bf16)o[r];
                    *reinterpret_cast<bf16x4 *>(&stage[(j * 32 + (lane & 31)) * EP_LD + nl]) = h;
                }
            }
        }
    }
    if (!OUT_F32) {
        constexpr int LANES_PER_ROW = WN / 8;            // 16 bytes per lane
        constexpr int ROWS_PER_STORE = 64 / LANES_PER_ROW;
        const int sr = lane / LANES_PER_ROW, sc = (lane % LANES_PER_ROW) * 8;
        __bf16 *Cb = static_cast<__bf16 *>(C) + n0 + wn * WN + sc;
#pragma unroll
        for (int r0 = 0; r0 < WM; r0 += ROWS_PER_STORE) {
            const int row = r0 + sr;
            const bf16x8 v = *reinterpret_cast<const bf16x8 *>(&stage[row * EP_LD + sc]);
            const int m = m0 + wm * WM + row;
            if (m < M) *reinterpret_cast<bf16x8 *>(Cb + (long long)m * ldc) = v;
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_F32, bool OUT_F32>
hipError_t launch_big_as(const FcProblem &a, hipStream_t s)
{
    const int grid_m = (a.M + BM - 1) / BM, grid_n = a.Npad / BN;
    const int tiles = grid_m * grid_n;
    const dim3 grid(tiles * a.groups), block(64 * WAVES_M * WAVES_N);
    constexpr size_t lds = big_lds_bytes<BM, BN>();
    auto k = fc_big_kernel<BM, BN, WAVES_M, WAVES_N, A_F32, OUT_F32>;
    hipLaunchKernelGGL(k, grid, block, lds, s, a.A, a.lda, a.a_stride, a.M, a.K, a.Kpad, a.g,
                       a.relu ? 1 : 0, a.C, a.ldc, a.c_stride, grid_m, grid_n, tiles);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_big(const FcProblem &a, hipStream_t s)
{
    if (a.a_f32) {
        if (a.out_f32) return launch_big_as<BM, BN, WAVES_M, WAVES_N, true, true>(a, s);
        return launch_big_as<BM, BN, WAVES_M, WAVES_N, true, false>(a, s);
    }
    if (a.out_f32) return launch_big_as<BM, BN, WAVES_M, WAVES_N, false, true>(a, s);
    return launch_big_as<BM, BN, WAVES_M, WAVES_N, false, false>(a, s);
}

// More than 64 KB of dynamic LDS has to be granted to a kernel before its first launch.
template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t grant_lds()
{
    constexpr size_t lds = big_lds_bytes<BM, BN>();
    if (lds <= 64 * 1024) return hipSuccess;
    const void *kernels[4] = {
        reinterpret_cast<const void *>(fc_big_kernel<BM, BN, WAVES_M, WAVES_N, false, false>),
        reinterpret_cast<const void *>(fc_big_kernel<BM, BN, WAVES_M, WAVES_N, false, true>),
        reinterpret_cast<const void *>(fc_big_kernel<BM, BN, WAVES_M, WAVES_N, true, false>),
        reinterpret_cast<const void *>(fc_big_kernel<BM, BN, WAVES_M, WAVES_N, true, true>)};
    for (const void *k : kernels) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Which block tile, if any: 256 x 256, 256 x 128 (bf16 input) or 128 x 128, the
// largest whose tiles still cover three quarters of the compute units.
int big_tile_choice(const FcProblem &a, int num_cus)
{
    if (a.dot_out || a.M < 1024 || a.Kpad % BK != 0 || a.groups < 1 || a.groups > MAX_GROUPS) return 0;
    if (a.a_f32 && (a.K % 8 != 0 || a.lda % 4 != 0 || a.a_stride % 4 != 0 ||
                    reinterpret_cast<uintptr_t>(a.A) % 16 != 0))
        return 0;
    const long long need = (long long)num_cus * 3 / 4;
    const long long m256 = (a.M + 255) / 256, m128 = (a.M + 127) / 128;
    if (!a.a_f32 && a.Npad % 256 == 0 && a.groups * m256 * (a.Npad / 256) >= need) return 1;
    if (!a.a_f32 && a.Npad % 128 == 0 && a.groups * m256 * (a.Npad / 128) >= need) return 2;
    if (a.Npad % 128 == 0 && a.groups * m128 * (a.Npad / 128) >= need) return 3;
    return 0;
}

}  // namespace

bool fc_big_applies(const FcProblem &a, int num_cus) { return big_tile_choice(a, num_cus) != 0; }

hipError_t fc_big_prepare()
{
    hipError_t e = grant_lds<256, 256, 2, 4>();
    if (e == hipSuccess) e = grant_lds<256, 128, 4, 2>();
    if (e == hipSuccess) e = grant_lds<128, 128, 2, 4>();
    return e;
}

hipError_t launch_fc_big(const FcProblem &a, int num_cus, hipStream_t s)
{
    switch (big_tile_choice(a, num_cus)) {
    case 1: return launch_big<256, 256, 2, 4>(a, s);
    case 2: return launch_big<256, 128, 4, 2>(a, s);
    case 3: return launch_big<128, 128, 2, 4>(a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace rec
