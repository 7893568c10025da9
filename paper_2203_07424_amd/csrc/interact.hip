// S3: pairwise-dot feature interaction and concatenation (and, at the end, the
// dense part of the plain-concatenation model, which has no interaction).
//
// Per sample, the T pooled vectors and the Bottom-FC output x0 form
// X = [x0; pooled_0; ...; pooled_{T-1}]  (V = T + 1 rows of D).  The Predict-FC
// input is [x0, <X_i, X_j> for i > j] (strict lower triangle, row-major),
// narrowed to bf16 and zero padded to the GEMM's leading dimension -
// concatenation and conversion are fused here (Sec. IV-A, operator fusion).
//
// LDS-tiled: a block stages X of a few samples in LDS and each wave computes
// 16 x 16 tiles of the Gram matrix X X^T (blocks J <= I) on the matrix cores.
// The fp32 matrix instruction is slow (1/16 of the bf16 rate), and narrowing X
// to bf16 would cost the interaction its fp32 accuracy, so X is split instead:
// x = hi + lo with hi = bf16(x) and lo = bf16(x - hi), and
//   <x, y> = <hi_x, hi_y> + <hi_x, lo_y> + <lo_x, hi_y>   (+ <lo_x, lo_y>, dropped: 2^-16 relative)
// is three v_mfma_f32_16x16x32_bf16 per 32 k with fp32 accumulation.  hi + lo
// carries 16 significant bits of x, so each product is good to about 2^-16
// relative: far below the 2^-9 of the bf16 narrowing of the output, which stays
// the only rounding that matters.  Lane l feeds row l % 16 of both operands and
// the 8 consecutive k picked by l / 16.  The two planes sit in LDS with rows
// padded by 16 bytes (conflict-free 16-byte reads of 16 consecutive rows).
// Results are collected in LDS as one bf16 output row per sample and written
// out with full 16-byte stores.
#include "rec_internal.h"

namespace rec {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int IT_THREADS = 256;
constexpr int IT_WAVES = IT_THREADS / 64;
constexpr int IT_BATCH = 4;           // 16-byte loads in flight per thread while staging
constexpr int IT_TILES_PER_WAVE = 1;  // tiles a wave should get (sets the samples per block)

struct Geometry {
    int V, Vpad, nblk, ntile, d4, dp, ld, ksteps;
    size_t plane;  // elements of one bf16 plane (hi or lo) of X per sample
};

__host__ __device__ inline Geometry geometry(int T, int D)
{
    Geometry g;
    g.V = T + 1;
    g.nblk = (g.V + 15) / 16;
    g.Vpad = g.nblk * 16;
    g.ntile = g.nblk * (g.nblk + 1) / 2;
    g.d4 = D / 4;
    g.dp = (D + 31) / 32 * 32;  // k extent, padded with zeros to whole MFMA steps
    g.ld = g.dp + 8;            // padded row stride (elements)
    g.ksteps = g.dp / 32;
    g.plane = (size_t)g.Vpad * g.ld;
    return g;
}

// KSTEPS > 0 fixes the number of 32-wide k steps so that the LDS reads of a
// tile are all issued before its MFMAs; 0 takes it at run time.
template <int KSTEPS>
__global__ __launch_bounds__(IT_THREADS) void interact_kernel(const float *__restrict__ x0, int ldx0,
                                                              const float *__restrict__ pooled,
                                                              int B, int T, int D,
                                                              __bf16 *__restrict__ out, int ldo,
                                                              int spb)
{
    extern __shared__ __attribute__((aligned(16))) __bf16 s_mem[];
    const Geometry g = geometry(T, D);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * spb;
    const int ns = min(spb, B - b0);  // samples of this block
    __bf16 *sHi = s_mem;                             // [spb][Vpad][ld]
    __bf16 *sLo = sHi + (size_t)spb * g.plane;       // [spb][Vpad][ld]
    __bf16 *sO = sLo + (size_t)spb * g.plane;        // [spb][ldo]

    // Stage X: row 0 = x0, rows 1..T = pooled (contiguous), rows V..Vpad and the
    // columns D..dp = 0.  A thread moves 4 consecutive columns at a time; loads
    // are issued IT_BATCH at a time before their LDS stores.
    const int c4n = g.dp / 4;             // 4-column groups per (padded) row
    const int n4 = g.Vpad * c4n;          // ... per sample
    // Item f = tid + k * IT_THREADS is row f / c4n, group f % c4n: divided once per
    // thread, then stepped (a division by a run-time value costs some 20 vector
    // instructions, and this kernel is bound by instruction issue).
    const int step_row = IT_THREADS / c4n, step_c4 = IT_THREADS % c4n;  // wave-uniform
    const int row_first = tid / c4n, c4_first = tid - row_first * c4n;
    for (int s = 0; s < ns; ++s) {
        const long long b = b0 + s;
        const float *px0 = x0 + b * ldx0;
        const float *pp = pooled + b * T * D - D;  // row r >= 1 sits at pp + r * D
        __bf16 *hi = sHi + s * g.plane, *lo = sLo + s * g.plane;
        int row_next = row_first, c4_next = c4_first;
        for (int f0 = tid; f0 < n4; f0 += IT_BATCH * IT_THREADS) {
            f32x4 v[IT_BATCH];
            int row[IT_BATCH], c4[IT_BATCH];
#pragma unroll
            for (int u = 0; u < IT_BATCH; ++u) {
                row[u] = row_next;
                c4[u] = c4_next;
                c4_next += step_c4;
                row_next += step_row;
                if (c4_next >= c4n) {
                    c4_next -= c4n;
                    ++row_next;
                }
                v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (row[u] < g.V && c4[u] < g.d4)  // rows past Vpad (items f >= n4) are past V too
                    v[u] = *reinterpret_cast<const f32x4 *>((row[u] == 0 ? px0 : pp + (size_t)row[u] * D) + 4 * c4[u]);
            }
#pragma unroll
            for (int u = 0; u < IT_BATCH; ++u) {
                if (f0 + u * IT_THREADS < n4) {
                    bf16x4 h, l;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        h[i] = (__bf16)v[u][i];
                        l[i] = (__bf16)(v[u][i] - (float)h[i]);
                    }
                    *reinterpret_cast<bf16x4 *>(hi + (size_t)row[u] * g.ld + 4 * c4[u]) = h;
                    *reinterpret_cast<bf16x4 *>(lo + (size_t)row[u] * g.ld + 4 * c4[u]) = l;
                }
            }
        }
    }
    __syncthreads();

    // Dense part (bf16(x0) is the hi plane of row 0) and zero padding.
    const int npairs = T * (T + 1) / 2, width = D + npairs;
    for (int s = 0; s < ns; ++s) {
        for (int c = tid; c < D; c += IT_THREADS) sO[s * ldo + c] = sHi[s * g.plane + c];
        for (int c = width + tid; c < ldo; c += IT_THREADS) sO[s * ldo + c] = (__bf16)0.0f;
    }

    // 16 x 16 tiles of the lower triangle, one wave per tile.
    const int r16 = lane & 15, kq = lane >> 4;
    for (int q = wave; q < ns * g.ntile; q += IT_WAVES) {
        int s = 0, tile = q;
        while (tile >= g.ntile) { tile -= g.ntile; ++s; }
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        const size_t offA = s * g.plane + (size_t)(16 * I + r16) * g.ld + 8 * kq;
        const size_t offB = s * g.plane + (size_t)(16 * J + r16) * g.ld + 8 * kq;
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (KSTEPS > 0) {
            bf16x8 ah[KSTEPS > 0 ? KSTEPS : 1], al[KSTEPS > 0 ? KSTEPS : 1], bh[KSTEPS > 0 ? KSTEPS : 1],
                bl[KSTEPS > 0 ? KSTEPS : 1];
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                ah[ks] = *reinterpret_cast<const bf16x8 *>(sHi + offA + 32 * ks);
                al[ks] = *reinterpret_cast<const bf16x8 *>(sLo + offA + 32 * ks);
                bh[ks] = *reinterpret_cast<const bf16x8 *>(sHi + offB + 32 * ks);
                bl[ks] = *reinterpret_cast<const bf16x8 *>(sLo + offB + 32 * ks);
            }
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[ks], bh[ks], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[ks], bl[ks], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[ks], bh[ks], acc, 0, 0, 0);
            }
        } else {
            for (int ks = 0; ks < g.ksteps; ++ks) {
                const bf16x8 ah = *reinterpret_cast<const bf16x8 *>(sHi + offA + 32 * ks);
                const bf16x8 al = *reinterpret_cast<const bf16x8 *>(sLo + offA + 32 * ks);
                const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(sHi + offB + 32 * ks);
                const bf16x8 bl = *reinterpret_cast<const bf16x8 *>(sLo + offB + 32 * ks);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bh, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bl, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bh, acc, 0, 0, 0);
            }
        }
        // acc[v] = <X_i, X_j>, i = 16 I + 4 (lane / 16) + v, j = 16 J + lane % 16.
        const int j = 16 * J + r16;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 16 * I + 4 * kq + v;
            if (i < g.V && j < i) sO[s * ldo + D + i * (i - 1) / 2 + j] = (__bf16)acc[v];
        }
    }
    __syncthreads();

    // Output rows, 16 bytes per lane (ldo is a multiple of 64 elements).
    const int row_u4 = ldo / 8;
    for (int s = 0; s < ns; ++s)
        for (int c = tid; c < row_u4; c += IT_THREADS)
            *reinterpret_cast<u32x4 *>(out + (long long)(b0 + s) * ldo + 8 * c) =
                *reinterpret_cast<const u32x4 *>(sO + s * ldo + 8 * c);
}

// Concatenation model (no interaction operator): the dense part of each
// Predict-FC input row, narrowed, and the zero padding behind the row.
__global__ __launch_bounds__(256) void concat_dense_kernel(const float *__restrict__ x0, int ldx0, int w0,
                                                           int B, __bf16 *__restrict__ z, int width,
                                                           int ldz)
{
    const int per_row = w0 + (ldz - width);
    const long long total = (long long)B * per_row;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long b = i / per_row;
        const int c = (int)(i - b * per_row);
        if (c < w0)
            z[b * ldz + c] = (__bf16)x0[b * ldx0 + c];
        else
            z[b * ldz + width + (c - w0)] = (__bf16)0.0f;
    }
}

}  // namespace

size_t interact_lds_bytes_per_sample(int T, int D)
{
    const Geometry g = geometry(T, D);
    const int ldo = pad_up(D + T * (T + 1) / 2);
    return 2 * g.plane * sizeof(__bf16) + (size_t)ldo * 2;
}

hipError_t launch_interact(const float *x0, int ldx0, const float *pooled, int B, int T, int D,
                           void *out_bf16, int ldo, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    const Geometry g = geometry(T, D);
    const size_t per = 2 * g.plane * sizeof(__bf16) + (size_t)ldo * 2;
    if (per > 64 * 1024) return hipErrorInvalidValue;  // rejected at model creation
    // Enough samples per block to give every wave about one tile; small blocks
    // (little LDS each) keep many of them resident, which hides the staging
    // latency of one behind the matrix work of the others.
    int spb = (IT_TILES_PER_WAVE * IT_WAVES + g.ntile - 1) / g.ntile;
    while (spb > 1 && spb * per > 32 * 1024) --spb;
    const dim3 grid((B + spb - 1) / spb), block(IT_THREADS);
    __bf16 *o = static_cast<__bf16 *>(out_bf16);
    const size_t lds = spb * per;
    switch (g.ksteps) {
    case 1: hipLaunchKernelGGL(interact_kernel<1>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    case 2: hipLaunchKernelGGL(interact_kernel<2>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    case 4: hipLaunchKernelGGL(interact_kernel<4>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    default: hipLaunchKernelGGL(interact_kernel<0>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    }
    return hipGetLastError();
}

hipError_t launch_concat_dense(const float *x0, int ldx0, int w0, int B, void *z_bf16, int width,
                               int ldz, hipStream_t s)
{
    const long long total = (long long)B * (w0 + ldz - width);
    if (total <= 0) return hipSuccess;
    const int blocks = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(concat_dense_kernel, dim3(blocks), dim3(256), 0, s, x0, ldx0, w0, B,
                       static_cast<__bf16 *>(z_bf16), width, ldz);
    return hipGetLastError();
}

}  // namespace rec
