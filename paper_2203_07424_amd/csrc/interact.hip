// S3: pairwise-dot feature interaction and concatenation (and, at the end, the
// dense part of the plain-concatenation model, which has no interaction).
//
// Per sample, the T pooled vectors and the Bottom-FC output x0 form
// X = [x0; pooled_0; ...; pooled_{T-1}]  (V = T + 1 rows of D).  The Predict-FC
// input is [x0, <X_i, X_j> for i > j] (strict lower triangle, row-major),
// narrowed to bf16 and zero padded to the GEMM's leading dimension -
// concatenation and conversion are fused here (Sec. IV-A, operator fusion).
//
// LDS-tiled: a block stages X of a few samples in LDS (16-byte columns of a
// row XOR-swizzled by the row number, so that the 16 lanes that read 16
// consecutive rows hit different banks).  The Gram matrix X X^T is a small
// dense contraction and plain vector FMAs make it ALU-bound, so each wave
// computes 16 x 16 tiles of it (blocks J <= I) with the fp32 matrix
// instruction v_mfma_f32_16x16x4_f32: fp32 operands, fp32 accumulation, the
// output's narrowing to bf16 is the only rounding.  Lane l feeds row l % 16 of
// both operands and 4 consecutive k picked by l / 16 (one 16-byte LDS read per
// operand serves four MFMAs).  Results are collected in LDS as one bf16 output
// row per sample and written out with full 16-byte stores.
#include "rec_internal.h"

namespace rec {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int IT_THREADS = 256;
constexpr int IT_WAVES = IT_THREADS / 64;
constexpr int IT_BATCH = 4;           // 16-byte loads in flight per thread while staging
constexpr int IT_TILES_PER_WAVE = 1;  // tiles a wave should get (sets the samples per block)

struct Geometry {
    int V, Vpad, nblk, ntile, d4, ksteps, swmask;
    size_t x_floats;  // floats of X per sample
};

__host__ __device__ inline Geometry geometry(int T, int D)
{
    Geometry g;
    g.V = T + 1;
    g.nblk = (g.V + 15) / 16;
    g.Vpad = g.nblk * 16;
    g.ntile = g.nblk * (g.nblk + 1) / 2;
    g.d4 = D / 4;
    g.ksteps = (g.d4 + 3) / 4;              // 16 k per step
    g.swmask = (g.d4 < 8 ? g.d4 : 8) - 1;  // d4 is a power of two
    g.x_floats = (size_t)g.Vpad * D;
    return g;
}

// KSTEPS > 0 fixes the number of 16-wide k steps (D = 16 * KSTEPS) so that the
// LDS reads of a tile are all issued before its MFMAs; 0 takes it at run time.
template <int KSTEPS>
__global__ __launch_bounds__(IT_THREADS) void interact_kernel(const float *__restrict__ x0, int ldx0,
                                                              const float *__restrict__ pooled,
                                                              int B, int T, int D,
                                                              __bf16 *__restrict__ out, int ldo,
                                                              int spb)
{
    extern __shared__ __attribute__((aligned(16))) float s_mem[];
    const Geometry g = geometry(T, D);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * spb;
    const int ns = min(spb, B - b0);  // samples of this block
    float *sX = s_mem;                                                  // [spb][Vpad][D], swizzled
    __bf16 *sO = reinterpret_cast<__bf16 *>(s_mem + (size_t)spb * g.x_floats);  // [spb][ldo]

    // Stage X: row 0 = x0, rows 1..T = pooled (contiguous), rows V..Vpad = 0.
    // d4 is a power of two, so rows and columns come from shifts; loads are
    // issued IT_BATCH at a time before their LDS stores.
    const int ld4 = __ffs(g.d4) - 1, n4 = g.Vpad << ld4;  // 16-byte words of X per sample
    for (int s = 0; s < ns; ++s) {
        const long long b = b0 + s;
        const float *px0 = x0 + b * ldx0;
        const float *pp = pooled + b * T * D - D;  // row r >= 1 sits at pp + r * D
        float *dst = sX + s * g.x_floats;
        for (int f0 = tid; f0 < n4; f0 += IT_BATCH * IT_THREADS) {
            f32x4 v[IT_BATCH];
#pragma unroll
            for (int u = 0; u < IT_BATCH; ++u) {
                const int f = f0 + u * IT_THREADS;
                const int row = f >> ld4, c4 = f & (g.d4 - 1);
                v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (f < n4 && row < g.V)
                    v[u] = *reinterpret_cast<const f32x4 *>((row == 0 ? px0 : pp + (size_t)row * D) + 4 * c4);
            }
#pragma unroll
            for (int u = 0; u < IT_BATCH; ++u) {
                const int f = f0 + u * IT_THREADS;
                const int row = f >> ld4, c4 = f & (g.d4 - 1);
                if (f < n4)
                    *reinterpret_cast<f32x4 *>(dst + (size_t)row * D + 4 * (c4 ^ (row & g.swmask))) = v[u];
            }
        }
    }
    __syncthreads();

    // Dense part (row 0 is not displaced by the swizzle) and zero padding.
    const int npairs = T * (T + 1) / 2, width = D + npairs;
    for (int s = 0; s < ns; ++s) {
        for (int c = tid; c < D; c += IT_THREADS) sO[s * ldo + c] = (__bf16)sX[s * g.x_floats + c];
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
        const int rowA = 16 * I + r16, rowB = 16 * J + r16;
        const float *xa = sX + s * g.x_floats + (size_t)rowA * D;
        const float *xb = sX + s * g.x_floats + (size_t)rowB * D;
        const int swa = rowA & g.swmask, swb = rowB & g.swmask;
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (KSTEPS > 0) {
            f32x4 a[KSTEPS > 0 ? KSTEPS : 1], b[KSTEPS > 0 ? KSTEPS : 1];
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const int c4 = 4 * ks + kq;
                a[ks] = *reinterpret_cast<const f32x4 *>(xa + 4 * (c4 ^ swa));
                b[ks] = *reinterpret_cast<const f32x4 *>(xb + 4 * (c4 ^ swb));
            }
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ks][v], b[ks][v], acc, 0, 0, 0);
        } else {
            for (int ks = 0; ks < g.ksteps; ++ks) {
                const int c4 = 4 * ks + kq;
                f32x4 a = {0.0f, 0.0f, 0.0f, 0.0f}, b = a;
                if (c4 < g.d4) {
                    a = *reinterpret_cast<const f32x4 *>(xa + 4 * (c4 ^ swa));
                    b = *reinterpret_cast<const f32x4 *>(xb + 4 * (c4 ^ swb));
                }
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v], b[v], acc, 0, 0, 0);
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
    return g.x_floats * sizeof(float) + (size_t)ldo * 2;
}

hipError_t launch_interact(const float *x0, int ldx0, const float *pooled, int B, int T, int D,
                           void *out_bf16, int ldo, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    const Geometry g = geometry(T, D);
    const size_t per = g.x_floats * sizeof(float) + (size_t)ldo * 2;
    if (per > 64 * 1024) return hipErrorInvalidValue;  // rejected at model creation
    // Enough samples per block to give every wave about one tile; small blocks
    // (little LDS each) keep many of them resident, which hides the staging
    // latency of one behind the matrix work of the others.
    int spb = (IT_TILES_PER_WAVE * IT_WAVES + g.ntile - 1) / g.ntile;
    while (spb > 1 && spb * per > 32 * 1024) --spb;
    const dim3 grid((B + spb - 1) / spb), block(IT_THREADS);
    __bf16 *o = static_cast<__bf16 *>(out_bf16);
    const size_t lds = spb * per;
    switch (D) {
    case 16: hipLaunchKernelGGL(interact_kernel<1>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    case 32: hipLaunchKernelGGL(interact_kernel<2>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    case 64: hipLaunchKernelGGL(interact_kernel<4>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
    case 128: hipLaunchKernelGGL(interact_kernel<8>, grid, block, lds, s, x0, ldx0, pooled, B, T, D, o, ldo, spb); break;
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
