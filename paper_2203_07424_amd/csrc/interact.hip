// S3: pairwise-dot feature interaction and concatenation.
//
// Per sample, the T pooled vectors and the Bottom-FC output x0 form
// X = [x0; pooled_0; ...; pooled_{T-1}]  ((T+1) x D).  The Predict-FC input is
// [x0, <X_i, X_j> for i > j] (strict lower triangle, row-major), narrowed to
// bf16 and zero padded to the GEMM's leading dimension - concatenation and
// conversion are fused here (Sec. IV-A, operator fusion).
//
// One wavefront per sample: X is staged in LDS with a row stride of D + 4
// floats (consecutive rows start 4 banks apart, so 16-byte reads of
// consecutive rows do not collide), each lane owns pairs p, p + 64, ... and
// walks D with 16-byte LDS reads.  fp32 arithmetic; the output is the only
// rounding.
#include "rec_internal.h"

namespace rec {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void interact_kernel(const float *__restrict__ x0, int ldx0,
                                                       const float *__restrict__ pooled, int B,
                                                       int T, int D, __bf16 *__restrict__ out,
                                                       int ldo, int waves_per_block)
{
    extern __shared__ __attribute__((aligned(16))) float s_x[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x * waves_per_block + wave;
    const bool active = b < B;  // the block is launched with exactly waves_per_block waves

    const int V = T + 1, ld = D + 4, d4 = D / 4;
    float *X = s_x + (size_t)wave * V * ld;

    // Stage x0 then the T pooled vectors (contiguous T * D floats).
    if (active) {
        for (int i = lane; i < d4; i += 64)
            *reinterpret_cast<f32x4 *>(X + 4 * i) =
                *reinterpret_cast<const f32x4 *>(x0 + (long long)b * ldx0 + 4 * i);
        const float *P = pooled + (long long)b * T * D;
        for (int i = lane; i < T * d4; i += 64) {
            const int r = i / d4, c = i - r * d4;
            *reinterpret_cast<f32x4 *>(X + (r + 1) * ld + 4 * c) =
                *reinterpret_cast<const f32x4 *>(P + 4 * i);
        }
    }
    __syncthreads();
    if (!active) return;

    __bf16 *o = out + (long long)b * ldo;
    for (int d = lane; d < D; d += 64) o[d] = (__bf16)X[d];

    const int npairs = T * (T + 1) / 2;
    // Pair p -> (i, j), i > j >= 0, p = i (i - 1) / 2 + j.
    int i = 1, j = lane;
    while (j >= i) { j -= i; ++i; }
    for (int p = lane; p < npairs; p += 64) {
        const float *xi = X + i * ld, *xj = X + j * ld;
        float acc = 0.0f;
        for (int c = 0; c < d4; ++c) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(xi + 4 * c);
            const f32x4 w = *reinterpret_cast<const f32x4 *>(xj + 4 * c);
            acc += a[0] * w[0];
            acc += a[1] * w[1];
            acc += a[2] * w[2];
            acc += a[3] * w[3];
        }
        o[D + p] = (__bf16)acc;
        j += 64;
        while (j >= i) { j -= i; ++i; }
    }
    for (int c = D + npairs + lane; c < ldo; c += 64) o[c] = (__bf16)0.0f;
}

}  // namespace

size_t interact_lds_bytes_per_sample(int T, int D)
{
    return (size_t)(T + 1) * (D + 4) * sizeof(float);
}

hipError_t launch_interact(const float *x0, int ldx0, const float *pooled, int B, int T, int D,
                           void *out_bf16, int ldo, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    const size_t per = interact_lds_bytes_per_sample(T, D);
    if (per > 64 * 1024) return hipErrorInvalidValue;  // rejected at model creation
    int wpb = (int)((64 * 1024) / per);
    wpb = wpb > 4 ? 4 : wpb;
    const dim3 grid((B + wpb - 1) / wpb), block(wpb * 64);
    hipLaunchKernelGGL(interact_kernel, grid, block, wpb * per, s, x0, ldx0, pooled, B, T, D,
                       static_cast<__bf16 *>(out_bf16), ldo, wpb);
    return hipGetLastError();
}

}  // namespace rec
