// Measurement helper (not part of the forward pass): the rate at which the
// matrix cores run v_mfma_f32_32x32x16_bf16 on register operands, on constant
// or on pseudo-random values.  With every compute unit busy the chip is
// power-limited and the rate depends on the operand bits; a benchmark puts it
// beside the published peak.
#include "rec_internal.h"
#include "rec_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_WAVES = 8;

__global__ __launch_bounds__(64 * PROBE_WAVES) void mfma_probe_kernel(int random_operands, int iters,
                                                                      float *__restrict__ sink)
{
    // Two weight-like and four activation-like fragments, as a 128 x 64 wave tile holds per step.
    bf16x8 fw[2], fa[4];
    // Six independent fragments: a GEMM feeds every instruction fresh operands, and the
    // power drawn follows how many operand bits change from one instruction to the next.
#pragma unroll
    for (int f = 0; f < 6; ++f) {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            unsigned h = ((threadIdx.x * 8u + (unsigned)e) * 6u + (unsigned)f) * 2654435761u + 777u + blockIdx.x * 40503u;
            h ^= h >> 15;
            h *= 2246822519u;
            h ^= h >> 13;
            v[e] = (__bf16)(random_operands ? (float)((int)(h & 0xffffu) - 32768) * (1.0f / 32768.0f) : 1.0f);
        }
        if (f < 2) fw[f] = v;
        else fa[f - 2] = v;
    }
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        // Sums stay bounded and the operands keep changing: flip the sign of one fragment.
        if (random_operands) {
            bf16x8 t = fw[0];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = -t[e];
            fw[0] = t;
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s += acc[i][j][0];
    if (blockIdx.x == 0 && threadIdx.x == 0) sink[0] = s;
}

}  // namespace

extern "C" rec_status rec_probe_mfma(int32_t random_operands, int32_t blocks, int32_t iters,
                                     float *dev_sink, void *stream)
{
    if (!dev_sink || blocks <= 0 || blocks > 65536 || iters <= 0 || iters > (1 << 20)) return REC_ERR_ARG;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(64 * PROBE_WAVES), 0,
                       static_cast<hipStream_t>(stream), random_operands, iters, dev_sink);
    return hipGetLastError() == hipSuccess ? REC_OK : REC_ERR_DEVICE;
}
