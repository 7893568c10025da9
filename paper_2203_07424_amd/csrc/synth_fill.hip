// Device-side filling of synthetic embedding tables (an input generator, not
// part of the forward pass).  Element (table, row, col) is a pure function of
// (seed, table, row, col): the n-th output of a SplitMix64 stream (Steele, Lea,
// Flood, OOPSLA 2014), n = ((table << 32) + row) * 1024 + col, mapped onto a
// 2^24-point grid of [-0.05, 0.05) with a single fp32 multiply.
#include <hip/hip_fp16.h>

#include "rec_internal.h"
#include "rec_synth.h"

namespace {

__device__ inline unsigned long long mix64(unsigned long long z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ inline float synth_value(unsigned long long seed, unsigned long long n)
{
    const unsigned long long z = mix64(seed + (n + 1ull) * 0x9E3779B97F4A7C15ull);
    const int u24 = (int)(z >> 40);
    return (float)(u24 - (1 << 23)) * (0.05f * 0x1p-23f);
}

template <bool HALF>
__global__ __launch_bounds__(256) void fill_kernel(void *dst, unsigned long long seed,
                                                   unsigned long long table, long long rows, int D)
{
    const long long total = rows * D;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const unsigned long long r = (unsigned long long)(i / D), c = (unsigned long long)(i % D);
        float v = synth_value(seed, ((table << 32) + r) * 1024ull + c);
        // The fp32 product must be rounded before it is narrowed: keep the
        // compiler from folding multiply and conversion into one rounding.
        asm volatile("" : "+v"(v));
        if (HALF)
            static_cast<_Float16 *>(dst)[i] = (_Float16)v;  // nearest even
        else
            static_cast<float *>(dst)[i] = v;
    }
}

}  // namespace

extern "C" rec_status rec_synth_fill_table(void *dev_rows, int32_t dtype, uint64_t seed,
                                           int32_t table, int64_t rows, int32_t emb_dim,
                                           void *stream)
{
    if (!dev_rows || rows <= 0 || emb_dim <= 0 || emb_dim > 1024 || table < 0 ||
        rows >= (1ll << 32) || (dtype != REC_F32 && dtype != REC_F16))
        return REC_ERR_ARG;
    const long long total = rows * emb_dim;
    const long long want = (total + 255) / 256;
    const int blocks = (int)(want < 65536 ? want : 65536);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == REC_F16)
        hipLaunchKernelGGL(fill_kernel<true>, dim3(blocks), dim3(256), 0, s, dev_rows,
                           (unsigned long long)seed, (unsigned long long)table, (long long)rows, emb_dim);
    else
        hipLaunchKernelGGL(fill_kernel<false>, dim3(blocks), dim3(256), 0, s, dev_rows,
                           (unsigned long long)seed, (unsigned long long)table, (long long)rows, emb_dim);
    return hipGetLastError() == hipSuccess ? REC_OK : REC_ERR_DEVICE;
}
