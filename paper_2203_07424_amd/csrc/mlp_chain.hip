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
#include "mlp_chain_body.h"

namespace rec {

namespace {

using namespace chain;

template <bool A_F32>
__global__ __launch_bounds__(CH_THREADS) void mlp_chain_kernel(const ChainProblem a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    mlp_chain_block<A_F32>(a, smem, blockIdx.x, blockIdx.y, gridDim.x);
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

hipError_t chain_finalize(const ChainProblem &p, ChainProblem &a)
{
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
    a = p;
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
    return hipSuccess;
}

hipError_t launch_mlp_chain(const ChainProblem &p, hipStream_t s)
{
    if (p.M <= 0) return hipSuccess;
    ChainProblem a;
    const hipError_t e = chain_finalize(p, a);
    if (e != hipSuccess) return e;
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
