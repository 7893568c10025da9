// Internal declarations shared by the gfx950 kernels and the C boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rec.h"

namespace rec {

// Device error record (64 bytes, lives at the start of the workspace).
// Positions are kept with atomicMin, so "none" is all ones.
struct ErrRecord {
    unsigned long long first_bad_len;  // smallest position of a negative length
    unsigned long long first_bad_idx;  // smallest position of an id outside its table
    unsigned int flags;                // ERR_* bits
    unsigned int pad[11];
};
enum : unsigned int { ERR_NEG_LENGTH = 1u, ERR_TOTAL_MISMATCH = 2u, ERR_INDEX_RANGE = 4u };

struct TableDesc {
    const void *base;
    long long rows;
    const int32_t *hot_ids;  // rows worth caching in LDS (may be null)
    int n_hot;
    int pad;
};

// S0: one scan block covers SCAN_TILE lengths.
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

// All activations and packed weights use leading dimensions that are
// multiples of this many elements.
constexpr int PAD = 64;
inline int pad_up(int x) { return (x + PAD - 1) / PAD * PAD; }

hipError_t launch_clear_err(ErrRecord *err, hipStream_t s);

// S0. offsets[k] = min(sum_{j<k} max(len[j], 0), nnz), k = 0..n; block_sums is
// scratch of ceil(n / SCAN_TILE) int64 entries.
// With a ConcatDense job (x0 != null) extra blocks of the second launch also do
// the work of launch_concat_dense(), which a model without Bottom-FC can start
// this early: its x0 is the dense input.
struct ConcatDense {
    const float *x0 = nullptr;
    int ldx0 = 0, w0 = 0, B = 0;
    void *z_bf16 = nullptr;
    int width = 0, ldz = 0;
};
// With `rider` (a stack of fully connected layers that fits the on-chip kernel,
// fp32 input, one stack) further blocks of the second launch run that stack:
// Bottom-FC does not depend on the sparse side (Sec. III-A), so it can share a
// launch with the scan instead of costing one of its own.
struct ChainProblem;
hipError_t launch_scan(const int32_t *lengths, int n, long long nnz, int32_t *offsets,
                       long long *block_sums, ErrRecord *err, const ConcatDense &job,
                       const ChainProblem *rider, hipStream_t s);
// Once per process and device, before the first launch (not under stream capture).
hipError_t scan_prepare();

// Where S1 leaves the sum of bag (t, b): fp32 pooled[b][t][:], or (z != null,
// concatenation model) narrowed to bf16 at z[b][col0 + t * D ...], row stride ldz.
struct PoolOut {
    float *pooled;
    void *z;
    int ldz, col0;
};

// S1. Sum of the rows of every bag, fp32 accumulation.  nnz (the batch's id
// count) only picks the launch shape: bags of a few ids share a wavefront.
// stream_rows: load rows with the non-temporal hint (id streams without reuse).
// max_rows: row count of the largest table (tables under 4 GiB take 32-bit offsets).
hipError_t launch_pool(const TableDesc *tables, int dtype, int T, int D, int B,
                       const int32_t *indices, const int32_t *offsets, PoolOut out, long long nnz,
                       bool stream_rows, long long max_rows, ErrRecord *err, hipStream_t s);

// S1 with the tables' hot rows served from an LDS copy (hcap: power of two >= the
// longest hot list, pool_hot_fits(hcap, rowbytes) must hold).
bool pool_hot_fits(int hcap, int rowbytes);
hipError_t launch_pool_hot(const TableDesc *tables, int dtype, int T, int D, int B,
                           const int32_t *indices, const int32_t *offsets, float *pooled, int hcap,
                           int num_cus, ErrRecord *err, hipStream_t s);

// S2 / S4. One layer of `groups` stacks that run side by side (the task towers
// of the Predict-FC; 1 for a single stack), stack g being
//   C_g[m][n] = act(sum_k A_g[m][k] * W_g[n][k] + bias_g[n])   on bf16 MFMA, with
//   A_g = A + g * a_stride: bf16 [M][lda] or (a_f32) fp32 [M][lda] with only k < K
//         valid; a_stride = 0 when all stacks read the same input
//   W_g: bf16 [Npad][Kpad], bias_g fp32 [Npad] (zero padded)
//   C_g = C + g * c_stride: bf16 [M][ldc] or (out_f32) fp32 [M][ldc]
// With dot_out != null (allowed when fc_can_fuse_dot(Npad)) C is not stored;
// instead dot_out[m * dot_ld + g] = sum_n act(C_g[m][n]) * dot_w_g[n] + dot_bias_g[0],
// the one-output layer that follows, in fp32.
constexpr int MAX_GROUPS = REC_MAX_TOWERS;
struct FcGroups {
    const void *W[MAX_GROUPS];
    const float *bias[MAX_GROUPS];
    const float *dot_w[MAX_GROUPS];
    const float *dot_bias[MAX_GROUPS];
};
struct FcProblem {
    const void *A; bool a_f32; int lda; long long a_stride;
    int M, K, Kpad, Npad; bool relu;
    void *C; bool out_f32; int ldc; long long c_stride;
    int groups;
    FcGroups g;
    float *dot_out; int dot_ld;
    int num_cus;  // compute units of the device; 0 = unknown (never picks the wide-tile kernels)
    bool corun;   // the launch will share the device with a pooling launch: keep register use low
};
bool fc_can_fuse_dot(int Npad);
hipError_t launch_fc(const FcProblem &p, hipStream_t s);

// The same product with 256-row block tiles (bf16 input, C stored), for layers
// wide and batches large enough that such tiles still cover the chip;
// launch_fc() takes this path by itself when fc_big_applies().
bool fc_big_applies(const FcProblem &p, int num_cus);
hipError_t launch_fc_big(const FcProblem &p, int num_cus, hipStream_t s);
// Once per process and device, before the first launch (not under stream
// capture): lets these kernels use their more-than-64-KB LDS tiles.
hipError_t fc_big_prepare();

// A run of layers of every stack in one launch, activations kept on chip:
//   X_0 = A_g (bf16 [M][lda], or fp32 with a_f32; columns >= K read as zero),
//   X_{L+1} = act_L(X_L W_{L,g}^T + bias_{L,g}),  act_L = ReLU where relu[L] != 0,
// each layer narrowing its input to bf16 as the per-layer path does.  Layer L is
// Kpad[L] -> Npad[L] with Kpad[L + 1] == Npad[L], all at most CHAIN_MAX_WIDTH
// and multiples of PAD; W[L][g] is the fragment order launch_pack_chain() writes.
// The last X goes to C_g = C + g * c_stride (CHAIN_OUT_BF16 / CHAIN_OUT_F32, row
// stride ldc), or (CHAIN_OUT_DOT) into the one-output layer that follows:
//   dot_out[m * dot_ld + g] = sum_n X[m][n] * dot_w[g][n] + dot_bias[g][0]   in fp32.
constexpr int CHAIN_MAX_LAYERS = 6;
constexpr int CHAIN_MAX_WIDTH = 1024;
enum { CHAIN_OUT_BF16 = 0, CHAIN_OUT_F32 = 1, CHAIN_OUT_DOT = 2 };
struct ChainProblem {
    const void *A; bool a_f32; int lda; long long a_stride;
    int M, K;
    int n_layers, groups;
    int Kpad[CHAIN_MAX_LAYERS], Npad[CHAIN_MAX_LAYERS], relu[CHAIN_MAX_LAYERS];
    const void *W[CHAIN_MAX_LAYERS][MAX_GROUPS];
    const float *bias[CHAIN_MAX_LAYERS][MAX_GROUPS];
    int out_mode;
    void *C; int ldc; long long c_stride;
    const float *dot_w[MAX_GROUPS];
    const float *dot_bias[MAX_GROUPS];
    float *dot_out; int dot_ld;
    int ld_lds, a_vec;  // filled in by chain_finalize()
};
bool chain_layer_fits(int Kpad, int Npad);
// Checks p and completes it (LDS row pitch, whether wide input loads apply) into a.
hipError_t chain_finalize(const ChainProblem &p, ChainProblem &a);
hipError_t launch_mlp_chain(const ChainProblem &p, hipStream_t s);
// Once per process and device, before the first launch (not under stream capture).
hipError_t chain_prepare();
// fp32 [N][K] -> bf16 [Npad * Kpad] in MFMA fragment order (nearest even, zero padded).
hipError_t launch_pack_chain(const float *W, int N, int K, int Npad, int Kpad, void *W_packed, hipStream_t s);

// Last Predict-FC layer of every stack: logits[m * ld + g] = sum_k A_g[m][k] * w_g[k] + bias_g[0]
// in fp32.  A_g = A + g * a_stride is fp32 [M][lda] (a_f32) or bf16 [M][lda];
// w_g = groups.dot_w[g] is fp32 [Kpad], zero padded, bias_g = groups.dot_bias[g].
hipError_t launch_rowdot(const void *A, bool a_f32, int lda, long long a_stride, int M, int Kpad,
                         const FcGroups &groups, int n_groups, float *logits, int ld, hipStream_t s);
hipError_t launch_pack_dot(const float *W, const float *b, int K, int Kpad, float *W_packed,
                           float *bias_packed, hipStream_t s);

// fp32 [N][K] -> bf16 [Npad][Kpad] (nearest even, zero padded), bias -> fp32 [Npad].
hipError_t launch_pack_fc(const float *W, const float *b, int N, int K, int Npad, int Kpad,
                          void *W_packed, float *bias_packed, hipStream_t s);

// S3. out[b] = bf16([x0[b], <v_i, v_j> i > j, 0 ...]) with v = [x0[b], pooled[b][0..T-1]].
size_t interact_lds_bytes_per_sample(int T, int D);
hipError_t launch_interact(const float *x0, int ldx0, const float *pooled, int B, int T, int D,
                           void *out_bf16, int ldo, hipStream_t s);


// Concatenation model: z[b][0 .. w0) = bf16(x0[b][0 .. w0)) and z[b][width .. ldz) = 0;
// the looked-up vectors in between are written by S1.
hipError_t launch_concat_dense(const float *x0, int ldx0, int w0, int B, void *z_bf16, int width,
                               int ldz, hipStream_t s);

}  // namespace rec
