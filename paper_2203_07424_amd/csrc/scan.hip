// S0: pooling lengths -> bag offsets (exclusive scan), staged in LDS.
//
// The sparse input gives, per (table, sample), how many ids follow (the pooling
// factor varies per lookup, Fig. 2(c)); the gather needs where each bag starts.
// Two passes over at most a few hundred thousand int32: per-tile sums, then
// per-tile scans in LDS that first reduce the sums of the tiles before them.
// One-launch variants were measured and dropped: blocks re-reading the earlier
// lengths themselves (5x slower, a single block pulls only tens of GB/s); tile
// totals reduced by each pooling wave (+28 us of pooling for -3 us of scan);
// a last-block-done ticket (its device-scope fences cost more than a launch).
#include <algorithm>
#include "mlp_chain_body.h"

namespace rec {

namespace {

__device__ inline long long wave_sum(long long v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;  // valid in lane 0
}

// Sum over the block, returned to every thread.
__device__ inline long long block_sum(long long v, long long *s_w)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) s_w[wave] = v;
    __syncthreads();
    long long r = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; ++w) r += s_w[w];
    return r;
}

__global__ __launch_bounds__(64) void clear_err_kernel(ErrRecord *err)
{
    if (threadIdx.x == 0) {
        err->first_bad_len = ~0ull;
        err->first_bad_idx = ~0ull;
        err->flags = 0u;
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_tile_sums(const int32_t *__restrict__ len,
                                                               int n, long long *__restrict__ tile_sums)
{
    __shared__ long long s_w[SCAN_THREADS / 64];
    const long long base = (long long)blockIdx.x * SCAN_TILE;
    long long sum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        const long long k = base + i * SCAN_THREADS + threadIdx.x;
        if (k < n) {
            const int v = len[k];
            if (v > 0) sum += v;
        }
    }
    sum = block_sum(sum, s_w);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = sum;
}

// Dense part of the Predict-FC input rows of a concatenation model, narrowed,
// and the zero padding behind each row: block `b` of `nb` blocks.
__device__ inline void concat_dense_block(const ConcatDense &job, int b, int nb)
{
    __bf16 *z = static_cast<__bf16 *>(job.z_bf16);
    const int per_row = job.w0 + (job.ldz - job.width);
    const long long total = (long long)job.B * per_row;
    const long long stride = (long long)nb * blockDim.x;
    for (long long i = (long long)b * blockDim.x + threadIdx.x; i < total; i += stride) {
        const long long r = i / per_row;
        const int c = (int)(i - r * per_row);
        if (c < job.w0)
            z[r * job.ldz + c] = (__bf16)job.x0[r * job.ldx0 + c];
        else
            z[r * job.ldz + job.width + (c - job.w0)] = (__bf16)0.0f;
    }
}

// Offsets of tile `tile`; the threads with threadIdx.x < SCAN_THREADS call it,
// all of them.
__device__ inline void scan_offsets_tile(const int32_t *__restrict__ len, int n, long long nnz,
                                         const long long *__restrict__ tile_sums,
                                         int32_t *__restrict__ offsets, ErrRecord *err, int tile)
{
    // One extra word per 32 keeps the 8-per-thread strided reads off one bank.
    __shared__ int s_tile[SCAN_TILE + SCAN_TILE / 32];
    __shared__ long long s_w[SCAN_THREADS / 64];
    __shared__ long long s_wave_excl[SCAN_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long base = (long long)tile * SCAN_TILE;

    // Sum of all earlier tiles: from their sums, or (no sums: a short input whose
    // first launch was left out) from the lengths themselves.
    long long before = 0;
    if (tile_sums) {
        for (int j = tid; j < tile; j += SCAN_THREADS) before += tile_sums[j];
    } else {
        // base is a multiple of SCAN_TILE: SCAN_ITEMS loads per thread and tile, all in flight together
        for (long long k0 = 0; k0 < base; k0 += SCAN_TILE) {
            int v[SCAN_ITEMS];
#pragma unroll
            for (int i = 0; i < SCAN_ITEMS; ++i) v[i] = len[k0 + i * SCAN_THREADS + tid];
#pragma unroll
            for (int i = 0; i < SCAN_ITEMS; ++i) before += v[i] > 0 ? v[i] : 0;
        }
    }
    before = block_sum(before, s_w);

    // Coalesced load of this tile; negative lengths count as 0.
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        const int p = i * SCAN_THREADS + tid;
        const long long k = base + p;
        int v = 0;
        if (k < n) v = len[k];
        if (v < 0) {
            atomicMin(&err->first_bad_len, (unsigned long long)k);
            atomicOr(&err->flags, ERR_NEG_LENGTH);
        }
        s_tile[p + (p >> 5)] = v > 0 ? v : 0;
    }
    __syncthreads();

    // Each thread owns SCAN_ITEMS consecutive entries.
    int mine[SCAN_ITEMS];
    long long tsum = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        const int p = tid * SCAN_ITEMS + i;
        mine[i] = s_tile[p + (p >> 5)];
        tsum += mine[i];
    }
    // Inclusive scan of the thread sums inside the wave, then across waves.
    long long incl = tsum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const long long up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    if (tid == 0) {
        long long run = 0;
#pragma unroll
        for (int w = 0; w < SCAN_THREADS / 64; ++w) {
            s_wave_excl[w] = run;
            run += s_w[w];
        }
    }
    __syncthreads();
    long long run = before + s_wave_excl[wave] + (incl - tsum);
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        const int p = tid * SCAN_ITEMS + i;
        // Clamping to nnz keeps every bag inside the ids the caller passed.
        s_tile[p + (p >> 5)] = (int)(run < nnz ? run : nnz);
        run += mine[i];
    }
    // `run` of the thread owning the last valid entry is the grand total.
    const long long last = (long long)n - 1 - base;
    if (last >= 0 && last < SCAN_TILE && tid == (int)(last / SCAN_ITEMS)) {
        long long total = before + s_wave_excl[wave] + (incl - tsum);
        for (int i = 0; i <= (int)(last % SCAN_ITEMS); ++i) total += mine[i];
        offsets[n] = (int)(total < nnz ? total : nnz);
        if (total != nnz) atomicOr(&err->flags, ERR_TOTAL_MISMATCH);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        const int p = i * SCAN_THREADS + tid;
        const long long k = base + p;
        if (k < n) offsets[k] = s_tile[p + (p >> 5)];
    }
}

// Second launch of the scan: blocks [0, tiles) write the offsets, the blocks
// behind them do a concatenation model's dense copy.
__global__ __launch_bounds__(SCAN_THREADS) void scan_tile_offsets(const int32_t *__restrict__ len,
                                                                  int n, long long nnz,
                                                                  const long long *__restrict__ tile_sums,
                                                                  int32_t *__restrict__ offsets,
                                                                  ErrRecord *err, int tiles,
                                                                  const ConcatDense job)
{
    if ((int)blockIdx.x < tiles)
        scan_offsets_tile(len, n, nnz, tile_sums, offsets, err, blockIdx.x);
    else
        concat_dense_block(job, blockIdx.x - tiles, gridDim.x - tiles);
}

// The same with a stack of fully connected layers riding along: blocks of
// chain::CH_THREADS threads; behind the scan's and the copy's blocks come
// chain_grid_x blocks that each take chain::CH_ROWS samples through the stack.
// A scan block uses its first SCAN_THREADS threads; the waves of the others end
// at once (a barrier counts only the waves of a group that have not ended).
__global__ __launch_bounds__(chain::CH_THREADS) void scan_offsets_ride_kernel(
    const int32_t *__restrict__ len, int n, long long nnz, const long long *__restrict__ tile_sums,
    int32_t *__restrict__ offsets, ErrRecord *err, int tiles, const ConcatDense job, int extra,
    const ChainProblem a, int chain_grid_x)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int b = blockIdx.x;
    if (b < tiles) {
        if (threadIdx.x < SCAN_THREADS) scan_offsets_tile(len, n, nnz, tile_sums, offsets, err, b);
    } else if (b < tiles + extra) {
        concat_dense_block(job, b - tiles, extra);
    } else {
        chain::mlp_chain_block<true>(a, smem, b - tiles - extra, 0, chain_grid_x);
    }
}

}  // namespace

hipError_t launch_clear_err(ErrRecord *err, hipStream_t s)
{
    hipLaunchKernelGGL(clear_err_kernel, dim3(1), dim3(64), 0, s, err);
    return hipGetLastError();
}

hipError_t scan_prepare()
{
    const int most = (int)chain::chain_lds_bytes(CHAIN_MAX_WIDTH + chain::CH_LDS_PAD);
    return hipFuncSetAttribute(reinterpret_cast<const void *>(scan_offsets_ride_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, most);
}

hipError_t launch_scan(const int32_t *lengths, int n, long long nnz, int32_t *offsets,
                       long long *block_sums, ErrRecord *err, const ConcatDense &job,
                       const ChainProblem *rider, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    int extra = 0;
    if (job.x0) {
        const long long total = (long long)job.B * (job.w0 + job.ldz - job.width);
        extra = (int)std::min<long long>((total + 8 * SCAN_THREADS - 1) / (8 * SCAN_THREADS), 256);
    }
    // With a stack riding along the second launch lasts as long as the stack, so
    // for a few tiles its scan blocks have the time to add up the earlier lengths
    // themselves and the first launch can go (alone, that was measured no faster
    // than two launches at 5 tiles and slower beyond).
    const bool has_rider = rider && rider->M > 0;
    const long long *sums = has_rider && tiles <= 8 ? nullptr : block_sums;
    if (tiles > 1 && sums) {
        hipLaunchKernelGGL(scan_tile_sums, dim3(tiles), dim3(SCAN_THREADS), 0, s, lengths, n,
                           block_sums);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (has_rider) {
        if (!rider->a_f32 || rider->groups != 1) return hipErrorInvalidValue;
        ChainProblem a;
        const hipError_t e = chain_finalize(*rider, a);
        if (e != hipSuccess) return e;
        const int chain_grid_x = (a.M + chain::CH_ROWS - 1) / chain::CH_ROWS;
        hipLaunchKernelGGL(scan_offsets_ride_kernel, dim3(tiles + extra + chain_grid_x),
                           dim3(chain::CH_THREADS), chain::chain_lds_bytes(a.ld_lds), s, lengths, n, nnz, sums,
                           offsets, err, tiles, job, extra, a, chain_grid_x);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(scan_tile_offsets, dim3(tiles + extra), dim3(SCAN_THREADS), 0, s, lengths, n, nnz,
                       sums, offsets, err, tiles, job);
    return hipGetLastError();
}

}  // namespace rec
