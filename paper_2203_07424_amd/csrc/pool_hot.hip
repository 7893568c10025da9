// S1 with a software-managed cache of hot rows in LDS.
//
// Embedding accesses have strong temporal locality, and the paper's partition
// stage ranks rows by access frequency to form hot embedding tables (Sec. IV-A,
// locality-aware embedding partition).  Here the hot rows of a table - a list
// the caller registers per table - are copied into LDS by every block that
// works on that table, together with a small open-addressing hash of their
// ids.  Each wave then splits the ids of its bag into a cold list and a hot
// list (wave ballot + prefix count, both lists in LDS): cold rows are gathered
// from memory exactly as in the plain kernel, hot rows come from LDS and never
// reach the L1's miss queue, which is what bounds the plain kernel on skewed
// ids.  Same sums; the order of accumulation (cold rows first, then hot rows)
// is fixed, so results are reproducible.
//
// Blocks own contiguous runs of the table-major bag list (XCD-aware, as in the
// plain kernel), so a block rebuilds its cache at most once per table boundary
// inside its run.
#include "rec_internal.h"

namespace rec {

namespace {

constexpr int PH_WAVES = 4;     // waves per block
constexpr int PH_THREADS = PH_WAVES * 64;
constexpr int PH_SEG = 128;     // ids split into cold / hot per pass
constexpr int PH_UNROLL = 4;    // cold row loads in flight per lane
constexpr int PH_EMPTY = -1;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// One more row into the sums; a row that does not count is cleared as raw bits
// first.  `one` is 1.0f held in a register: the product form lets each fp16
// element be widened and added by a single mixed-precision fused multiply-add
// (bit-identical to widening and adding, the product being exact).
template <bool HALF>
__device__ inline void add_row(float *acc, u32x4 raw, bool ok, float one)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) raw[i] = ok ? raw[i] : 0u;
    if (HALF) {
        const f16x8 h = __builtin_bit_cast(f16x8, raw);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf((float)h[i], one, acc[i]);
    } else {
        const f32x4 f = __builtin_bit_cast(f32x4, raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += f[i];
    }
}

// Multiplicative hashing, top bits: ids that form an arithmetic progression
// (popular ranks pushed through an affine permutation do) spread evenly.
__device__ inline unsigned hash_id(int id, int log2_slots)
{
    return ((unsigned)id * 2654435761u) >> (32 - log2_slots);
}

template <int LPR, bool HALF>
__global__ __launch_bounds__(PH_THREADS) void pool_hot_kernel(
    const TableDesc *__restrict__ tables, const int32_t *__restrict__ indices,
    const int32_t *__restrict__ offsets, float *__restrict__ pooled, int B, int T, int nbags,
    int bags_per_block, int hcap, float one, ErrRecord *err)
{
    typedef const __attribute__((address_space(1))) char *table_ptr;
    typedef const __attribute__((address_space(1))) u32x4 *row_ptr;
    constexpr int RPW = 64 / LPR;
    constexpr int ROWBYTES = LPR * 16;
    constexpr int NACC = HALF ? 8 : 4;
    constexpr int D = ROWBYTES / (HALF ? 2 : 4);

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int HS = 4 * hcap;  // hash slots (load factor <= 1/4), a power of two
    const int log2_hs = 31 - __builtin_clz(HS);
    unsigned char *s_rows = smem;                                       // [hcap][ROWBYTES]
    int *s_key = reinterpret_cast<int *>(smem + (size_t)hcap * ROWBYTES);  // [HS]
    int *s_slot = s_key + HS;                                           // [HS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int *my_cold = s_slot + HS + wave * 2 * PH_SEG;                     // [PH_SEG] row ids
    int *my_hot = my_cold + PH_SEG;                                     // [PH_SEG] cache slots

    const int sub = lane / LPR, chunk = lane % LPR;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    // The grid is a multiple of 8 blocks; XCD x gets the x-th eighth of the runs.
    const int per = gridDim.x >> 3;
    const long long vblk = (long long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
    long long p0 = vblk * bags_per_block;
    const long long last = p0 + bags_per_block < nbags ? p0 + bags_per_block : nbags;

    while (p0 < last) {  // one pass per table the run touches (block-uniform)
        const int t = (int)(p0 / B);
        const long long table_end = (long long)(t + 1) * B;
        const long long pend = last < table_end ? last : table_end;
        const char *base = static_cast<const char *>(tables[t].base);
        const long long rows = tables[t].rows;
        const int32_t *hot_ids = tables[t].hot_ids;
        const int nh = tables[t].n_hot < hcap ? tables[t].n_hot : hcap;

        // ---- (re)build the cache: hash of ids, then the rows themselves
        __syncthreads();
        for (int i = tid; i < HS; i += PH_THREADS) s_key[i] = PH_EMPTY;
        __syncthreads();
        for (int i = tid; i < nh; i += PH_THREADS) {
            const int id = hot_ids[i];
            if ((unsigned long long)(long long)id < (unsigned long long)rows) {
                unsigned h = hash_id(id, log2_hs);
                for (int probe = 0; probe < HS; ++probe) {  // load factor <= 1/4: ends early
                    const int old = atomicCAS(&s_key[h], PH_EMPTY, id);
                    if (old == PH_EMPTY) { s_slot[h] = i; break; }
                    if (old == id) break;  // listed twice: the first copy serves
                    h = (h + 1) & (HS - 1);
                }
            }
        }
        for (int e = tid; e < nh * LPR; e += PH_THREADS) {
            const int i = e / LPR, c = e - i * LPR;
            const int id = hot_ids[i];
            if ((unsigned long long)(long long)id < (unsigned long long)rows)
                *reinterpret_cast<f32x4 *>(s_rows + (size_t)i * ROWBYTES + c * 16) =
                    *reinterpret_cast<const f32x4 *>(base + (long long)id * ROWBYTES + c * 16);
        }
        __syncthreads();

        // ---- the bags of this pass, one per wave at a time
        const table_ptr lane_base = (table_ptr)base + chunk * 16;
        for (long long bag = p0 + wave; bag < pend; bag += PH_WAVES) {
            const int b = (int)(bag - (long long)t * B);
            const int start = __builtin_amdgcn_readfirstlane(offsets[bag]);
            const int end = __builtin_amdgcn_readfirstlane(offsets[bag + 1]);
            float acc[NACC];
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = 0.0f;

            for (int seg = start; seg < end; seg += PH_SEG) {
                const int nseg = min(PH_SEG, end - seg);
                int ncold = 0, nhot = 0;
                // All ids of the pass are requested before the first one is looked up.
                int seg_ids[PH_SEG / 64];
#pragma unroll
                for (int c = 0; c < PH_SEG / 64; ++c) {
                    const int pos = c * 64 + lane;
                    seg_ids[c] = pos < nseg ? indices[seg + pos] : 0;
                }
#pragma unroll
                for (int c = 0; c < PH_SEG / 64; ++c) {
                    const int pos = c * 64 + lane;
                    bool valid = pos < nseg;
                    const int id = seg_ids[c];
                    if (valid && (unsigned long long)(long long)id >= (unsigned long long)rows) {
                        atomicMin(&err->first_bad_idx, (unsigned long long)(seg + pos));
                        atomicOr(&err->flags, ERR_INDEX_RANGE);
                        valid = false;
                    }
                    int slot = -1;
                    if (valid) {
                        unsigned h = hash_id(id, log2_hs);
                        for (int probe = 0; probe < HS; ++probe) {
                            const int k = s_key[h];
                            if (k == id) { slot = s_slot[h]; break; }
                            if (k == PH_EMPTY) break;
                            h = (h + 1) & (HS - 1);
                        }
                    }
                    const bool is_cold = valid && slot < 0, is_hot = valid && slot >= 0;
                    const unsigned long long cm = __ballot(is_cold), hm = __ballot(is_hot);
                    if (is_cold) my_cold[ncold + __popcll(cm & lt_mask)] = id;
                    if (is_hot) my_hot[nhot + __popcll(hm & lt_mask)] = slot;
                    ncold += __popcll(cm);
                    nhot += __popcll(hm);
                }
                __builtin_amdgcn_wave_barrier();

                // cold rows: from memory, PH_UNROLL wave-wide loads in flight
                const int csteps = (ncold + RPW - 1) / RPW;
                for (int j = 0; j < csteps; j += PH_UNROLL) {
                    u32x4 raw[PH_UNROLL];
                    bool ok[PH_UNROLL];
#pragma unroll
                    for (int u = 0; u < PH_UNROLL; ++u) {
                        const int p = (j + u) * RPW + sub;
                        const int id = my_cold[p < PH_SEG ? p : PH_SEG - 1];
                        ok[u] = p < ncold;
                        const long long row = ok[u] ? id : 0;
                        raw[u] = *(row_ptr)(lane_base + row * ROWBYTES);
                    }
#pragma unroll
                    for (int u = 0; u < PH_UNROLL; ++u) add_row<HALF>(acc, raw[u], ok[u], one);
                }
                // hot rows: from the LDS copy
                const int hsteps = (nhot + RPW - 1) / RPW;
                for (int j = 0; j < hsteps; ++j) {
                    const int p = j * RPW + sub;
                    const bool ok = p < nhot;
                    const int slot = ok ? my_hot[p < PH_SEG ? p : PH_SEG - 1] : 0;
                    const u32x4 raw =
                        *reinterpret_cast<const u32x4 *>(s_rows + (size_t)slot * ROWBYTES + chunk * 16);
                    add_row<HALF>(acc, raw, ok, one);
                }
                __builtin_amdgcn_wave_barrier();
            }

            // Fold the RPW partial sums: lanes l and l ^ m hold the same columns.
#pragma unroll
            for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
                for (int i = 0; i < NACC; ++i) acc[i] += __shfl_xor(acc[i], m, 64);
            }
            if (sub == 0) {
                float *out = pooled + ((long long)b * T + t) * D + chunk * NACC;
#pragma unroll
                for (int i = 0; i < NACC; i += 4) {
                    f32x4 o = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
                    *reinterpret_cast<f32x4 *>(out + i) = o;
                }
            }
        }
        p0 = pend;
    }
}

size_t hot_lds_bytes(int hcap, int rowbytes)
{
    return (size_t)hcap * rowbytes + sizeof(int) * (8 * (size_t)hcap + PH_WAVES * 2 * PH_SEG);
}

template <int LPR>
hipError_t launch_lpr(bool half, const TableDesc *tables, int T, int B, const int32_t *indices,
                      const int32_t *offsets, float *pooled, int hcap, int num_cus, ErrRecord *err,
                      hipStream_t s)
{
    const int nbags = T * B;
    const size_t lds = hot_lds_bytes(hcap, LPR * 16);
    // Runs are dealt out once, so every block must be resident from the start:
    // ask the runtime how many fit a CU with this much LDS and these registers.
    int per_cu = 0;
    const hipError_t oe =
        half ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pool_hot_kernel<LPR, true>, PH_THREADS, lds)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pool_hot_kernel<LPR, false>, PH_THREADS, lds);
    if (oe != hipSuccess) return oe;
    per_cu = per_cu < 1 ? 1 : per_cu;
    int blocks = num_cus * per_cu / 8 * 8;
    int bpb = (nbags + blocks - 1) / blocks;
    if (bpb < 16) bpb = 16;  // a cache build must serve a few bags
    blocks = ((nbags + bpb - 1) / bpb + 7) / 8 * 8;
    const dim3 grid(blocks), block(PH_THREADS);
    if (half)
        hipLaunchKernelGGL((pool_hot_kernel<LPR, true>), grid, block, lds, s, tables, indices, offsets,
                           pooled, B, T, nbags, bpb, hcap, 1.0f, err);
    else
        hipLaunchKernelGGL((pool_hot_kernel<LPR, false>), grid, block, lds, s, tables, indices, offsets,
                           pooled, B, T, nbags, bpb, hcap, 1.0f, err);
    return hipGetLastError();
}

}  // namespace

bool pool_hot_fits(int hcap, int rowbytes) { return hot_lds_bytes(hcap, rowbytes) <= 64 * 1024; }

hipError_t launch_pool_hot(const TableDesc *tables, int dtype, int T, int D, int B,
                           const int32_t *indices, const int32_t *offsets, float *pooled, int hcap,
                           int num_cus, ErrRecord *err, hipStream_t s)
{
    if (T <= 0 || B <= 0) return hipSuccess;
    const bool half = dtype == REC_F16;
    const int rowbytes = D * (half ? 2 : 4);
    if (!pool_hot_fits(hcap, rowbytes) || (hcap & (hcap - 1)) != 0) return hipErrorInvalidValue;
    switch (rowbytes / 16) {
    case 1: return launch_lpr<1>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 2: return launch_lpr<2>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 4: return launch_lpr<4>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 8: return launch_lpr<8>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 16: return launch_lpr<16>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 32: return launch_lpr<32>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    case 64: return launch_lpr<64>(half, tables, T, B, indices, offsets, pooled, hcap, num_cus, err, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace rec
