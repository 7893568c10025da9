// S1: embedding-bag pooling (SparseLengthsSum; "Gather-Reduce", Sec. VI-B).
//
// pooled[b][t][:] = sum of rows E_t[id][:] over the ids of bag (t, b).
//
// One 64-lane wavefront per bag.  A row is D * sizeof(element) bytes; a lane
// moves 16 bytes (one 128-bit load), so LPR = rowbytes / 16 lanes cover a row
// and one wave-wide load fetches RPW = 64 / LPR different rows of the bag.
// The wave reads 64 ids with one coalesced load, hands them out by cross-lane
// permute, keeps several row loads in flight, accumulates in fp32 and folds the
// RPW partial sums in a fixed order, so results do not vary from run to run.
//
// The work is random-gather traffic, but a wave64 vector instruction holds its
// SIMD for four cycles, and a version that spent some 33 vector instructions
// per wave-wide load (address arithmetic, validity selects, widen + select +
// add per element) was bound by instruction issue even with every row in the
// L1.  Per wave-wide load the loop below spends one permute, one add, the load
// and one fused multiply-add per element: rows come through a buffer descriptor
// whose range check returns zero for the offsets that stand for "no row", the
// permute's slot is an immediate, and loads a partial group does not need are
// skipped by wave-uniform branches.
//
// Bags of a few ids (one lookup per table and no pooling, Table I row MT-WnD)
// would leave most of such a wave idle: pool_short_kernel gives each group of
// LPR lanes a bag of its own, RPW bags per wave.  (Giving bags of 20-50 ids, the
// DLRM-RMC3 range of Table I, 4 * LPR lanes each was measured too: slower than
// one wave per bag.)
//
// STREAM: the rows are loaded with the non-temporal hint (they are not kept in
// the caches ahead of other lines).  For id streams without reuse (uniform ids)
// that is 2.5 % faster; for skewed ids, whose hot rows the caches serve, it is
// 20 % slower, so it is an option the caller sets from what it knows of its ids.
//
// In the concatenation model the sums go, narrowed to bf16, straight into the
// Predict-FC input row of their sample (concatenation and conversion fused,
// Sec. IV-A) instead of the fp32 pooled buffer.
#include <hip/hip_fp16.h>

#include "rec_internal.h"

namespace rec {

namespace {

// Both were swept on the RMC2-style workload (2..8 loads, 2..8 waves); these are the best.
constexpr int POOL_WAVES = 4;   // bags per block
constexpr int POOL_UNROLL = 4;  // row loads in flight per lane and step

constexpr int SHORT_UNROLL = 4;  // row loads in flight per lane in the short-bag kernel
constexpr int SHORT_BAGS = 2;    // bags a group of lanes works on at a time
constexpr int SHORT_MEAN = 4;    // mean ids per bag up to which bags share a wave

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <bool HALF>
struct Acc {
    static constexpr int N = HALF ? 8 : 4;
    float v[N];
};

// One more row into the sums.  `one` is 1.0f held in a register: the product
// form lets each fp16 element be widened, and added, by a single mixed-precision
// fused multiply-add (bit-identical to widening and adding, the product being exact).
template <bool HALF>
__device__ inline void accumulate(Acc<HALF> &a, const u32x4 raw, float one)
{
    if (HALF) {
        const f16x8 h = __builtin_bit_cast(f16x8, raw);
#pragma unroll
        for (int i = 0; i < 8; ++i) a.v[i] = __builtin_fmaf((float)h[i], one, a.v[i]);
    } else {
        const f32x4 f = __builtin_bit_cast(f32x4, raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) a.v[i] += f[i];
    }
}

// Rows of one table, 16 bytes per lane.  NARROW (table smaller than 4 GiB): a
// buffer descriptor over the table and 32-bit byte offsets; an offset past the
// table reads as zero, which is how ids marked invalid (key 0xFFFFFFFF..) add
// nothing.  Otherwise 64-bit addresses, invalid keys masked by hand.
template <int ROWBYTES, bool NARROW, bool STREAM>
struct RowSource {
    __amdgpu_buffer_rsrc_t rsrc;
    const __attribute__((address_space(1))) char *lane_base;
    unsigned lane_off;

    __device__ inline RowSource(const void *base, long long rows, int chunk)
    {
        lane_off = chunk * 16;
        if (NARROW)
            rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0,
                                                     (int)(unsigned)(rows * ROWBYTES), 0x00020000);
        else
            lane_base = (const __attribute__((address_space(1))) char *)base + chunk * 16;
    }
    // What a lane hands out for id (id < 0: invalid).
    __device__ static inline unsigned key(int id) { return NARROW ? (unsigned)id * ROWBYTES : (unsigned)id; }
    __device__ inline u32x4 fetch(unsigned k) const
    {
        if (NARROW) return __builtin_amdgcn_raw_buffer_load_b128(rsrc, k + lane_off, 0, STREAM ? 2 : 0);
        const bool ok = (int)k >= 0;
        typedef const __attribute__((address_space(1))) u32x4 *row_ptr;
        const row_ptr src = (row_ptr)(lane_base + (unsigned long long)(ok ? k : 0u) * ROWBYTES);
        u32x4 v = STREAM ? __builtin_nontemporal_load(src) : *src;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = ok ? v[i] : 0u;
        return v;
    }
};

// The NACC sums a lane holds (columns chunk * NACC ... of bag (t, b)) to where they belong.
template <bool HALF, bool CONCAT>
__device__ inline void store_sums(const Acc<HALF> &acc, const PoolOut &out, int vec_ok, int b, int t,
                                  int T, int D, int chunk)
{
    constexpr int NACC = HALF ? 8 : 4;
    if (CONCAT) {
        __bf16 *o = static_cast<__bf16 *>(out.z) + (long long)b * out.ldz + out.col0 + t * D + chunk * NACC;
        if (vec_ok) {
            if (HALF) {
                bf16x8 v;
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = (__bf16)acc.v[i];
                *reinterpret_cast<bf16x8 *>(o) = v;
            } else {
                bf16x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (__bf16)acc.v[i];
                *reinterpret_cast<bf16x4 *>(o) = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < NACC; ++i) o[i] = (__bf16)acc.v[i];
        }
    } else {
        float *o = out.pooled + ((long long)b * T + t) * D + chunk * NACC;
#pragma unroll
        for (int i = 0; i < NACC; i += 4) {
            f32x4 v = {acc.v[i], acc.v[i + 1], acc.v[i + 2], acc.v[i + 3]};
            *reinterpret_cast<f32x4 *>(o + i) = v;
        }
    }
}

template <int LPR, bool HALF, bool CONCAT, bool STREAM, bool NARROW>
__global__ __launch_bounds__(POOL_WAVES * 64) void pool_kernel(
    const TableDesc *__restrict__ tables, const int32_t *__restrict__ indices,
    const int32_t *__restrict__ offsets, const PoolOut out, int vec_ok, int B, int T, int nbags,
    float one, ErrRecord *err)
{
    constexpr int RPW = 64 / LPR;
    constexpr int ROWBYTES = LPR * 16;
    constexpr int NACC = HALF ? 8 : 4;
    constexpr int D = ROWBYTES / (HALF ? 2 : 4);
    typedef RowSource<ROWBYTES, NARROW, STREAM> Rows;

    const int lane = threadIdx.x & 63;
    // Blocks are handed to the 8 XCDs round-robin; give XCD x the x-th eighth
    // of the (table-major) bag list so that each L2 sees few tables at a time.
    // The grid is a multiple of 8 blocks; surplus blocks fall past nbags.
    const int per = gridDim.x >> 3;
    const int vblk = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    int bag = vblk * POOL_WAVES + (threadIdx.x >> 6);
    if (bag >= nbags) return;
    bag = __builtin_amdgcn_readfirstlane(bag);
    const int t = bag / B;
    const int b = bag - t * B;
    const int start = offsets[bag];
    const int end = offsets[bag + 1];
    const long long rows = tables[t].rows;

    const int sub = lane / LPR;  // which of the RPW rows of a wave-wide load
    const int chunk = lane % LPR;
    const Rows src(tables[t].base, rows, chunk);

    Acc<HALF> acc;
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc.v[i] = 0.0f;

    int ids = -1;
    if (start + lane < end) ids = indices[start + lane];
    for (int k0 = start; k0 < end; k0 += 64) {
        const int n = min(64, end - k0);
        int cur = ids;  // -1 in the lanes past the end of the bag
        // Ids outside the table contribute zero and leave a record.
        if (lane < n && (unsigned long long)(long long)cur >= (unsigned long long)rows) {
            atomicMin(&err->first_bad_idx, (unsigned long long)(k0 + lane));
            atomicOr(&err->flags, ERR_INDEX_RANGE);
            cur = -1;
        }
        const unsigned key = Rows::key(cur);
        // Next 64 ids, requested before the row loads of this step.
        ids = -1;
        if (k0 + 64 + lane < end) ids = indices[k0 + 64 + lane];

        const int steps = (n + RPW - 1) / RPW;  // wave-wide loads this chunk needs
        // slot4: byte address of this lane's slot in the cross-lane permute (the
        // hardware takes it modulo the wave).
        int j = 0;
        for (; j + POOL_UNROLL <= steps; j += POOL_UNROLL) {
            const int slot4 = (j * RPW + sub) * 4;
            u32x4 raw[POOL_UNROLL];
#pragma unroll
            for (int u = 0; u < POOL_UNROLL; ++u)
                raw[u] = src.fetch(__builtin_amdgcn_ds_bpermute(slot4 + u * RPW * 4, key));
#pragma unroll
            for (int u = 0; u < POOL_UNROLL; ++u) accumulate<HALF>(acc, raw[u], one);
        }
        if (j < steps) {  // the last, partial group: loads it does not need are not issued
            const int slot4 = (j * RPW + sub) * 4;
            u32x4 raw[POOL_UNROLL - 1];
#pragma unroll
            for (int u = 0; u < POOL_UNROLL - 1; ++u)
                if (j + u < steps) raw[u] = src.fetch(__builtin_amdgcn_ds_bpermute(slot4 + u * RPW * 4, key));
#pragma unroll
            for (int u = 0; u < POOL_UNROLL - 1; ++u)
                if (j + u < steps) accumulate<HALF>(acc, raw[u], one);
        }
    }

    // Fold the RPW partial sums: lanes l and l ^ m hold the same columns.
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc.v[i] += __shfl_xor(acc.v[i], m, 64);
    }
    if (sub == 0) store_sums<HALF, CONCAT>(acc, out, vec_ok, b, t, T, D, chunk);
}

// SHORT_BAGS bags per group of LPR lanes, their load chains (offsets -> ids ->
// rows) running side by side; group g of the launch takes bags g, g + groups,
// ...  Slots past the last bag work on a copy of it and store nothing.
template <int LPR, bool HALF, bool CONCAT>
__global__ __launch_bounds__(POOL_WAVES * 64) void pool_short_kernel(
    const TableDesc *__restrict__ tables, const int32_t *__restrict__ indices,
    const int32_t *__restrict__ offsets, const PoolOut out, int vec_ok, int B, int T, int nbags,
    int groups, float one, ErrRecord *err)
{
    typedef const __attribute__((address_space(1))) char *table_ptr;
    typedef const __attribute__((address_space(1))) u32x4 *row_ptr;
    constexpr int RPW = 64 / LPR;
    constexpr int ROWBYTES = LPR * 16;
    constexpr int NACC = HALF ? 8 : 4;
    constexpr int D = ROWBYTES / (HALF ? 2 : 4);
    constexpr int PER_BAG = SHORT_UNROLL / SHORT_BAGS;  // row loads in flight per bag

    const int lane = threadIdx.x & 63;
    const int sub = lane / LPR, chunk = lane % LPR;
    const int per = gridDim.x >> 3;
    const int vblk = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    const long long group = ((long long)vblk * POOL_WAVES + (threadIdx.x >> 6)) * RPW + sub;

    bool live[SHORT_BAGS];
    int t[SHORT_BAGS], b[SHORT_BAGS], pos[SHORT_BAGS], end[SHORT_BAGS];
    table_ptr lane_base[SHORT_BAGS];
    long long rows[SHORT_BAGS];
    Acc<HALF> acc[SHORT_BAGS];
#pragma unroll
    for (int g = 0; g < SHORT_BAGS; ++g) {
        const long long slot = group + (long long)g * groups;
        live[g] = slot < nbags;
        const int bag = live[g] ? (int)slot : nbags - 1;
        t[g] = bag / B;
        b[g] = bag - t[g] * B;
        pos[g] = offsets[bag];
        end[g] = live[g] ? offsets[bag + 1] : pos[g];
        lane_base[g] = (table_ptr)tables[t[g]].base + chunk * 16;
        rows[g] = tables[t[g]].rows;
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[g].v[i] = 0.0f;
    }

    bool more = false;
#pragma unroll
    for (int g = 0; g < SHORT_BAGS; ++g) more |= pos[g] < end[g];
    while (more) {
        u32x4 raw[SHORT_BAGS][PER_BAG];
#pragma unroll
        for (int g = 0; g < SHORT_BAGS; ++g) {
#pragma unroll
            for (int u = 0; u < PER_BAG; ++u) {
                const int k = pos[g] + u;
                bool ok = k < end[g];
                // positions past the bag re-read its last id (or, for an empty bag, nothing: id 0)
                const int kk = ok ? k : (end[g] > 0 ? end[g] - 1 : 0);
                const int id = pos[g] < end[g] ? indices[kk] : 0;
                if (ok && (unsigned long long)(long long)id >= (unsigned long long)rows[g]) {
                    if (chunk == 0) {
                        atomicMin(&err->first_bad_idx, (unsigned long long)k);
                        atomicOr(&err->flags, ERR_INDEX_RANGE);
                    }
                    ok = false;
                }
                const long long row = ok ? id : 0;
                u32x4 v = *(row_ptr)(lane_base[g] + row * ROWBYTES);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = ok ? v[i] : 0u;
                raw[g][u] = v;
            }
        }
        more = false;
#pragma unroll
        for (int g = 0; g < SHORT_BAGS; ++g) {
#pragma unroll
            for (int u = 0; u < PER_BAG; ++u) accumulate<HALF>(acc[g], raw[g][u], one);
            pos[g] = min(pos[g] + PER_BAG, end[g]);
            more |= pos[g] < end[g];
        }
    }
#pragma unroll
    for (int g = 0; g < SHORT_BAGS; ++g)
        if (live[g]) store_sums<HALF, CONCAT>(acc[g], out, vec_ok, b[g], t[g], T, D, chunk);
}

template <int LPR, bool HALF, bool CONCAT>
hipError_t launch_shape(bool short_bags, bool stream_rows, bool narrow, const TableDesc *tables, int T, int B, const int32_t *indices,
                        const int32_t *offsets, const PoolOut &out, ErrRecord *err, hipStream_t s)
{
    constexpr int NACC = HALF ? 8 : 4;
    const int nbags = T * B;
    const int vec_ok = CONCAT && out.col0 % NACC == 0 && reinterpret_cast<uintptr_t>(out.z) % 16 == 0;
    const dim3 block(POOL_WAVES * 64);
    if (short_bags) {
        const int groups_per_block = POOL_WAVES * (64 / LPR);
        const int per_block = groups_per_block * SHORT_BAGS;
        const dim3 grid(((nbags + per_block - 1) / per_block + 7) / 8 * 8);
        const int groups = (int)grid.x * groups_per_block;
        hipLaunchKernelGGL((pool_short_kernel<LPR, HALF, CONCAT>), grid, block, 0, s, tables, indices,
                           offsets, out, vec_ok, B, T, nbags, groups, 1.0f, err);
    } else {
        const dim3 grid(((nbags + POOL_WAVES - 1) / POOL_WAVES + 7) / 8 * 8);
#define REC_POOL_LAUNCH(STREAM, NARROW)                                                                  \
    hipLaunchKernelGGL((pool_kernel<LPR, HALF, CONCAT, STREAM, NARROW>), grid, block, 0, s, tables, indices, \
                       offsets, out, vec_ok, B, T, nbags, 1.0f, err)
        if (stream_rows) {
            if (narrow) REC_POOL_LAUNCH(true, true); else REC_POOL_LAUNCH(true, false);
        } else {
            if (narrow) REC_POOL_LAUNCH(false, true); else REC_POOL_LAUNCH(false, false);
        }
#undef REC_POOL_LAUNCH
    }
    return hipGetLastError();
}

template <int LPR>
hipError_t launch_lpr(bool half, bool short_bags, bool stream_rows, bool narrow, const TableDesc *tables, int T, int B,
                      const int32_t *indices, const int32_t *offsets, const PoolOut &out, ErrRecord *err,
                      hipStream_t s)
{
    if (out.z) {
        if (half) return launch_shape<LPR, true, true>(short_bags, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
        return launch_shape<LPR, false, true>(short_bags, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    }
    if (half) return launch_shape<LPR, true, false>(short_bags, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    return launch_shape<LPR, false, false>(short_bags, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
}

}  // namespace

hipError_t launch_pool(const TableDesc *tables, int dtype, int T, int D, int B,
                       const int32_t *indices, const int32_t *offsets, PoolOut out, long long nnz,
                       bool stream_rows, long long max_rows, ErrRecord *err, hipStream_t s)
{
    if (T <= 0 || B <= 0) return hipSuccess;
    const bool half = dtype == REC_F16;
    const int rowbytes = D * (half ? 2 : 4);
    // 32-bit byte offsets reach every row, and leave room above the table for the
    // offsets that stand for "no row".
    const bool narrow = max_rows * rowbytes <= 0xFFFF0000ll;
    const bool sh = rowbytes < 1024 && nnz <= (long long)SHORT_MEAN * T * B;
    switch (rowbytes / 16) {
    case 1: return launch_lpr<1>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 2: return launch_lpr<2>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 4: return launch_lpr<4>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 8: return launch_lpr<8>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 16: return launch_lpr<16>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 32: return launch_lpr<32>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    case 64: return launch_lpr<64>(half, sh, stream_rows, narrow, tables, T, B, indices, offsets, out, err, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace rec
