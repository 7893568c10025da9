// C boundary of the forward pass: model bookkeeping on the host and the fixed
// launch sequence  scan -> pool -> Bottom-FC -> interaction -> Predict-FC
// (interaction = pairwise dots, or plain concatenation for the MT-WnD shape of
// Table I, whose Predict-FC is N towers run side by side).
// Bottom-FC does not depend on the SparseNet and Predict-FC waits for both
// (Sec. III-A); on one in-order stream that dependency is the launch order.
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "rec_internal.h"

using namespace rec;

// Scratch memory of rec_forward_static(): one copy per GPU the library runs on,
// held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress(); kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[REC_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Layer {
    int K = 0, N = 0, Kpad = 0, Npad = 0;
    const void *W = nullptr;      // bf16 [Npad][Kpad]; fp32 [Kpad] for the one-output layer
    const float *bias = nullptr;  // fp32 [Npad]
    bool dot = false;             // last Predict-FC layer: fp32 dot product, not a GEMM
    bool chain = false;           // narrow enough for the kernel that runs several layers on chip
    const void *Wc = nullptr;     // chain layers: the same weights in MFMA fragment order
    bool loaded = false;
    size_t w_bytes() const { return dot ? sizeof(float) * Kpad : 2 * (size_t)Npad * Kpad; }
    size_t chain_bytes() const { return chain ? 2 * (size_t)Npad * Kpad : 0; }
};

}  // namespace

// Where the parts of a forward's scratch memory sit inside one block of device
// memory (byte offsets; every part 256-byte aligned).  The error record and the
// table descriptors exist once; what one batch passes through (a frame) once
// up to four times.
constexpr int MAX_FRAMES = 4;
struct Frame {
    size_t off_offsets = 0, off_tile_sums = 0, off_pooled = 0, off_x0 = 0, off_act[3] = {0, 0, 0};
};
struct Carve {
    size_t off_err = 0, off_tables = 0, bytes = 0;
    Frame fr[MAX_FRAMES];
};

struct rec_model {
    int T = 0, D = 0, F = 0, dtype = REC_F32;
    int interaction = REC_INTERACT_DOT;
    int towers = 1, n_top = 0;  // top holds towers * n_top layers, tower-major
    int w0 = 0;                 // width of the dense part x0 of the Predict-FC input
    int z_width = 0;            // width of the Predict-FC input
    int max_batch = 0;
    long long max_nnz = 0;
    std::vector<long long> rows;
    long long max_rows = 0;  // of the largest table
    std::vector<Layer> bottom, top;
    std::vector<char> table_loaded;
    std::vector<TableDesc> desc;  // host copy of the device descriptors
    int num_cus = 256;

    Carve lay;               // carve-up of the bound workspace, sized for max_batch
    int z_ld = 0;            // padded width of the interaction output (act[0])
    int act_ld = 0;          // widest padded hidden activation row (elements), act[1], act[2]
    size_t act_row_bytes = 0;  // bytes of one activation row: bf16 everywhere, fp32 into the dot layer
    int x0_ld = 0;           // row stride of the Bottom-FC output in the workspace
    char *ws = nullptr;

    // Bottom-FC runs on a stream of the library's own, beside scan and pooling.
    bool overlap_dense = false;
    bool stream_rows = false;  // pooling loads rows with the non-temporal hint
    int fuse_mlp = 1;          // runs of narrow layers through the on-chip chain kernel: 0 never, 1 where it pays, 2 always
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;

    // Sparse-dense pipeline: a batch owns one of four frames of the workspace
    // until its logits are written.  Scan and Bottom-FC run on the caller's
    // stream, pooling on two streams in turn, interaction and Predict-FC on a
    // fourth; these events order them.
    bool pipeline = false;
    hipStream_t dense_stream = nullptr;              // the caller's choice, else `side`
    hipStream_t pool_stream[2] = {nullptr, nullptr}; // the caller's choice, else own_stream
    hipStream_t own_stream[2] = {nullptr, nullptr};
    hipEvent_t ev_scan[MAX_FRAMES] = {}, ev_bottom[MAX_FRAMES] = {}, ev_pool[MAX_FRAMES] = {}, ev_tail[MAX_FRAMES] = {};
    bool tail_pending[MAX_FRAMES] = {};  // Predict-FC of that frame's batch enqueued, not yet waited for
    int next_frame = 0, last_frame = 0;
    int pool_turn = 0;                   // which pooling stream takes the next batch

    // Stage timing: forward number i records into slot i % slots.
    std::vector<hipEvent_t> ev;  // slots * EV_PER_SLOT
    std::vector<char> slot_mode; // per slot: 1 recorded by a pipelined forward, 2 in order with Bottom-FC inside the scan's launch
    int slots = 0, period = 1;
    long long forwards = 0;      // forwards seen since profiling was switched on

    template <class P>
    P *at(size_t off) const { return reinterpret_cast<P *>(ws + off); }
};

namespace {

// Scratch layout of model m for batches of up to `batch` samples, with `frames`
// (1 or MAX_FRAMES) copies of the per-batch part.
Carve carve(const rec_model *m, int batch, int frames)
{
    const bool concat = m->interaction == REC_INTERACT_CONCAT;
    const size_t nb = (size_t)m->T * batch;
    Carve c;
    size_t o = 0;
    c.off_err = o;    o += align_up(sizeof(ErrRecord));
    c.off_tables = o; o += align_up(sizeof(TableDesc) * m->T);
    for (int f = 0; f < frames; ++f) {
        Frame &fr = c.fr[f];
        fr.off_offsets = o;   o += align_up(sizeof(int32_t) * (nb + 1));
        fr.off_tile_sums = o; o += align_up(sizeof(long long) * ((nb + SCAN_TILE - 1) / SCAN_TILE));
        fr.off_pooled = o;    o += concat ? 0 : align_up(sizeof(float) * nb * m->D);
        fr.off_x0 = o;        o += !m->bottom.empty() ? align_up(sizeof(float) * (size_t)batch * m->x0_ld) : 0;
        // act[0] holds the Predict-FC input (kept for inspection); the hidden
        // activations of both stacks alternate between act[1] and act[2].
        fr.off_act[0] = o; o += align_up(2 * (size_t)batch * m->z_ld);
        fr.off_act[1] = o; o += align_up((size_t)batch * m->act_row_bytes);
        fr.off_act[2] = o; o += align_up((size_t)batch * m->act_row_bytes);
    }
    for (int f = frames; f < MAX_FRAMES; ++f) c.fr[f] = c.fr[0];
    c.bytes = o;
    return c;
}

}  // namespace

namespace {

bool all_loaded(const rec_model *m)
{
    for (char c : m->table_loaded)
        if (!c) return false;
    for (const Layer &l : m->bottom)
        if (!l.loaded) return false;
    for (const Layer &l : m->top)
        if (!l.loaded) return false;
    return true;
}

Layer *find_layer(rec_model *m, int which, int layer)
{
    if (which == REC_BOTTOM) {
        if (layer < 0 || layer >= (int)m->bottom.size()) return nullptr;
        return &m->bottom[layer];
    }
    const int tower = which - REC_TOP;
    if (tower < 0 || tower >= m->towers || layer < 0 || layer >= m->n_top) return nullptr;
    return &m->top[(size_t)tower * m->n_top + layer];
}

}  // namespace

namespace {

// The buffers one forward passes through: pointers into a scratch block.
struct Bufs {
    ErrRecord *err;
    const TableDesc *tables;
    int32_t *offsets;
    long long *tile_sums;
    float *pooled;
    float *x0;      // Bottom-FC output (unused without a Bottom-FC)
    void *act[3];
};

Bufs bufs_at(char *base, const Carve &c, int frame)
{
    const Frame &f = c.fr[frame];
    Bufs b;
    b.err = reinterpret_cast<ErrRecord *>(base + c.off_err);
    b.tables = reinterpret_cast<const TableDesc *>(base + c.off_tables);
    b.offsets = reinterpret_cast<int32_t *>(base + f.off_offsets);
    b.tile_sums = reinterpret_cast<long long *>(base + f.off_tile_sums);
    b.pooled = reinterpret_cast<float *>(base + f.off_pooled);
    b.x0 = reinterpret_cast<float *>(base + f.off_x0);
    for (int i = 0; i < 3; ++i) b.act[i] = base + f.off_act[i];
    return b;
}

// Arguments of one forward.
struct Call {
    const float *dense;
    const int32_t *indices;
    const int32_t *lengths;
    int B;
    long long nnz;
    float *logits;
};

// Stage events of one timed forward (null: not timed).  Slot i of the array is
// recorded by mark(i); which events bracket which stage depends on where the
// stages were enqueued (stage_events()).
enum { EV_BEGIN = 0, EV_SCAN_END = 1, EV_POOL_END = 2, EV_BOTTOM_FIRST_END = 3, EV_BOTTOM_END = 4,
       EV_INTERACT_END = 5, EV_TOP_FIRST_END = 6, EV_END = 7, EV_BOTTOM_BEGIN = 8, EV_INTERACT_BEGIN = 9,
       EV_POOL_BEGIN = 10, EV_PER_SLOT = 11 };

inline hipError_t mark(hipEvent_t *ev, int which, hipStream_t s)
{
    return ev ? hipEventRecord(ev[which], s) : hipSuccess;
}

#define REC_TRY(call)                          \
    do {                                       \
        const hipError_t e_ = (call);          \
        if (e_ != hipSuccess) return e_;       \
    } while (0)

// A run of chain layers [i, j) of one or several stacks side by side, layer l of
// stack k being layers[k * per_stack + l].
void chain_run(const Layer *layers, int per_stack, int G, int i, int j, ChainProblem &c)
{
    c.n_layers = j - i;
    c.groups = G;
    c.K = layers[i].K;
    for (int l = i; l < j; ++l) {
        c.Kpad[l - i] = layers[l].Kpad;
        c.Npad[l - i] = layers[l].Npad;
        c.relu[l - i] = 1;
        for (int k = 0; k < G; ++k) {
            c.W[l - i][k] = layers[(size_t)k * per_stack + l].Wc;
            c.bias[l - i][k] = layers[(size_t)k * per_stack + l].bias;
        }
    }
}

// How far a chain that starts at layer i of n reaches (i: no chain here).  Every
// block of a chain streams all weights of its run, which costs more than the
// launches it saves once they no longer are a small fraction of a block's L1
// bandwidth over a launch time: left to itself (fuse_mlp == 1) the library
// chains runs of up to CHAIN_AUTO_BYTES of weights, and only where that saves
// a launch (dot_after: the one-output layer follows layer n - 1).
int chain_end(const rec_model *m, const Layer *layers, int i, int n, bool dot_after)
{
    constexpr size_t CHAIN_AUTO_BYTES = 256 * 1024;
    if (m->fuse_mlp == 0 || (m->pipeline && m->fuse_mlp == 1)) return i;
    int j = i;
    size_t bytes = 0;
    while (j < n && layers[j].chain && j - i < CHAIN_MAX_LAYERS) bytes += layers[j++].chain_bytes();
    if (m->fuse_mlp == 2 || j == i) return j;
    const int saved = (j - i - 1) + (dot_after && j == n && !fc_can_fuse_dot(layers[j - 1].Npad) ? 1 : 0);
    return bytes > CHAIN_AUTO_BYTES || saved < 1 ? i : j;
}

// S2: ReLU after every layer; the last one leaves fp32 for the interaction.
hipError_t enqueue_bottom(const rec_model *m, const Bufs &u, const Call &c, hipStream_t s, hipEvent_t *ev)
{
    const int n = (int)m->bottom.size();
    const Layer *layers = m->bottom.data();
    const void *A = c.dense;
    bool a_f32 = true;
    int lda = m->F, launches = 0;
    for (int i = 0; i < n;) {
        const int j = chain_end(m, layers, i, n, false);
        const int upto = j > i ? j : i + 1;
        const bool last = upto == n;
        void *C = last ? static_cast<void *>(u.x0) : u.act[1 + (launches & 1)];
        const int ldc = last ? m->x0_ld : m->act_ld;
        if (j > i) {
            ChainProblem cp{};
            cp.A = A; cp.a_f32 = a_f32; cp.lda = lda; cp.a_stride = 0; cp.M = c.B;
            chain_run(layers, n, 1, i, j, cp);
            cp.out_mode = last ? CHAIN_OUT_F32 : CHAIN_OUT_BF16;
            cp.C = C; cp.ldc = ldc; cp.c_stride = 0;
            REC_TRY(launch_mlp_chain(cp, s));
        } else {
            const Layer &l = layers[i];
            FcProblem p{};
            p.A = A; p.a_f32 = a_f32; p.lda = lda;
            p.M = c.B; p.relu = true; p.groups = 1; p.num_cus = m->num_cus; p.corun = m->pipeline;
            p.K = l.K; p.Kpad = l.Kpad; p.Npad = l.Npad;
            p.g.W[0] = l.W; p.g.bias[0] = l.bias;
            p.C = C; p.out_f32 = last; p.ldc = ldc;
            REC_TRY(launch_fc(p, s));
        }
        A = C; lda = ldc; a_f32 = false;
        if (launches++ == 0) REC_TRY(mark(ev, EV_BOTTOM_FIRST_END, s));  // the first launch is timed on its own
        i = upto;
    }
    if (launches == 0) REC_TRY(mark(ev, EV_BOTTOM_FIRST_END, s));
    return mark(ev, EV_BOTTOM_END, s);
}

// S0 and S1.  With hot lists registered (and use_hot), hot rows are served from
// LDS.  In the concatenation model the sums go straight into the Predict-FC
// input rows.
// A concatenation model without Bottom-FC has the dense part of its Predict-FC
// input rows written by spare blocks of the scan: one launch less in front of S4.
bool concat_rides_on_scan(const rec_model *m)
{
    return m->interaction == REC_INTERACT_CONCAT && m->bottom.empty();
}

// Bottom-FC does not depend on the sparse side (Sec. III-A): when the whole
// stack is one run of the on-chip kernel, an in-order forward lets it ride on
// the scan's second launch instead of giving it a launch of its own (9-11 us on
// every workload here, whatever its size).
bool bottom_rides_on_scan(const rec_model *m)
{
    const int n = (int)m->bottom.size();
    return n > 0 && !m->pipeline && !m->overlap_dense && chain_end(m, m->bottom.data(), 0, n, false) == n;
}

hipError_t enqueue_scan(const rec_model *m, const Bufs &u, const Call &c, hipStream_t s, bool with_bottom)
{
    ConcatDense job;
    if (concat_rides_on_scan(m)) {
        job.x0 = c.dense; job.ldx0 = m->F; job.w0 = m->w0; job.B = c.B;
        job.z_bf16 = u.act[0]; job.width = m->z_width; job.ldz = m->z_ld;
    }
    ChainProblem cp{};
    if (with_bottom) {
        const int n = (int)m->bottom.size();
        cp.A = c.dense; cp.a_f32 = true; cp.lda = m->F; cp.a_stride = 0; cp.M = c.B;
        chain_run(m->bottom.data(), n, 1, 0, n, cp);
        cp.out_mode = CHAIN_OUT_F32;
        cp.C = u.x0; cp.ldc = m->x0_ld; cp.c_stride = 0;
    }
    return launch_scan(c.lengths, m->T * c.B, c.nnz, u.offsets, u.tile_sums, u.err, job,
                       with_bottom ? &cp : nullptr, s);
}

hipError_t enqueue_pool(const rec_model *m, const Bufs &u, const Call &c, bool use_hot, hipStream_t s)
{
    const int B = c.B, T = m->T, D = m->D;
    const bool concat = m->interaction == REC_INTERACT_CONCAT;
    int hmax = 0;
    if (use_hot)
        for (const TableDesc &d : m->desc) hmax = d.n_hot > hmax ? d.n_hot : hmax;
    if (hmax > 0 && !concat) {
        // Capacity: at least the longest list; a sparse hash (128 slots of rows
        // or more, where LDS allows) keeps the per-wave probe chains short.
        const int rowbytes = D * (m->dtype == REC_F16 ? 2 : 4);
        int hcap = 16;
        while (hcap < hmax) hcap *= 2;
        while (hcap < 128 && pool_hot_fits(hcap * 2, rowbytes)) hcap *= 2;
        REC_TRY(launch_pool_hot(u.tables, m->dtype, T, D, B, c.indices, u.offsets, u.pooled, hcap,
                                m->num_cus, u.err, s));
    } else {
        const PoolOut out = concat ? PoolOut{nullptr, u.act[0], m->z_ld, m->w0}
                                   : PoolOut{u.pooled, nullptr, 0, 0};
        REC_TRY(launch_pool(u.tables, m->dtype, T, D, B, c.indices, u.offsets, out, c.nnz, m->stream_rows,
                            m->max_rows, u.err, s));
    }
    return hipSuccess;
}

hipError_t enqueue_sparse(const rec_model *m, const Bufs &u, const Call &c, bool use_hot, hipStream_t s,
                          hipEvent_t *ev, bool with_bottom = false)
{
    REC_TRY(enqueue_scan(m, u, c, s, with_bottom));
    REC_TRY(mark(ev, EV_SCAN_END, s));
    REC_TRY(enqueue_pool(m, u, c, use_hot, s));
    return mark(ev, EV_POOL_END, s);
}

// S3 and S4.
hipError_t enqueue_tail(const rec_model *m, const Bufs &u, const Call &c, hipStream_t s, hipEvent_t *ev)
{
    const int B = c.B, T = m->T, D = m->D;
    const bool concat = m->interaction == REC_INTERACT_CONCAT;
    // Without a Bottom-FC the dense part of the Predict-FC input is the dense input.
    const float *x0 = m->bottom.empty() ? c.dense : u.x0;
    const int x0_ld = m->bottom.empty() ? m->F : m->x0_ld;
    // S3 -> act[0], row stride z_ld, zero filled up to it
    if (concat) {
        if (!concat_rides_on_scan(m))
            REC_TRY(launch_concat_dense(x0, x0_ld, m->w0, B, u.act[0], m->z_width, m->z_ld, s));
    } else
        REC_TRY(launch_interact(x0, x0_ld, u.pooled, B, T, D, u.act[0], m->z_ld, s));
    REC_TRY(mark(ev, EV_INTERACT_END, s));
    // S4: the towers run side by side, their hidden activations in adjacent
    // column blocks of one row.  ReLU on all layers but the last.  The last layer
    // is one fp32 dot per sample and tower: folded into the epilogue of the layer
    // before it when that layer's block tile spans whole rows, else that layer
    // leaves fp32 for a dot kernel.
    const int G = m->towers, n_top = m->n_top;
    FcProblem p{};
    p.A = u.act[0]; p.a_f32 = false; p.lda = m->z_ld; p.a_stride = 0;
    p.M = B; p.relu = true; p.groups = G; p.num_cus = m->num_cus; p.corun = m->pipeline;
    for (int k = 0; k < G; ++k) {
        const Layer &dotl = m->top[(size_t)k * n_top + n_top - 1];
        p.g.dot_w[k] = static_cast<const float *>(dotl.W);
        p.g.dot_bias[k] = dotl.bias;
    }
    bool cur_f32 = false, done = false, first_marked = false;
    const Layer *layers = m->top.data();
    const int n = n_top - 1;  // layers ahead of the one-output layer
    int launches = 0;
    for (int i = 0; i < n && !done;) {
        const Layer &l = layers[i];  // shape of layer i in every tower
        const int j = chain_end(m, layers, i, n, true);
        if (j > i) {
            ChainProblem cp{};
            cp.A = p.A; cp.a_f32 = false; cp.lda = p.lda; cp.a_stride = p.a_stride; cp.M = B;
            chain_run(layers, n_top, G, i, j, cp);
            if (j == n) {
                cp.out_mode = CHAIN_OUT_DOT;
                for (int k = 0; k < G; ++k) { cp.dot_w[k] = p.g.dot_w[k]; cp.dot_bias[k] = p.g.dot_bias[k]; }
                cp.dot_out = c.logits; cp.dot_ld = G;
                done = true;
            } else {
                cp.out_mode = CHAIN_OUT_BF16;
                cp.C = u.act[1 + (launches & 1)]; cp.ldc = G * layers[j - 1].Npad; cp.c_stride = layers[j - 1].Npad;
                p.A = cp.C; p.lda = cp.ldc; p.a_stride = cp.c_stride; p.a_f32 = false;
            }
            REC_TRY(launch_mlp_chain(cp, s));
            i = j;
        } else {
            for (int k = 0; k < G; ++k) {
                p.g.W[k] = m->top[(size_t)k * n_top + i].W;
                p.g.bias[k] = m->top[(size_t)k * n_top + i].bias;
            }
            p.K = l.K; p.Kpad = l.Kpad; p.Npad = l.Npad;
            const bool feeds_dot = i + 1 == n;
            if (feeds_dot && fc_can_fuse_dot(l.Npad)) {
                p.C = nullptr; p.out_f32 = false; p.ldc = 0; p.c_stride = 0;
                p.dot_out = c.logits; p.dot_ld = G;
                REC_TRY(launch_fc(p, s));
                done = true;
            } else {
                p.C = u.act[1 + (launches & 1)]; p.out_f32 = feeds_dot; p.ldc = G * l.Npad; p.c_stride = l.Npad;
                REC_TRY(launch_fc(p, s));
                p.A = p.C; p.lda = p.ldc; p.a_stride = p.c_stride; p.a_f32 = false;
                cur_f32 = feeds_dot;
            }
            ++i;
        }
        ++launches;
        if (!first_marked) {  // the first launch (the widest layer, or the run it starts) is timed on its own
            REC_TRY(mark(ev, EV_TOP_FIRST_END, s));
            first_marked = true;
        }
    }
    if (!done)
        REC_TRY(launch_rowdot(p.A, cur_f32, p.lda, p.a_stride, B, m->top[n_top - 1].Kpad, p.g, G, c.logits, G, s));
    if (!first_marked) REC_TRY(mark(ev, EV_TOP_FIRST_END, s));
    return mark(ev, EV_END, s);
}

// The whole pass in order on one stream: S0, S1, S2, S3, S4.
hipError_t enqueue_in_order(const rec_model *m, const Bufs &u, const Call &c, bool use_hot, hipStream_t s,
                            hipEvent_t *ev)
{
    REC_TRY(mark(ev, EV_BEGIN, s));
    const bool ride = bottom_rides_on_scan(m);
    REC_TRY(enqueue_sparse(m, u, c, use_hot, s, ev, ride));
    if (ride) {  // S2 ran inside S0's second launch: its stages read zero
        REC_TRY(mark(ev, EV_BOTTOM_FIRST_END, s));
        REC_TRY(mark(ev, EV_BOTTOM_END, s));
    } else {
        REC_TRY(enqueue_bottom(m, u, c, s, ev));
    }
    return enqueue_tail(m, u, c, s, ev);
}

// Device address of `scratch` on each GPU, looked up once per device with that
// device current.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
char *g_scratch_ptr[MAX_DEVICES] = {};

rec_status static_scratch(char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return REC_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return REC_ERR_DEVICE;
        if (fc_big_prepare() != hipSuccess || chain_prepare() != hipSuccess || scan_prepare() != hipSuccess)
            return REC_ERR_DEVICE;
        g_scratch_ptr[dev] = static_cast<char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return REC_OK;
}

// Table descriptors by value: what rec_forward_static() writes into its scratch
// at the start of every call.
struct StaticTables {
    const void *base[REC_STATIC_MAX_TABLES];
    long long rows[REC_STATIC_MAX_TABLES];
};

__global__ __launch_bounds__(64) void static_begin_kernel(const StaticTables st, int T, TableDesc *dst,
                                                          ErrRecord *err)
{
    const int t = threadIdx.x;
    if (t < T) {
        dst[t].base = st.base[t];
        dst[t].rows = st.rows[t];
        dst[t].hot_ids = nullptr;
        dst[t].n_hot = 0;
        dst[t].pad = 0;
    }
    if (t == 0) {
        err->first_bad_len = ~0ull;
        err->first_bad_idx = ~0ull;
        err->flags = 0u;
    }
}

// fault[0] = the status rec_check() would give for this call, fault[1] = its position.
__global__ __launch_bounds__(64) void static_end_kernel(const ErrRecord *err, long long *fault)
{
    if (threadIdx.x != 0) return;
    const unsigned flags = err->flags;
    long long st = REC_OK, pos = -1;
    if (flags & (ERR_NEG_LENGTH | ERR_TOTAL_MISMATCH)) {
        st = REC_ERR_LENGTHS;
        if (flags & ERR_NEG_LENGTH) pos = (long long)err->first_bad_len;
    } else if (flags & ERR_INDEX_RANGE) {
        st = REC_ERR_INDEX_RANGE;
        pos = (long long)err->first_bad_idx;
    }
    fault[0] = st;
    fault[1] = pos;
}

// Host-checkable faults of a forward call.
rec_status check_call(const rec_model *m, const float *dev_dense, const int32_t *dev_indices,
                      const int32_t *dev_lengths, int32_t batch, int64_t nnz, const float *dev_logits)
{
    if (!m) return REC_ERR_ARG;
    if (batch < 0 || batch > m->max_batch || nnz < 0 || nnz > m->max_nnz) return REC_ERR_ARG;
    if (!m->ws || !all_loaded(m)) return REC_ERR_STATE;
    if (batch == 0) return REC_OK;
    if (!dev_dense || !dev_lengths || !dev_logits || (nnz > 0 && !dev_indices)) return REC_ERR_ARG;
    return REC_OK;
}

}  // namespace

extern "C" {

const char *rec_status_string(int status)
{
    // An int, not the enum: a caller may pass a number that is no enumerator, and
    // reading such a value through the enum type is undefined in C++.
    switch (status) {
    case REC_OK: return "ok";
    case REC_ERR_ARG: return "bad argument";
    case REC_ERR_SHAPE: return "layer widths or embedding size do not fit the model";
    case REC_ERR_STATE: return "call made before what it depends on";
    case REC_ERR_LENGTHS: return "negative length or sum(lengths) != nnz";
    case REC_ERR_INDEX_RANGE: return "row id outside its table";
    case REC_ERR_OVERFLOW: return "count exceeds 32-bit index range";
    case REC_ERR_DEVICE: return "HIP call failed";
    case REC_ERR_CAPACITY: return "call needs more scratch than the static array holds";
    }
    return "unknown status";
}

rec_status rec_create(const rec_config *cfg, rec_model **out)
{
    if (!out) return REC_ERR_ARG;
    *out = nullptr;
    if (!cfg || !cfg->rows || !cfg->bottom_widths || !cfg->top_widths) return REC_ERR_ARG;
    if (cfg->num_tables <= 0 || cfg->emb_dim <= 0 || cfg->num_dense <= 0 || cfg->n_bottom < 0 ||
        cfg->n_top <= 0 || cfg->max_batch <= 0 || cfg->max_nnz < 0)
        return REC_ERR_ARG;
    if (cfg->table_dtype != REC_F32 && cfg->table_dtype != REC_F16) return REC_ERR_ARG;
    if (cfg->interaction != REC_INTERACT_DOT && cfg->interaction != REC_INTERACT_CONCAT) return REC_ERR_ARG;
    if (cfg->num_towers < 0 || cfg->num_towers > REC_MAX_TOWERS) return REC_ERR_ARG;
    const int towers = cfg->num_towers > 0 ? cfg->num_towers : 1;
    const bool concat = cfg->interaction == REC_INTERACT_CONCAT;

    const int T = cfg->num_tables, D = cfg->emb_dim;
    // A row must be 16 * 2^k bytes (k = 0..6) for the 128-bit gather.
    const long long rowbytes = (long long)D * (cfg->table_dtype == REC_F16 ? 2 : 4);
    if (rowbytes % 16 != 0) return REC_ERR_SHAPE;
    const long long lpr = rowbytes / 16;
    if (lpr > 64 || (lpr & (lpr - 1)) != 0) return REC_ERR_SHAPE;

    for (int t = 0; t < T; ++t) {
        if (cfg->rows[t] <= 0) return REC_ERR_ARG;
        if (cfg->rows[t] >= (1ll << 31)) return REC_ERR_OVERFLOW;
    }
    if (cfg->max_nnz >= (1ll << 31)) return REC_ERR_OVERFLOW;
    if ((long long)T * cfg->max_batch >= (1ll << 31)) return REC_ERR_OVERFLOW;

    for (int i = 0; i <= cfg->n_bottom; ++i)
        if (cfg->bottom_widths[i] <= 0 || cfg->bottom_widths[i] >= (1 << 24)) return REC_ERR_SHAPE;
    for (int i = 0; i <= cfg->n_top; ++i)
        if (cfg->top_widths[i] <= 0 || cfg->top_widths[i] >= (1 << 24)) return REC_ERR_SHAPE;
    const int w0 = cfg->bottom_widths[cfg->n_bottom];
    const long long width = concat ? w0 + (long long)T * D : D + (long long)T * (T + 1) / 2;
    if (width >= (1ll << 24)) return REC_ERR_OVERFLOW;
    if (cfg->bottom_widths[0] != cfg->num_dense || (!concat && w0 != D)) return REC_ERR_SHAPE;
    if (cfg->top_widths[0] != width || cfg->top_widths[cfg->n_top] != 1) return REC_ERR_SHAPE;
    if (!concat && interact_lds_bytes_per_sample(T, D) > 64 * 1024) return REC_ERR_SHAPE;

    rec_model *m = new (std::nothrow) rec_model();
    if (!m) return REC_ERR_ARG;
    m->T = T; m->D = D; m->F = cfg->num_dense; m->dtype = cfg->table_dtype;
    m->interaction = cfg->interaction; m->towers = towers; m->n_top = cfg->n_top;
    m->w0 = w0; m->z_width = (int)width;
    m->max_batch = cfg->max_batch; m->max_nnz = cfg->max_nnz;
    m->rows.assign(cfg->rows, cfg->rows + T);
    for (int t = 0; t < T; ++t) m->max_rows = std::max<long long>(m->max_rows, cfg->rows[t]);
    m->table_loaded.assign(T, 0);
    m->desc.assign(T, TableDesc{nullptr, 0, nullptr, 0, 0});
    for (int t = 0; t < T; ++t) m->desc[t].rows = cfg->rows[t];
    m->x0_ld = pad_up(w0);
    m->z_ld = pad_up((int)width);
    m->act_ld = PAD;
    // Hidden activations of the towers sit side by side in one row.
    auto fill = [&](Layer *v, const int32_t *w, int n, int side_by_side) {
        for (int i = 0; i < n; ++i) {
            v[i].K = w[i]; v[i].N = w[i + 1];
            v[i].Kpad = pad_up(w[i]); v[i].Npad = pad_up(w[i + 1]);
            v[i].chain = chain_layer_fits(v[i].Kpad, v[i].Npad);
            if (i + 1 < n || side_by_side == 1)  // the one-output layer leaves no activation row
                m->act_ld = std::max(m->act_ld, side_by_side * v[i].Npad);
        }
    };
    m->bottom.resize(cfg->n_bottom);
    fill(m->bottom.data(), cfg->bottom_widths, cfg->n_bottom, 1);
    m->top.resize((size_t)towers * cfg->n_top);
    for (int k = 0; k < towers; ++k) {
        fill(&m->top[(size_t)k * cfg->n_top], cfg->top_widths, cfg->n_top, towers);
        m->top[(size_t)k * cfg->n_top + cfg->n_top - 1].dot = true;
        m->top[(size_t)k * cfg->n_top + cfg->n_top - 1].chain = false;
    }
    m->act_row_bytes = 2 * (size_t)m->act_ld;
    if (cfg->n_top > 1)  // the layer feeding the dot leaves fp32
        m->act_row_bytes = std::max(m->act_row_bytes, sizeof(float) * towers * m->top[cfg->n_top - 2].Npad);

    m->lay = carve(m, m->max_batch, 1);
    *out = m;
    return REC_OK;
}

void rec_destroy(rec_model *m)
{
    if (!m) return;
    for (hipEvent_t e : m->ev)
        if (e) (void)hipEventDestroy(e);
    if (m->ev_fork) (void)hipEventDestroy(m->ev_fork);
    if (m->ev_join) (void)hipEventDestroy(m->ev_join);
    for (int k = 0; k < MAX_FRAMES; ++k)
        for (hipEvent_t e : {m->ev_scan[k], m->ev_pool[k], m->ev_tail[k], m->ev_bottom[k]})
            if (e) (void)hipEventDestroy(e);
    for (hipStream_t o : m->own_stream)
        if (o) (void)hipStreamDestroy(o);
    if (m->side) (void)hipStreamDestroy(m->side);
    delete m;
}

size_t rec_workspace_bytes(const rec_model *m) { return m ? m->lay.bytes : 0; }

rec_status rec_bind_workspace(rec_model *m, void *dev_ptr, size_t bytes, void *stream)
{
    if (!m || !dev_ptr) return REC_ERR_ARG;
    if (bytes < m->lay.bytes || reinterpret_cast<uintptr_t>(dev_ptr) % ALIGN != 0) return REC_ERR_ARG;
    if (!m->side) {
        // Default priority; the two events only order work, they carry no timing.
        if (hipStreamCreateWithFlags(&m->side, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming) != hipSuccess)
            return REC_ERR_DEVICE;
        for (int k = 0; k < MAX_FRAMES; ++k)
            if (hipEventCreateWithFlags(&m->ev_scan[k], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&m->ev_pool[k], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&m->ev_tail[k], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&m->ev_bottom[k], hipEventDisableTiming) != hipSuccess)
                return REC_ERR_DEVICE;
    }
    if (m->pipeline)
        for (hipStream_t &o : m->own_stream)
            if (!o && hipStreamCreateWithFlags(&o, hipStreamNonBlocking) != hipSuccess) return REC_ERR_DEVICE;
    for (bool &b : m->tail_pending) b = false;
    m->next_frame = m->last_frame = 0;
    m->pool_turn = 0;
    if (fc_big_prepare() != hipSuccess || chain_prepare() != hipSuccess || scan_prepare() != hipSuccess)
            return REC_ERR_DEVICE;
    {   // set-up is also where the static scratch of this device is looked up
        char *unused = nullptr;
        if (static_scratch(&unused) != REC_OK) return REC_ERR_DEVICE;
    }
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        m->num_cus = cus;
    m->ws = static_cast<char *>(dev_ptr);
    // The descriptors live in the workspace: tables and hot lists are to be registered again.
    std::fill(m->table_loaded.begin(), m->table_loaded.end(), 0);
    for (TableDesc &d : m->desc) { d.base = nullptr; d.hot_ids = nullptr; d.n_hot = 0; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_clear_err(m->at<ErrRecord>(m->lay.off_err), s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    return REC_OK;
}

rec_status rec_load_tables(rec_model *m, int32_t table, const void *dev_rows)
{
    if (!m || !dev_rows || table < 0 || table >= m->T) return REC_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(dev_rows) % 16 != 0) return REC_ERR_ARG;
    if (!m->ws) return REC_ERR_STATE;
    m->desc[table].base = dev_rows;
    if (hipMemcpy(m->at<TableDesc>(m->lay.off_tables) + table, &m->desc[table], sizeof(TableDesc),
                  hipMemcpyHostToDevice) != hipSuccess)
        return REC_ERR_DEVICE;
    m->table_loaded[table] = 1;
    return REC_OK;
}

rec_status rec_load_hot_rows(rec_model *m, int32_t table, const int32_t *dev_ids, int32_t n)
{
    if (!m || table < 0 || table >= m->T || n < 0 || n > REC_MAX_HOT_ROWS || (n > 0 && !dev_ids))
        return REC_ERR_ARG;
    if (!m->ws) return REC_ERR_STATE;
    int hcap = 16;
    while (hcap < n) hcap *= 2;
    const int rowbytes = m->D * (m->dtype == REC_F16 ? 2 : 4);
    if (n > 0 && !pool_hot_fits(hcap, rowbytes)) return REC_ERR_ARG;
    m->desc[table].hot_ids = n > 0 ? dev_ids : nullptr;
    m->desc[table].n_hot = n;
    if (hipMemcpy(m->at<TableDesc>(m->lay.off_tables) + table, &m->desc[table], sizeof(TableDesc),
                  hipMemcpyHostToDevice) != hipSuccess)
        return REC_ERR_DEVICE;
    return REC_OK;
}

size_t rec_mlp_packed_bytes(const rec_model *m, int32_t which, int32_t layer)
{
    if (!m) return 0;
    const Layer *l = find_layer(const_cast<rec_model *>(m), which, layer);
    if (!l) return 0;
    return align_up(l->w_bytes()) + align_up(sizeof(float) * l->Npad) + align_up(l->chain_bytes());
}

rec_status rec_load_mlp(rec_model *m, int32_t which, int32_t layer, const float *dev_W,
                        const float *dev_b, void *dev_packed, void *stream)
{
    if (!m || !dev_W || !dev_b || !dev_packed) return REC_ERR_ARG;
    Layer *l = find_layer(m, which, layer);
    if (!l) return REC_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(dev_packed) % ALIGN != 0) return REC_ERR_ARG;
    char *p = static_cast<char *>(dev_packed);
    float *bias = reinterpret_cast<float *>(p + align_up(l->w_bytes()));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = l->dot ? launch_pack_dot(dev_W, dev_b, l->K, l->Kpad, reinterpret_cast<float *>(p), bias, s)
                                : launch_pack_fc(dev_W, dev_b, l->N, l->K, l->Npad, l->Kpad, p, bias, s);
    if (e != hipSuccess) return REC_ERR_DEVICE;
    if (l->chain) {
        char *pc = p + align_up(l->w_bytes()) + align_up(sizeof(float) * l->Npad);
        if (launch_pack_chain(dev_W, l->N, l->K, l->Npad, l->Kpad, pc, s) != hipSuccess) return REC_ERR_DEVICE;
        l->Wc = pc;
    }
    l->W = p;
    l->bias = bias;
    l->loaded = true;
    return REC_OK;
}

rec_status rec_forward(rec_model *m, const float *dev_dense, const int32_t *dev_indices,
                       const int32_t *dev_lengths, int32_t batch, int64_t nnz, float *dev_logits,
                       void *stream)
{
    const rec_status st = check_call(m, dev_dense, dev_indices, dev_lengths, batch, nnz, dev_logits);
    if (st != REC_OK || batch == 0) return st;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const Call c{dev_dense, dev_indices, dev_lengths, batch, nnz, dev_logits};
    // Forward number i is timed when i is a multiple of the period; it is the
    // (i / period)-th timed one.
    const bool prof = m->slots > 0 && m->forwards % m->period == 0;
    const size_t slot = prof ? (size_t)((m->forwards / m->period) % m->slots) : 0;
    hipEvent_t *ev = prof ? &m->ev[slot * EV_PER_SLOT] : nullptr;
#define REC_DEV(call)                                  \
    do {                                               \
        if ((call) != hipSuccess) return REC_ERR_DEVICE; \
    } while (0)

    if (m->pipeline) {
        // Four queues (Sec. IV-A, S-D pipeline; dependencies of Sec. III-A): scan
        // (S0) and Bottom-FC (S2) on the caller's stream, pooling (S1) on two
        // streams in turn, interaction and Predict-FC (S3, S4) on a fourth.  Two
        // pooling launches are in flight at any time, so neither the packets between
        // launches nor the ramps of a launch leave the memory system idle; a batch
        // owns one of four frames until its logits are written.
        const int k = m->next_frame;
        const Bufs u = bufs_at(m->ws, m->lay, k);
        hipStream_t p = m->pool_stream[m->pool_turn] ? m->pool_stream[m->pool_turn] : m->own_stream[m->pool_turn];
        hipStream_t d = m->dense_stream ? m->dense_stream : m->side;
        if (m->tail_pending[k]) {  // the batch that used this frame four calls ago
            REC_DEV(hipStreamWaitEvent(s, m->ev_tail[k], 0));
            m->tail_pending[k] = false;
        }
        REC_DEV(mark(ev, EV_BEGIN, s));
        REC_DEV(enqueue_scan(m, u, c, s, false));
        REC_DEV(mark(ev, EV_SCAN_END, s));
        REC_DEV(hipEventRecord(m->ev_scan[k], s));
        REC_DEV(hipStreamWaitEvent(p, m->ev_scan[k], 0));
        REC_DEV(mark(ev, EV_POOL_BEGIN, p));
        REC_DEV(enqueue_pool(m, u, c, true, p));
        REC_DEV(mark(ev, EV_POOL_END, p));
        REC_DEV(hipEventRecord(m->ev_pool[k], p));
        if (!m->bottom.empty()) {
            REC_DEV(mark(ev, EV_BOTTOM_BEGIN, s));
            REC_DEV(enqueue_bottom(m, u, c, s, ev));
        }
        REC_DEV(hipEventRecord(m->ev_bottom[k], s));
        REC_DEV(hipStreamWaitEvent(d, m->ev_bottom[k], 0));
        REC_DEV(hipStreamWaitEvent(d, m->ev_pool[k], 0));
        REC_DEV(mark(ev, EV_INTERACT_BEGIN, d));
        REC_DEV(enqueue_tail(m, u, c, d, ev));
        REC_DEV(hipEventRecord(m->ev_tail[k], d));
        m->tail_pending[k] = true;
        m->last_frame = k;
        m->next_frame = (k + 1) % MAX_FRAMES;
        m->pool_turn ^= 1;
        if (prof) m->slot_mode[slot] = 1;
    } else {
        const Bufs u = bufs_at(m->ws, m->lay, 0);
        m->last_frame = 0;
        // S2 does not depend on S0/S1: with overlap it is enqueued on the side
        // stream, forked from and joined back into the caller's stream.
        if (m->overlap_dense && !m->bottom.empty()) {
            REC_DEV(mark(ev, EV_BEGIN, s));
            REC_DEV(hipEventRecord(m->ev_fork, s));
            REC_DEV(hipStreamWaitEvent(m->side, m->ev_fork, 0));
            REC_DEV(enqueue_bottom(m, u, c, m->side, nullptr));
            REC_DEV(hipEventRecord(m->ev_join, m->side));
            REC_DEV(enqueue_sparse(m, u, c, true, s, ev));
            // the "bottom" stage then times only what pooling did not hide
            REC_DEV(hipStreamWaitEvent(s, m->ev_join, 0));
            REC_DEV(mark(ev, EV_BOTTOM_FIRST_END, s));
            REC_DEV(mark(ev, EV_BOTTOM_END, s));
            REC_DEV(enqueue_tail(m, u, c, s, ev));
        } else {
            REC_DEV(enqueue_in_order(m, u, c, true, s, ev));
        }
        if (prof) m->slot_mode[slot] = !m->overlap_dense && bottom_rides_on_scan(m) ? 2 : 0;
    }
#undef REC_DEV
    if (m->slots > 0) ++m->forwards;
    return REC_OK;
}

rec_status rec_forward_static(rec_model *m, const float *dev_dense, const int32_t *dev_indices,
                              const int32_t *dev_lengths, int32_t batch, int64_t nnz, float *dev_logits,
                              int64_t *dev_fault, void *stream)
{
    const rec_status st = check_call(m, dev_dense, dev_indices, dev_lengths, batch, nnz, dev_logits);
    if (st != REC_OK) return st;
    if (m->T > REC_STATIC_MAX_TABLES) return REC_ERR_CAPACITY;
    const Carve lay = carve(m, batch > 0 ? batch : 1, 1);
    if (lay.bytes > REC_STATIC_SCRATCH_BYTES) return REC_ERR_CAPACITY;
    char *base = nullptr;
    const rec_status sp = static_scratch(&base);
    if (sp != REC_OK) return sp;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const Bufs u = bufs_at(base, lay, 0);
    // The array keeps what the last call left: descriptors and error record are
    // written afresh; every other part is fully overwritten before it is read.
    StaticTables tabs{};
    for (int t = 0; t < m->T; ++t) {
        tabs.base[t] = m->desc[t].base;
        tabs.rows[t] = m->desc[t].rows;
    }
    hipLaunchKernelGGL(static_begin_kernel, dim3(1), dim3(64), 0, s, tabs, m->T,
                       const_cast<TableDesc *>(u.tables), u.err);
    if (hipGetLastError() != hipSuccess) return REC_ERR_DEVICE;
    if (batch > 0) {
        const Call c{dev_dense, dev_indices, dev_lengths, batch, nnz, dev_logits};
        if (enqueue_in_order(m, u, c, false, s, nullptr) != hipSuccess) return REC_ERR_DEVICE;
    }
    if (dev_fault) {
        hipLaunchKernelGGL(static_end_kernel, dim3(1), dim3(64), 0, s, u.err,
                           reinterpret_cast<long long *>(dev_fault));
        if (hipGetLastError() != hipSuccess) return REC_ERR_DEVICE;
    }
    return REC_OK;
}

rec_status rec_drain(rec_model *m, void *stream)
{
    if (!m) return REC_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Every batch's last stage runs on the one dense stream, in order: the event
    // of the latest call stands for all of them.
    if (m->tail_pending[m->last_frame] &&
        hipStreamWaitEvent(s, m->ev_tail[m->last_frame], 0) != hipSuccess)
        return REC_ERR_DEVICE;
    for (bool &p : m->tail_pending) p = false;
    return REC_OK;
}

rec_status rec_check(rec_model *m, void *stream, int64_t *first_bad_pos)
{
    if (!m) return REC_ERR_ARG;
    if (!m->ws) return REC_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ErrRecord h;
    ErrRecord *d = m->at<ErrRecord>(m->lay.off_err);
    if (rec_drain(m, stream) != REC_OK) return REC_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipMemcpy(&h, d, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return REC_ERR_DEVICE;
    if (first_bad_pos) *first_bad_pos = -1;
    if (h.flags == 0) return REC_OK;
    if (launch_clear_err(d, s) != hipSuccess) return REC_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return REC_ERR_DEVICE;
    if (h.flags & (ERR_NEG_LENGTH | ERR_TOTAL_MISMATCH)) {
        if (first_bad_pos && (h.flags & ERR_NEG_LENGTH)) *first_bad_pos = (int64_t)h.first_bad_len;
        return REC_ERR_LENGTHS;
    }
    if (first_bad_pos) *first_bad_pos = (int64_t)h.first_bad_idx;
    return REC_ERR_INDEX_RANGE;
}

rec_status rec_debug_get(rec_model *m, int32_t what, const void **dev_ptr, int64_t *ld_out)
{
    if (!m || !dev_ptr) return REC_ERR_ARG;
    if (!m->ws) return REC_ERR_STATE;
    int64_t ld = 0;
    const Frame &f = m->lay.fr[m->last_frame];
    switch (what) {
    case REC_DBG_OFFSETS: *dev_ptr = m->at<void>(f.off_offsets); ld = 0; break;
    case REC_DBG_POOLED:
        if (m->interaction != REC_INTERACT_DOT) return REC_ERR_STATE;
        *dev_ptr = m->at<void>(f.off_pooled); ld = m->D; break;
    case REC_DBG_BOTTOM_OUT:
        if (m->bottom.empty()) return REC_ERR_STATE;
        *dev_ptr = m->at<void>(f.off_x0); ld = m->x0_ld; break;
    case REC_DBG_INTERACT: *dev_ptr = m->at<void>(f.off_act[0]); ld = m->z_ld; break;
    default: return REC_ERR_ARG;
    }
    if (ld_out) *ld_out = ld;
    return REC_OK;
}

rec_status rec_set_option(rec_model *m, int32_t option, int32_t value)
{
    if (!m) return REC_ERR_ARG;
    switch (option) {
    case REC_OPT_OVERLAP_DENSE: m->overlap_dense = value != 0; return REC_OK;
    case REC_OPT_STREAM_ROWS: m->stream_rows = value != 0; return REC_OK;
    case REC_OPT_FUSE_MLP:
        if (value < 0 || value > 2) return REC_ERR_ARG;
        m->fuse_mlp = value;
        return REC_OK;
    case REC_OPT_PIPELINE:
        // Decides the size of the workspace: only while none is bound.
        if (m->ws) return REC_ERR_STATE;
        m->pipeline = value != 0;
        m->lay = carve(m, m->max_batch, m->pipeline ? MAX_FRAMES : 1);
        return REC_OK;
    default: return REC_ERR_ARG;
    }
}

rec_status rec_set_dense_stream(rec_model *m, void *stream)
{
    if (!m) return REC_ERR_ARG;
    for (int k = 0; k < MAX_FRAMES; ++k)
        if (m->tail_pending[k]) return REC_ERR_STATE;  // work is still ordered on the old one
    m->dense_stream = static_cast<hipStream_t>(stream);
    return REC_OK;
}

rec_status rec_set_pool_streams(rec_model *m, void *stream_a, void *stream_b)
{
    if (!m) return REC_ERR_ARG;
    for (int k = 0; k < MAX_FRAMES; ++k)
        if (m->tail_pending[k]) return REC_ERR_STATE;
    m->pool_stream[0] = static_cast<hipStream_t>(stream_a);
    m->pool_stream[1] = static_cast<hipStream_t>(stream_b);
    return REC_OK;
}

rec_status rec_set_profiling(rec_model *m, int32_t slots, int32_t period)
{
    if (!m || slots < 0 || slots > 65536 || (slots > 0 && period < 1)) return REC_ERR_ARG;
    for (hipEvent_t e : m->ev)
        if (e) (void)hipEventDestroy(e);
    m->ev.assign((size_t)slots * EV_PER_SLOT, nullptr);
    m->slot_mode.assign((size_t)slots, 0);
    m->slots = 0;
    m->forwards = 0;
    for (hipEvent_t &e : m->ev)
        if (hipEventCreate(&e) != hipSuccess) return REC_ERR_DEVICE;
    m->slots = slots;
    m->period = slots > 0 ? period : 1;
    return REC_OK;
}

rec_status rec_stage_ms(rec_model *m, int32_t slot, float *ms)
{
    if (!m || !ms) return REC_ERR_ARG;
    const long long timed = (m->forwards + m->period - 1) / m->period;  // timed forwards so far
    if (m->slots <= 0 || slot < 0 || slot >= m->slots || slot >= timed) return REC_ERR_STATE;
    hipEvent_t *ev = &m->ev[(size_t)slot * EV_PER_SLOT];
    // Stage i ran between events begin[i] and end[i]; in a pipelined forward the
    // dense stages sit on another stream and have begin events of their own.
    static const int end[REC_NUM_STAGES] = {EV_SCAN_END, EV_POOL_END, EV_BOTTOM_FIRST_END, EV_BOTTOM_END,
                                            EV_INTERACT_END, EV_TOP_FIRST_END, EV_END};
    static const int begin_in_order[REC_NUM_STAGES] = {EV_BEGIN, EV_SCAN_END, EV_POOL_END, EV_BOTTOM_FIRST_END,
                                                       EV_BOTTOM_END, EV_INTERACT_END, EV_TOP_FIRST_END};
    static const int begin_pipelined[REC_NUM_STAGES] = {EV_BEGIN, EV_POOL_BEGIN, EV_BOTTOM_BEGIN,
                                                        EV_BOTTOM_FIRST_END, EV_INTERACT_BEGIN,
                                                        EV_INTERACT_END, EV_TOP_FIRST_END};
    const int *begin = m->slot_mode[slot] == 1 ? begin_pipelined : begin_in_order;
    if (hipEventSynchronize(ev[EV_END]) != hipSuccess) return REC_ERR_DEVICE;
    for (int i = 0; i < REC_NUM_STAGES; ++i) {
        ms[i] = 0.0f;
        const bool bottom_stage = i == REC_STAGE_BOTTOM_FIRST || i == REC_STAGE_BOTTOM_REST;
        if (bottom_stage && ((m->slot_mode[slot] == 1 && m->bottom.empty()) || m->slot_mode[slot] == 2))
            continue;  // no launch of its own: nothing to time
        if (hipEventElapsedTime(&ms[i], ev[begin[i]], ev[end[i]]) != hipSuccess) return REC_ERR_DEVICE;
    }
    return REC_OK;
}

}  // extern "C"
