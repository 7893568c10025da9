/*
 * rec.h - C boundary of the DLRM-class forward pass on one MI355X (gfx950).
 *
 * One inference query carries, for each of its items ("query size", Sec. II-A),
 * a vector of dense features and, per embedding table, a variable-length list
 * of row ids (the pooling factor, Fig. 2(c)); the model (Fig. 2(a), Table I)
 * returns one click-through score per item.  rec_forward() computes that for a
 * batch of fused items ("query fusion", Sec. II-B):
 *
 *   offsets   = exclusive scan of the pooling lengths
 *   pooled    = per (sample, table): sum of the gathered rows
 *               (SparseNet; "Gather-Reduce" / SLS, Sec. VI-B)
 *   x0        = Bottom-FC(dense)                  (DenseNet, Table I)
 *   z         = [x0, <v_i, v_j> for i > j] over v = [x0, pooled_0, ...]
 *               (pairwise-dot interaction of the DLRM model the paper cites)
 *   logit     = Predict-FC(z)                     (DenseNet, Table I)
 *
 * A second model shape (Table I, row MT-WnD: one lookup per table, no pooling,
 * no Bottom-FC, N Predict-FC towers) has no interaction operator:
 *
 *   z         = [x0, pooled_0, ..., pooled_{T-1}]     (x0 = dense when there is
 *                                                      no Bottom-FC)
 *   logit_k   = tower_k(z), k = 0..N-1                (one logit per task)
 *
 * Bottom-FC runs independently of the SparseNet and Predict-FC waits for both
 * (Sec. III-A).  Element-wise work (bias, ReLU, narrowing, concatenation) is
 * fused into the producing kernels (Sec. IV-A, operator fusion).
 *
 * Conventions
 *   - Every pointer named dev_* is DEVICE memory owned by the caller and
 *     borrowed by the library; it must stay valid while the model uses it.
 *     The library itself allocates no device memory.
 *   - `stream` arguments are a hipStream_t passed as void* (NULL = the null
 *     stream).  rec_forward() only enqueues work on that stream.
 *   - Every call returns a rec_status; nothing aborts or throws.
 *   - A model is not thread-safe; forwards of one model that overlap on the
 *     device race on its workspace.
 */
#ifndef REC_H
#define REC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbol (the library is built with hidden visibility by default). */
#define REC_API __attribute__((visibility("default")))

typedef struct rec_model rec_model;

typedef enum {
    REC_OK = 0,
    REC_ERR_ARG = 1,         /* null pointer, id out of range, bad enum          */
    REC_ERR_SHAPE = 2,       /* layer widths do not chain / unsupported emb_dim  */
    REC_ERR_STATE = 3,       /* call made before what it depends on              */
    REC_ERR_LENGTHS = 4,     /* device: negative length, or sum(lengths) != nnz  */
    REC_ERR_INDEX_RANGE = 5, /* device: a row id outside [0, rows)               */
    REC_ERR_OVERFLOW = 6,    /* a count does not fit the 32-bit index math       */
    REC_ERR_DEVICE = 7,      /* a HIP call failed                                */
    REC_ERR_CAPACITY = 8     /* rec_forward_static(): call exceeds the static scratch */
} rec_status;

typedef enum { REC_F32 = 0, REC_F16 = 1 } rec_dtype;

/* Which stack a layer belongs to: REC_BOTTOM, or REC_TOP + k for tower k of the
 * Predict-FC (REC_TOP alone when there is one stack). */
enum { REC_BOTTOM = 0, REC_TOP = 1 };

/* How the dense part and the pooled vectors become the Predict-FC input. */
enum {
    REC_INTERACT_DOT = 0,    /* [x0, pairwise dots]: DLRM-RMC rows of Table I        */
    REC_INTERACT_CONCAT = 1  /* [x0, pooled vectors]: MT-WnD row of Table I          */
};

/* Most Predict-FC towers a model can have. */
#define REC_MAX_TOWERS 8

/* Intermediate buffers rec_debug_get() can expose (all inside the workspace). */
enum {
    REC_DBG_OFFSETS = 0,   /* int32 [T*B + 1], table-major                       */
    REC_DBG_POOLED = 1,    /* fp32  [B][T][D]; REC_INTERACT_DOT only             */
    REC_DBG_BOTTOM_OUT = 2,/* fp32  [B][ld]; models with a Bottom-FC only        */
    REC_DBG_INTERACT = 3   /* bf16  [B][ld], ld = *ld_out; columns >= width are 0:
                              the Predict-FC input of either model shape          */
};

/* Stages timed by rec_set_profiling().  Bottom-FC and Predict-FC are each split
 * into their first launch (the widest matrix product of the stack, or the run of
 * layers it starts) and the rest. */
enum {
    REC_STAGE_SCAN = 0, REC_STAGE_POOL = 1, REC_STAGE_BOTTOM_FIRST = 2, REC_STAGE_BOTTOM_REST = 3,
    REC_STAGE_INTERACT = 4, REC_STAGE_TOP_FIRST = 5, REC_STAGE_TOP_REST = 6, REC_NUM_STAGES = 7
};

/*
 * Model shape (Table I columns: # of Embs, Emb Size, Bottom-FC, Predict-FC).
 *   rows[t]         rows of table t, each < 2^31
 *   emb_dim         D; D * sizeof(element) must be 16 * 2^k bytes, k = 0..6
 *   bottom_widths   n_bottom + 1 entries: num_dense, ..., w0.  n_bottom = 0
 *                   (one entry) means no Bottom-FC: x0 is the dense input.
 *                   REC_INTERACT_DOT needs w0 = emb_dim.
 *   top_widths      n_top + 1 entries, the first being the width of z:
 *                   emb_dim + T(T+1)/2 (REC_INTERACT_DOT) or w0 + T * emb_dim
 *                   (REC_INTERACT_CONCAT), the last being 1
 *   max_batch       largest batch rec_forward() will be given
 *   max_nnz         largest total number of ids per batch, < 2^31
 *   interaction     REC_INTERACT_*
 *   num_towers      Predict-FC stacks of widths top_widths, each with weights
 *                   of its own, all reading the same z; 0 counts as 1
 * The arrays are copied; they need not outlive rec_create().
 */
typedef struct {
    int32_t num_tables;
    int32_t emb_dim;
    const int64_t *rows;
    int32_t table_dtype;          /* rec_dtype */
    int32_t num_dense;
    int32_t n_bottom;
    const int32_t *bottom_widths;
    int32_t n_top;
    const int32_t *top_widths;
    int32_t max_batch;
    int64_t max_nnz;
    int32_t interaction;
    int32_t num_towers;
} rec_config;

/* Validates the shape and builds the host-side model.  No device work.
 * REC_ERR_ARG (null / non-positive counts, bad enum, more than REC_MAX_TOWERS
 * towers), REC_ERR_SHAPE (width chain, emb_dim), REC_ERR_OVERFLOW (rows,
 * max_nnz or T*max_batch >= 2^31). */
REC_API rec_status rec_create(const rec_config *cfg, rec_model **out);

/* Frees the host-side model.  Device buffers stay the caller's. */
REC_API void rec_destroy(rec_model *m);

/* Bytes of device workspace the model needs (offsets, pooled vectors,
 * activations, error record); 0 if m is null. */
REC_API size_t rec_workspace_bytes(const rec_model *m);

/* Hands the model its workspace: dev_ptr is 256-byte aligned device memory of
 * at least rec_workspace_bytes().  Clears the device error record on `stream`
 * and waits for it; the first call also creates the library's side stream and
 * its two ordering events on the current device, and every call sets the
 * kernels' LDS limits there (so: not under stream capture).  REC_ERR_ARG if too small or
 * misaligned. */
REC_API rec_status rec_bind_workspace(rec_model *m, void *dev_ptr, size_t bytes, void *stream);

/* Registers table `table`: dev_rows is [rows[table]][emb_dim], row-major, of
 * the configured dtype, 16-byte aligned.  Needs a bound workspace
 * (REC_ERR_STATE otherwise); copies one descriptor to the device and waits. */
REC_API rec_status rec_load_tables(rec_model *m, int32_t table, const void *dev_rows);

/* Longest hot list rec_load_hot_rows() accepts. */
#define REC_MAX_HOT_ROWS 1024

/* Registers the hot rows of table `table` (locality-aware embedding partition,
 * Sec. IV-A: the entries accessed most often, found by profiling the id
 * stream): dev_ids is int32 [n] row ids in device memory, borrowed for the
 * life of the model.  With a hot list on any table the pooling kernel keeps a
 * copy of the listed rows in LDS, refreshed from the table on every forward,
 * and serves lookups of those ids from there; the pooled sums are the same.
 * Ids listed twice or outside the table are ignored.  n = 0 removes the list.
 * REC_INTERACT_CONCAT models accept the lists and ignore them.
 * REC_ERR_ARG if n > REC_MAX_HOT_ROWS or n rows do not fit the 64 KB LDS
 * budget (about 384 rows of 128 bytes); REC_ERR_STATE without a workspace. */
REC_API rec_status rec_load_hot_rows(rec_model *m, int32_t table, const int32_t *dev_ids, int32_t n);

/* Bytes of the packed form of one layer (bf16 weights padded to the tile grid
 * followed by fp32 bias); 0 on a bad layer id. */
REC_API size_t rec_mlp_packed_bytes(const rec_model *m, int32_t which, int32_t layer);

/* Packs layer `layer` of stack `which` (REC_BOTTOM, or REC_TOP + tower):
 * dev_W is fp32 [out][in] row-major, dev_b fp32 [out]; dev_packed (256-byte aligned, rec_mlp_packed_bytes()) receives
 * the weights rounded to bf16 (nearest even) and zero padded.  Enqueued on
 * `stream`; dev_W / dev_b may be released once the stream has passed it,
 * dev_packed is borrowed for the life of the model. */
REC_API rec_status rec_load_mlp(rec_model *m, int32_t which, int32_t layer, const float *dev_W,
                        const float *dev_b, void *dev_packed, void *stream);

/*
 * Enqueues one forward pass on `stream`.
 *   dev_dense    fp32  [batch][num_dense]
 *   dev_indices  int32 [nnz], bags concatenated table-major
 *   dev_lengths  int32 [num_tables * batch], entry t*batch + b = bag (t, b)
 *   dev_logits   fp32  [batch][num_towers]  (pre-sigmoid)
 * No allocation, no synchronisation, no host read of device data.
 * Host-checkable faults return at once: REC_ERR_ARG (null, batch < 0 or
 * > max_batch, nnz < 0 or > max_nnz), REC_ERR_STATE (workspace, a table or a
 * layer missing).  batch == 0 enqueues nothing.  Faults only the device can
 * see never stop the pass: a negative length counts as 0, an id outside its
 * table contributes zero, ids past `nnz` are not read; each sets a sticky
 * device error record that rec_check() reports.
 * An empty bag pools to zero; duplicate ids count with multiplicity.
 */
REC_API rec_status rec_forward(rec_model *m, const float *dev_dense, const int32_t *dev_indices,
                       const int32_t *dev_lengths, int32_t batch, int64_t nnz,
                       float *dev_logits, void *stream);

/*
 * rec_forward() for callers that cannot allocate device memory or hand over a
 * workspace of their own at call time: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same pass, same kernels,
 * same results, but every intermediate (offsets, tile sums, pooled vectors,
 * activations, table descriptors, error record) lives in a static device
 * array of REC_STATIC_SCRATCH_BYTES that the library holds on each GPU it runs
 * on until the process ends, laid out for `batch` (not max_batch) samples.
 * The call allocates nothing and synchronises nothing; the bound workspace is
 * not touched.  The model is set up as for rec_forward() (tables and layers
 * registered); hot-row lists, REC_OPT_OVERLAP_DENSE, REC_OPT_PIPELINE and
 * stage timing do not apply here.  The device of `stream` must be current.
 *   dev_fault   device int64 [2], may be NULL: receives what rec_check() would
 *               report for this call: [0] REC_OK / REC_ERR_LENGTHS /
 *               REC_ERR_INDEX_RANGE, [1] the first bad position or -1.
 * REC_ERR_CAPACITY if the model has more than REC_STATIC_MAX_TABLES tables or
 * this batch needs more than REC_STATIC_SCRATCH_BYTES (nothing is enqueued);
 * otherwise errors as rec_forward().  All calls on one GPU share the one
 * array: calls that overlap on a GPU (two streams, two models) race.
 */
#define REC_STATIC_SCRATCH_BYTES (64u << 20)
#define REC_STATIC_MAX_TABLES 64
REC_API rec_status rec_forward_static(rec_model *m, const float *dev_dense, const int32_t *dev_indices,
                              const int32_t *dev_lengths, int32_t batch, int64_t nnz,
                              float *dev_logits, int64_t *dev_fault, void *stream);

/* Waits for `stream` (and, pipelined, for every outstanding stage), reads
 * and clears the device error record.  Returns REC_OK,
 * REC_ERR_LENGTHS (first_bad_pos = position in lengths of the first negative
 * one, or -1 when only the total disagreed with nnz) or REC_ERR_INDEX_RANGE
 * (first_bad_pos = smallest position in indices of an id outside its table).
 * Length faults win over index faults.  first_bad_pos may be null. */
REC_API rec_status rec_check(rec_model *m, void *stream, int64_t *first_bad_pos);

/* Device pointer of an intermediate buffer of the last forward (REC_DBG_*);
 * pipelined models: of the last call's frame, valid once its dense stages are done.
 * ld_out (may be null) receives the row stride in elements where it applies. */
REC_API rec_status rec_debug_get(rec_model *m, int32_t what, const void **dev_ptr, int64_t *ld_out);

/* Options of rec_set_option(). */
enum {
    /* 1: Bottom-FC is enqueued on a stream of the library's own
     * (default priority), forked from and joined back into the caller's
     * stream with events, so that it runs beside the offsets scan and the
     * pooling, on which it does not depend (Sec. III-A; the sparse / dense
     * split of Sec. IV-A).  0 (default): everything on the caller's stream, in
     * order; the cross-stream waits cost more than small dense stacks take. */
    REC_OPT_OVERLAP_DENSE = 0,
    /* 1: the pooling kernel loads table rows with the non-temporal hint, i.e.
     * tells the caches not to keep them ahead of other lines.  For the caller
     * that knows its id stream has no reuse worth caching (uniform ids: a few
     * per cent faster).  0 (default): rows are cached; production id streams are
     * skewed (the "hot" entries of Sec. IV-A) and the caches then serve a large
     * share of the lookups (streaming is 20 % slower on Zipf(1.05) ids).  The
     * pooled sums are the same either way. */
    REC_OPT_STREAM_ROWS = 1,
    /* Consecutive FC layers of at most 1024 (padded) inputs and outputs can run
     * as one kernel per stack, their activations held on chip between layers.
     * 2: always; 0: never, every layer is a kernel of its own; 1 (default):
     * where it was measured to pay, runs that save at least one launch and
     * whose weights total at most 256 KiB (every block of such a kernel
     * streams all weights of its run; never in a pipelined model, where its
     * 8-wave blocks would find no room beside the pooling launch).  Same
     * arithmetic either way: bf16 operands, fp32 accumulation, the one-output
     * layer in fp32; sums are taken in a different order. */
    REC_OPT_FUSE_MLP = 2,
    /* 1: sparse-dense pipeline across batches (Sec. IV-A, "S-D pipeline": the
     * SparseNet of one query runs beside the DenseNet of others; Predict-FC
     * waits for both, Sec. III-A).  rec_forward() then spreads a batch over four
     * streams, ordered by events: the offsets scan and Bottom-FC on the
     * caller's stream, the pooling launch on one of two pooling streams taken in
     * turn (rec_set_pool_streams()), interaction and Predict-FC on the dense
     * stream (rec_set_dense_stream()).  The caller's stream never waits for
     * pooling, so while two pooling launches are in flight the other streams
     * run the first stages of later batches and the last stages of earlier ones.
     * The workspace holds four copies of the per-batch buffers (a batch owns one
     * until its logits are written; the fifth call makes the caller's stream
     * wait for the first), so the option is set before rec_workspace_bytes()
     * and rec_bind_workspace() (REC_ERR_STATE once a workspace is bound).
     * What changes for the caller: every input is still read in stream order
     * behind `stream`, but the logits of a call, and the right to reuse or free
     * that call's input and output buffers, are ordered on `stream` only behind
     * rec_drain(); all calls of one model go to one stream.
     * Same kernels, same results.  Under stream capture the other streams fork
     * from `stream` through those events and rejoin it in rec_drain().
     * 0 (default): everything in order on the caller's stream. */
    REC_OPT_PIPELINE = 3
};
REC_API rec_status rec_set_option(rec_model *m, int32_t option, int32_t value);

/* The stream on which a pipelined model (REC_OPT_PIPELINE) runs interaction
 * and Predict-FC: a hipStream_t of default priority that the caller owns and
 * keeps alive, ideally one that the device runs beside the others (streams
 * share a few hardware queues; two on the same queue take turns).
 * NULL: a stream of the library's own.  REC_ERR_STATE while stages are
 * outstanding (call rec_drain() first). */
REC_API rec_status rec_set_dense_stream(rec_model *m, void *stream);

/* The two streams on which a pipelined model runs its pooling launches in
 * turn: hipStream_t of default priority that the caller owns and keeps alive,
 * ideally on hardware queues of their own beside `stream` of rec_forward() and
 * the dense stream.  NULL for either: a stream of the library's own.
 * REC_ERR_STATE while stages are outstanding (call rec_drain() first). */
REC_API rec_status rec_set_pool_streams(rec_model *m, void *stream_a, void *stream_b);

/* Pipelined models: makes `stream` wait (on the device; the host does not
 * block) for the outstanding stages of every call so far, after which their
 * logits are ordered on `stream` like any other result.  Needed before ending
 * a stream capture that contains pipelined forwards.  Does nothing for a model
 * that is not pipelined. */
REC_API rec_status rec_drain(rec_model *m, void *stream);

/* Per-stage timing.  rec_set_profiling(m, slots, period) with slots > 0 makes
 * rec_forward() bracket each stage with HIP events on its stream for every
 * period-th forward (counted from this call, starting with the first); the
 * j-th timed forward records into slot j % slots.  Event records cost a few
 * microseconds each on the device, hence the period.  slots = 0 switches it
 * off.  rec_stage_ms() waits for the events of `slot` and fills
 * ms[REC_NUM_STAGES]; REC_ERR_STATE if that slot has not been recorded.
 * With REC_OPT_OVERLAP_DENSE the first Bottom-FC stage is only the time the
 * caller's stream waited for Bottom-FC after pooling had finished, and the
 * second reads about zero.  An in-order forward whose Bottom-FC runs inside the
 * scan's second launch (a stack that fits the on-chip kernel) reports it under
 * REC_STAGE_SCAN and gives 0 for both Bottom-FC stages.  With REC_OPT_PIPELINE every stage is bracketed on
 * the stream it runs on (a stage's time then includes whatever shared the
 * device with it). */
REC_API rec_status rec_set_profiling(rec_model *m, int32_t slots, int32_t period);
REC_API rec_status rec_stage_ms(rec_model *m, int32_t slot, float *ms);

/* Text for a status; any other number gives "unknown status". */
REC_API const char *rec_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* REC_H */
