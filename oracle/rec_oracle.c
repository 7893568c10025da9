/*
 * CPU oracle for the forward pass of a DLRM-class recommendation model.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the forward pass computes; it exists so that a device implementation can be
 * checked against it.  Only tests, a smoke check and the CPU-baseline leg of a
 * benchmark may call it.  It shares no code, header, table or helper with any
 * device implementation.
 *
 * The model (Sec. II-A, Fig. 2(a), Table I): a SparseNet of embedding tables,
 * each looked up with a variable number of row ids per sample whose rows are
 * pooled by summation ("Gather-Reduce", SparseLengthsSum; Sec. VI-B), and a
 * DenseNet made of a Bottom-FC stack on the dense features and a Predict-FC
 * stack that depends on both (Sec. III-A).  The paper defers the rest of the
 * definition to the DLRM model it cites: the pooled vectors and the Bottom-FC
 * output are combined by pairwise dot products, and the Predict-FC output is
 * one click-through logit per sample.
 *
 * Every step below is the textbook definition written as scalar loops with
 * fp64 accumulators, in the order the definition states.  No blocking, fusion
 * or reordering.  Stored operands (fp16 / fp32 rows, fp32 weights) are widened
 * exactly.  Parity pins live in the CPU test-suite: integer identities of the
 * scan; single-id bags, all-ones tables, row-id tables, one-hot matrix
 * products for pooling; numpy fp64 products for one layer; symmetry,
 * squared norms and constant vectors for the interaction; an independent
 * nested-loop Python forward for the whole path.
 *
 * Readings taken where the paper is silent:
 *   - pairwise dot interaction over the T+1 vectors [bottom output, pooled
 *     table 0, ..., pooled table T-1]; strict lower triangle in row-major
 *     order (1,0), (2,0), (2,1), (3,0) ...; bottom output concatenated first;
 *   - ReLU after every Bottom-FC layer and after every Predict-FC layer but
 *     the last, which is linear and yields the logit; sigmoid is separate;
 *   - every layer has a bias;
 *   - an empty bag pools to the zero vector, duplicate ids count with
 *     multiplicity, an id outside [0, rows) contributes zero and is reported.
 *
 * Second model shape (Table I, row MT-WnD: 26 tables, one lookup per table,
 * no pooling, no Bottom-FC, Predict-FC = N towers of 1024-512-256):
 * oracle_forward_towers().  Readings: the looked-up vectors and the dense
 * part are concatenated, dense part first, with no interaction operator
 * (Table I has none for this row); each of the N task towers reads that same
 * vector, has ReLU on its hidden layers and ends in a linear one-output
 * layer, one logit per task; the stack of lookups is the general pooled sum,
 * of which one id per bag is the special case (Sec. VI-B: lookup only, no
 * Gather-Reduce).  Pins: numpy's concatenate, rows reproduced bit for bit,
 * tower-wise reduction to single layers, the independent nested-loop forward.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1 };
enum { ORACLE_EXACT = 0, ORACLE_BF16_MIRROR = 1 };

/* Threads used by the loops over samples (1 = serial).  Returns the count in
 * effect; without OpenMP that is always 1. */
int oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* number formats                                                      */
/* ------------------------------------------------------------------ */

/* IEEE 754 binary16 bit pattern -> its exact value. */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* subnormal: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

/* Nearest bfloat16 (8 exponent bits, 7 fraction bits) to x, ties to even,
 * returned as a double.  x is first rounded to fp32, as the device holds
 * activations in fp32 before narrowing.  Finite inputs only. */
double oracle_round_bf16(double x)
{
    float f = (float)x;
    if (f == 0.0f || !isfinite(f))
        return (double)f;
    int e;
    double fr = frexp((double)f, &e);              /* f = fr * 2^e, 0.5 <= |fr| < 1 */
    /* bf16 keeps 8 significant bits: fr * 2^8 rounded to an integer. */
    double scaled = fr * 256.0;
    double r = nearbyint(scaled);                   /* default mode: ties to even */
    return ldexp(r, e - 8);
}

/* ------------------------------------------------------------------ */
/* S0: offsets                                                         */
/* ------------------------------------------------------------------ */

/* off[k] = sum of len[0..k-1], k = 0..n.  Returns -1 if a length is negative
 * (first such position in *bad), else 0. */
int oracle_offsets(const int32_t *len, int64_t n, int64_t *off, int64_t *bad)
{
    int64_t acc = 0;
    int rc = 0;
    off[0] = 0;
    for (int64_t k = 0; k < n; ++k) {
        if (len[k] < 0 && rc == 0) {
            rc = -1;
            if (bad) *bad = k;
        }
        acc += len[k] > 0 ? len[k] : 0;
        off[k + 1] = acc;
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* S1: embedding-bag pooling (SparseLengthsSum)                        */
/* ------------------------------------------------------------------ */

static double table_elem(const void *table, int dtype, int64_t row, int D, int d)
{
    if (dtype == ORACLE_F16)
        return oracle_half_to_double(((const uint16_t *)table)[row * D + d]);
    return (double)((const float *)table)[row * D + d];
}

/*
 * P[b][t][d] = sum over the bag (t, b) of E_t[id][d], ids in bag order.
 * lengths and indices are table-major: bag (t, b) is entry t*B + b.
 * P is [B][T][D] in fp64; the caller rounds if it wants fp32.
 * abs_sum (optional, same shape) receives sum |E_t[id][d]|, the scale against
 * which a summation-order error is judged.
 * Returns the number of ids outside [0, rows[t]); *first_bad gets the position
 * (in `indices`) of the first one.
 */
int64_t oracle_pool(const void *const *tables, int dtype, const int64_t *rows,
                    int T, int D, int B, const int32_t *indices,
                    const int32_t *lengths, double *P, double *abs_sum,
                    int64_t *first_bad)
{
    int64_t n = (int64_t)T * B;
    int64_t *off = (int64_t *)malloc((size_t)(n + 1) * sizeof(int64_t));
    int64_t nbad = 0;
    oracle_offsets(lengths, n, off, NULL);
    if (first_bad) *first_bad = -1;
    /* ids outside the table, in position order */
    for (int t = 0; t < T; ++t) {
        for (int64_t k = off[(int64_t)t * B]; k < off[(int64_t)(t + 1) * B]; ++k) {
            int64_t id = indices[k];
            if (id < 0 || id >= rows[t]) {
                if (nbad == 0 && first_bad) *first_bad = k;
                ++nbad;
            }
        }
    }
    for (int t = 0; t < T; ++t) {
#pragma omp parallel for schedule(static)
        for (int b = 0; b < B; ++b) {
            int64_t k0 = off[(int64_t)t * B + b], k1 = off[(int64_t)t * B + b + 1];
            double *out = P + ((int64_t)b * T + t) * D;
            double *aout = abs_sum ? abs_sum + ((int64_t)b * T + t) * D : NULL;
            for (int d = 0; d < D; ++d) {
                double acc = 0.0, aacc = 0.0;
                for (int64_t k = k0; k < k1; ++k) {
                    int64_t id = indices[k];
                    if (id < 0 || id >= rows[t])
                        continue;
                    double v = table_elem(tables[t], dtype, id, D, d);
                    acc += v;
                    aacc += fabs(v);
                }
                out[d] = acc;
                if (aout) aout[d] = aacc;
            }
        }
    }
    free(off);
    return nbad;
}

/* ------------------------------------------------------------------ */
/* S2 / S4: one fully connected layer                                  */
/* ------------------------------------------------------------------ */

/*
 * y[b][o] = act( sum_i W[o][i] * x[b][i] + bias[o] ),  act = ReLU or identity.
 * x is [B][n_in] fp64, W is [n_out][n_in] fp32 row-major, y is [B][n_out] fp64.
 * mode ORACLE_EXACT uses W and x as given.  ORACLE_BF16_MIRROR first rounds
 * every weight and every input activation to bfloat16 (bias stays fp32), the
 * precision a bf16 matrix unit is fed with; accumulation stays fp64.
 */
void oracle_fc(const double *x, const float *W, const float *bias, int B,
               int n_in, int n_out, int relu, int mode, double *y)
{
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int o = 0; o < n_out; ++o) {
            double acc = 0.0;
            for (int i = 0; i < n_in; ++i) {
                double w = (double)W[(int64_t)o * n_in + i];
                double a = x[(int64_t)b * n_in + i];
                if (mode == ORACLE_BF16_MIRROR) {
                    w = oracle_round_bf16(w);
                    a = oracle_round_bf16(a);
                }
                acc += w * a;
            }
            acc += (double)bias[o];
            if (relu && acc < 0.0)
                acc = 0.0;
            y[(int64_t)b * n_out + o] = acc;
        }
    }
}

/* ------------------------------------------------------------------ */
/* S3: pairwise-dot feature interaction                                */
/* ------------------------------------------------------------------ */

/*
 * Z[b] = X[b] X[b]^T with X[b] = [x0[b]; P[b][0]; ...; P[b][T-1]]  ((T+1) x D).
 * Z is [B][T+1][T+1]; the full matrix, diagonal included, for inspection.
 */
void oracle_gram(const double *x0, const double *P, int B, int T, int D, double *Z)
{
    int V = T + 1;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < V; ++i) {
            const double *xi = i == 0 ? x0 + (int64_t)b * D
                                      : P + ((int64_t)b * T + (i - 1)) * D;
            for (int j = 0; j < V; ++j) {
                const double *xj = j == 0 ? x0 + (int64_t)b * D
                                          : P + ((int64_t)b * T + (j - 1)) * D;
                double acc = 0.0;
                for (int d = 0; d < D; ++d)
                    acc += xi[d] * xj[d];
                Z[((int64_t)b * V + i) * V + j] = acc;
            }
        }
    }
}

/*
 * out[b] = [ x0[b] (D values), Z[b][i][j] for i = 1..T, j = 0..i-1 ]
 * width D + T(T+1)/2.
 */
void oracle_interact(const double *x0, const double *P, int B, int T, int D,
                     double *out)
{
    int V = T + 1;
    int64_t width = D + (int64_t)T * (T + 1) / 2;
    double *Z = (double *)malloc((size_t)B * V * V * sizeof(double));
    oracle_gram(x0, P, B, T, D, Z);
    for (int b = 0; b < B; ++b) {
        double *o = out + (int64_t)b * width;
        for (int d = 0; d < D; ++d)
            o[d] = x0[(int64_t)b * D + d];
        int64_t p = D;
        for (int i = 1; i < V; ++i)
            for (int j = 0; j < i; ++j)
                o[p++] = Z[((int64_t)b * V + i) * V + j];
    }
    free(Z);
}

double oracle_sigmoid(double x)
{
    return 1.0 / (1.0 + exp(-x));
}

/* ------------------------------------------------------------------ */
/* whole forward                                                       */
/* ------------------------------------------------------------------ */

/*
 * dense [B][F] fp32; tables / indices / lengths as in oracle_pool;
 * bottom_widths has n_bottom+1 entries (F ... D), top_widths n_top+1 entries
 * (D + T(T+1)/2 ... 1); bottom_W[i], top_W[i] are [out][in] fp32.
 * Outputs (each may be NULL): pooled [B][T][D], bottom_out [B][D],
 * interact [B][D + T(T+1)/2], logits [B], all fp64.
 * Returns 0, or -1 on a width chain that does not fit the model.
 */
int oracle_forward(const float *dense, const void *const *tables, int dtype,
                   const int64_t *rows, int T, int D, int B,
                   const int32_t *indices, const int32_t *lengths,
                   int n_bottom, const int32_t *bottom_widths,
                   const float *const *bottom_W, const float *const *bottom_b,
                   int n_top, const int32_t *top_widths,
                   const float *const *top_W, const float *const *top_b,
                   int mode, double *pooled, double *bottom_out,
                   double *interact, double *logits)
{
    int64_t width = D + (int64_t)T * (T + 1) / 2;
    if (bottom_widths[n_bottom] != D || top_widths[0] != width ||
        top_widths[n_top] != 1)
        return -1;

    int maxw = 1;
    for (int i = 0; i <= n_bottom; ++i)
        if (bottom_widths[i] > maxw) maxw = bottom_widths[i];
    for (int i = 0; i <= n_top; ++i)
        if (top_widths[i] > maxw) maxw = top_widths[i];

    double *P = (double *)malloc((size_t)B * T * D * sizeof(double));
    double *h0 = (double *)malloc((size_t)B * maxw * sizeof(double));
    double *h1 = (double *)malloc((size_t)B * maxw * sizeof(double));

    /* SparseNet */
    oracle_pool(tables, dtype, rows, T, D, B, indices, lengths, P, NULL, NULL);

    /* Bottom-FC: ReLU after every layer */
    int F = bottom_widths[0];
    for (int64_t i = 0; i < (int64_t)B * F; ++i)
        h0[i] = (double)dense[i];
    for (int l = 0; l < n_bottom; ++l) {
        oracle_fc(h0, bottom_W[l], bottom_b[l], B, bottom_widths[l],
                  bottom_widths[l + 1], 1, mode, h1);
        double *tmp = h0; h0 = h1; h1 = tmp;
    }
    if (bottom_out)
        memcpy(bottom_out, h0, (size_t)B * D * sizeof(double));

    /* interaction; h0 = bottom output [B][D] -> h1 = [B][width] */
    oracle_interact(h0, P, B, T, D, h1);
    /* The interaction output is what the Predict-FC matrix unit is fed with:
     * the mirror narrows it here, whatever layer consumes it. */
    if (mode == ORACLE_BF16_MIRROR)
        for (int64_t i = 0; i < (int64_t)B * width; ++i)
            h1[i] = oracle_round_bf16(h1[i]);
    if (interact)
        memcpy(interact, h1, (size_t)B * width * sizeof(double));
    { double *tmp = h0; h0 = h1; h1 = tmp; }

    /* Predict-FC: ReLU on all layers but the last.  The last layer has one
     * output, a dot product per sample rather than a matrix product, so the
     * bf16 mirror leaves its weights and inputs un-narrowed. */
    for (int l = 0; l < n_top; ++l) {
        int last = l + 1 == n_top;
        oracle_fc(h0, top_W[l], top_b[l], B, top_widths[l], top_widths[l + 1],
                  !last, last ? ORACLE_EXACT : mode, h1);
        double *tmp = h0; h0 = h1; h1 = tmp;
    }
    if (logits)
        memcpy(logits, h0, (size_t)B * sizeof(double));
    if (pooled)
        memcpy(pooled, P, (size_t)B * T * D * sizeof(double));

    free(P); free(h0); free(h1);
    return 0;
}

/* ------------------------------------------------------------------ */
/* concatenation model with N towers (Table I, MT-WnD row)             */
/* ------------------------------------------------------------------ */

/*
 * out[b] = [ x0[b] (w0 values), P[b][0][:], ..., P[b][T-1][:] ],
 * width w0 + T * D.  No products between the vectors.
 */
void oracle_concat(const double *x0, int w0, const double *P, int B, int T,
                   int D, double *out)
{
    int64_t width = w0 + (int64_t)T * D;
    for (int b = 0; b < B; ++b) {
        double *o = out + (int64_t)b * width;
        for (int i = 0; i < w0; ++i)
            o[i] = x0[(int64_t)b * w0 + i];
        for (int t = 0; t < T; ++t)
            for (int d = 0; d < D; ++d)
                o[w0 + (int64_t)t * D + d] = P[((int64_t)b * T + t) * D + d];
    }
}

/*
 * Forward of the concatenation model.  Inputs as in oracle_forward, except:
 *   n_bottom may be 0: bottom_widths then has the single entry F and the
 *     dense part of the concatenation is the dense features themselves;
 *   the Predict-FC stack exists n_towers times with the same widths
 *     top_widths (n_top + 1 entries: w0 + T*D ... 1) and its own weights:
 *     top_W[k * n_top + l] is layer l of tower k.
 * Outputs (each may be NULL): pooled [B][T][D], bottom_out [B][w0],
 * concat [B][w0 + T*D], logits [B][n_towers], all fp64.
 * Returns 0, or -1 on a width chain that does not fit.
 */
int oracle_forward_towers(const float *dense, const void *const *tables,
                          int dtype, const int64_t *rows, int T, int D, int B,
                          const int32_t *indices, const int32_t *lengths,
                          int n_bottom, const int32_t *bottom_widths,
                          const float *const *bottom_W,
                          const float *const *bottom_b, int n_towers,
                          int n_top, const int32_t *top_widths,
                          const float *const *top_W, const float *const *top_b,
                          int mode, double *pooled, double *bottom_out,
                          double *concat, double *logits)
{
    int w0 = bottom_widths[n_bottom];
    int64_t width = w0 + (int64_t)T * D;
    if (n_bottom < 0 || n_towers < 1 || n_top < 1 || top_widths[0] != width ||
        top_widths[n_top] != 1)
        return -1;

    int64_t maxw = width;
    for (int i = 0; i <= n_bottom; ++i)
        if (bottom_widths[i] > maxw) maxw = bottom_widths[i];
    for (int i = 0; i <= n_top; ++i)
        if (top_widths[i] > maxw) maxw = top_widths[i];

    double *P = (double *)malloc((size_t)B * T * D * sizeof(double));
    double *h0 = (double *)malloc((size_t)B * maxw * sizeof(double));
    double *h1 = (double *)malloc((size_t)B * maxw * sizeof(double));
    double *z = (double *)malloc((size_t)B * width * sizeof(double));

    oracle_pool(tables, dtype, rows, T, D, B, indices, lengths, P, NULL, NULL);

    int F = bottom_widths[0];
    for (int64_t i = 0; i < (int64_t)B * F; ++i)
        h0[i] = (double)dense[i];
    for (int l = 0; l < n_bottom; ++l) {
        oracle_fc(h0, bottom_W[l], bottom_b[l], B, bottom_widths[l],
                  bottom_widths[l + 1], 1, mode, h1);
        double *tmp = h0; h0 = h1; h1 = tmp;
    }
    if (bottom_out)
        memcpy(bottom_out, h0, (size_t)B * w0 * sizeof(double));

    oracle_concat(h0, w0, P, B, T, D, z);
    /* What the towers' matrix units are fed with: the mirror narrows it here. */
    if (mode == ORACLE_BF16_MIRROR)
        for (int64_t i = 0; i < (int64_t)B * width; ++i)
            z[i] = oracle_round_bf16(z[i]);
    if (concat)
        memcpy(concat, z, (size_t)B * width * sizeof(double));

    for (int k = 0; k < n_towers; ++k) {
        memcpy(h0, z, (size_t)B * width * sizeof(double));
        for (int l = 0; l < n_top; ++l) {
            int last = l + 1 == n_top;
            /* the one-output layer is a dot product: never narrowed */
            oracle_fc(h0, top_W[k * n_top + l], top_b[k * n_top + l], B,
                      top_widths[l], top_widths[l + 1], !last,
                      last ? ORACLE_EXACT : mode, h1);
            double *tmp = h0; h0 = h1; h1 = tmp;
        }
        if (logits)
            for (int b = 0; b < B; ++b)
                logits[(int64_t)b * n_towers + k] = h0[b];
    }
    if (pooled)
        memcpy(pooled, P, (size_t)B * T * D * sizeof(double));

    free(P); free(h0); free(h1); free(z);
    return 0;
}
