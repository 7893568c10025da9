/*
 * rec_synth.h - device-side filling of synthetic embedding tables.
 *
 * Production embedding tables (Table I: 1M-20M rows each, up to ~100 tables)
 * are not public; benchmarks use procedural values instead: element
 * (table, row, col) is a pure function of (seed, table, row, col) so that a
 * table set larger than host memory can be filled in place on the device and
 * any row can be recomputed elsewhere.
 *
 *   n     = ((table << 32) + row) * 1024 + col
 *   z     = the n-th output of a SplitMix64 stream seeded with `seed`
 *           (Steele, Lea, Flood, OOPSLA 2014): mix64(seed + (n+1) * 0x9e3779b97f4a7c15)
 *   value = ((z >> 40) - 2^23) * (0.05f * 2^-23)      one fp32 multiply
 *   stored as fp32, or rounded to fp16 (nearest even)
 *
 * This is an input generator, not part of the forward pass.
 */
#ifndef REC_SYNTH_H
#define REC_SYNTH_H

#include <stdint.h>
#include "rec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Fills dev_rows ([rows][emb_dim] of `dtype`, device memory) on `stream`.
 * REC_ERR_ARG on null / non-positive sizes / emb_dim > 1024 / rows >= 2^32. */
REC_API rec_status rec_synth_fill_table(void *dev_rows, int32_t dtype, uint64_t seed, int32_t table,
                                int64_t rows, int32_t emb_dim, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* REC_SYNTH_H */
