/*
 * rsr_dense.h - a comparator, not part of the RSR path: the same product out = v . A for a binary
 * {0,1} or ternary {-1,0,1} matrix computed on the same GPU from the bit-packed matrix itself, one
 * bit per entry and part (rows*cols/8 bytes per part: less than the RSR index, whose permutations
 * cost 16 bits per row and block).  It answers on one chip where RSR++ wins and where it loses
 * (Section 5 compares RSR with the standard product; the paper's related work names the Four
 * Russians method, which is what this kernel does with the rows: the sums of every group of four
 * activations are tabulated once per workgroup and a column takes one table entry per four rows).
 *
 * Conventions as in rsr.h: plain C types, HOST / DEVICE stated per pointer, RSR_OK or a negative
 * rsr_status, message through rsr_last_error().
 */
#ifndef RSR_DENSE_H_
#define RSR_DENSE_H_

#include <stdint.h>

#include "rsr.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rsr_dense rsr_dense; /* opaque; owns the bit planes and a buffer of partial sums on the device */

/* A: HOST, row-major rows x cols int8 in {-1,0,1} (any -1 makes it ternary: two bit planes).
 * rows, cols >= 1.  Returns NULL on error.  Synchronous. */
rsr_dense *rsr_dense_preprocess(const int8_t *A, int64_t rows, int64_t cols);

/* v: DEVICE [batch][rows] float (int8 for _i8); out: DEVICE [batch][cols] float (int32), fully
 * overwritten.  Asynchronous on `stream`; two kernels (partial sums per tile of 512 rows into the
 * handle's buffer, then their sum in a fixed order: results are reproducible).  Calls on one handle
 * must not overlap.  batch 1 .. 16. */
int rsr_dense_matvec(rsr_dense *h, const float *v, float *out, int batch, void *stream);
int rsr_dense_matvec_i8(rsr_dense *h, const int8_t *v, int32_t *out, int batch, void *stream);

/* bytes of the bit planes on the device (what one product reads) */
int64_t rsr_dense_table_bytes(const rsr_dense *h);

void rsr_dense_destroy(rsr_dense *h); /* NULL allowed */

#ifdef __cplusplus
}
#endif
#endif /* RSR_DENSE_H_ */
