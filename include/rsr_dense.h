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

/*
 * rsr_dense_matvec_static - rsr_dense_matvec for callers that cannot allocate and want nothing
 * allocated on their behalf: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The partial sums go to a buffer that is part of the library's image on the
 * device (RSR_DENSE_STATIC_BYTES; every GPU the library runs on holds it until the process ends)
 * instead of the buffer the handle allocated at preprocess time.  The call allocates nothing and
 * frees nothing (no hipMalloc, hipFree or allocating library routine).
 *   Arguments and results (bit for bit) as rsr_dense_matvec.  The device of the handle must be
 *   current.  The buffer's address on a device is looked up once, at rsr_dense_preprocess on that
 *   device (else at the first call there).
 *   Fails with RSR_ERR_UNSUPPORTED when the partial sums, 4 * ceil(rows/512) * batch * cols bytes,
 *   exceed RSR_DENSE_STATIC_BYTES, with RSR_ERR_INVALID_ARGUMENT when another device is current.
 *   All calls on one GPU share the one buffer and it keeps what the last call left there (nothing
 *   needs to start at zero: a call reads only what it has written itself): calls that overlap on
 *   a GPU - other streams, other host threads, other handles - race.
 */
#define RSR_DENSE_STATIC_BYTES (4u << 20)
int rsr_dense_matvec_static(rsr_dense *h, const float *v, float *out, int batch, void *stream);

/* bytes of the bit planes on the device (what one product reads) */
int64_t rsr_dense_table_bytes(const rsr_dense *h);

void rsr_dense_destroy(rsr_dense *h); /* NULL allowed */

#ifdef __cplusplus
}
#endif
#endif /* RSR_DENSE_H_ */
