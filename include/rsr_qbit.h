/*
 * rsr_qbit.h - the product out = v . A for a matrix whose entries have q bits, by the route the
 * paper's appendix "Generalization" names: the matrix is written as a weighted sum of binary
 * matrices, each is preprocessed and multiplied by the binary RSR++ path of rsr.h, and the results
 * are combined.  The decomposition used here is the two's complement one,
 *
 *     A = sum_{i=0}^{q-2} 2^i B_i  -  2^(q-1) B_{q-1},     B_i[r][c] = bit i of A[r][c],
 *
 * q binary matrices (the appendix speaks of recursive use of Proposition 2.1 and of a larger number
 * of matrices; any decomposition into weighted binary matrices gives the same product, and this one
 * has the fewest).  One product costs q launches of the binary kernel: the first writes v . B_0,
 * the others add their weighted products (rsr_matvec_acc).
 *
 * Conventions as in rsr.h: plain C types, HOST / DEVICE stated per pointer, RSR_OK or a negative
 * rsr_status, message through rsr_last_error().
 */
#ifndef RSR_QBIT_H_
#define RSR_QBIT_H_

#include <stdint.h>

#include "rsr.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rsr_qbit rsr_qbit; /* opaque; owns q handles of rsr.h */

/* A: HOST, row-major rows x cols int8, every entry in -2^(q-1) .. 2^(q-1)-1.  q: 2 .. 8.
 * rows, cols, k as for rsr_preprocess.  Returns NULL on error (an entry out of range is
 * RSR_ERR_INVALID_ARGUMENT).  Synchronous; A is not retained. */
rsr_qbit *rsr_qbit_preprocess(const int8_t *A, int64_t rows, int64_t cols, int k, int q);

/* v: DEVICE [batch][rows]; out: DEVICE [batch][cols], fully overwritten.  Asynchronous on `stream`
 * (q launches per row tile, in order).  Float: every plane's product is rounded as in rsr_matvec,
 * the weights are powers of two (exact), the q-1 additions round once each;
 * |out - exact| <= 1e-5 * 2^(q-1) * sum_i |v_i|.  int8: exact; |sum| <= 127 * 128 * rows < 2^31. */
int rsr_qbit_matvec(rsr_qbit *h, const float *v, float *out, int batch, void *stream);
int rsr_qbit_matvec_i8(rsr_qbit *h, const int8_t *v, int32_t *out, int batch, void *stream);

/* planes (= q) and the bytes of all their tables on the device */
int rsr_qbit_planes(const rsr_qbit *h);
int64_t rsr_qbit_table_bytes(const rsr_qbit *h);

void rsr_qbit_destroy(rsr_qbit *h); /* NULL allowed */

#ifdef __cplusplus
}
#endif
#endif /* RSR_QBIT_H_ */
