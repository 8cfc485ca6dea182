/*
 * CPU oracle for the vector x binary/ternary-matrix product  out = v . A.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the correctness reference that the
 * HIP library is compared against; it is never part of the product path and
 * shares no code, header, table or helper with it.
 *
 * What it computes: the plain definition of the product (paper, Section 2.2,
 * Problem 1 / Problem 2, with the n x m footnote):
 *
 *     out[b][c] = sum_{r=0}^{rows-1} v[b][r] * A[r][c]
 *
 * for every batch lane b and every column c, where A is a row-major
 * rows x cols matrix with entries in {-1, 0, 1} (binary matrices use {0, 1}),
 * v[b] has `rows` entries and out[b] has `cols` entries.  The redundant-segment
 * method of the paper reaches exactly this value (Lemma 4.2 states the per-block
 * identity; Section 5.3 reports that the authors checked equality of results),
 * so the oracle is the definition written out: one pass over the rows, one
 * accumulator per column.  It builds no column blocks, permutations, segments or
 * folds.
 *
 * Precision: activations given as float are accumulated in double; activations
 * given as int8 are accumulated in int64 (no overflow is possible: |sum| <=
 * 127 * rows).
 *
 * The *_cols variants restrict the computation to a half-open column range; they
 * are the same loop on a stripe of columns and exist so that the timing harness
 * can run independent stripes on several host threads.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* out has batch*cols doubles; only columns [c_begin, c_end) of each lane are written. */
void rsr_oracle_matvec_f32_cols(const int8_t *A, int64_t rows, int64_t cols, const float *v,
                                int64_t batch, double *out, int64_t c_begin, int64_t c_end) {
  for (int64_t b = 0; b < batch; ++b) {
    double *acc = out + b * cols;
    const float *vb = v + b * rows;
    for (int64_t c = c_begin; c < c_end; ++c) acc[c] = 0.0;
    for (int64_t r = 0; r < rows; ++r) {
      const int8_t *Ar = A + r * cols;
      const double x = (double)vb[r];
      for (int64_t c = c_begin; c < c_end; ++c) acc[c] += x * (double)Ar[c];
    }
  }
}

void rsr_oracle_matvec_i8_cols(const int8_t *A, int64_t rows, int64_t cols, const int8_t *v,
                               int64_t batch, int64_t *out, int64_t c_begin, int64_t c_end) {
  for (int64_t b = 0; b < batch; ++b) {
    int64_t *acc = out + b * cols;
    const int8_t *vb = v + b * rows;
    for (int64_t c = c_begin; c < c_end; ++c) acc[c] = 0;
    for (int64_t r = 0; r < rows; ++r) {
      const int8_t *Ar = A + r * cols;
      const int64_t x = (int64_t)vb[r];
      for (int64_t c = c_begin; c < c_end; ++c) acc[c] += x * (int64_t)Ar[c];
    }
  }
}

/* Whole product, one thread. */
void rsr_oracle_matvec_f32(const int8_t *A, int64_t rows, int64_t cols, const float *v,
                           int64_t batch, double *out) {
  rsr_oracle_matvec_f32_cols(A, rows, cols, v, batch, out, 0, cols);
}

void rsr_oracle_matvec_i8(const int8_t *A, int64_t rows, int64_t cols, const int8_t *v,
                          int64_t batch, int64_t *out) {
  rsr_oracle_matvec_i8_cols(A, rows, cols, v, batch, out, 0, cols);
}

/* Returns 0 if every entry of A is in {-1,0,1}; otherwise 1 + the flat index of the first offender. */
int64_t rsr_oracle_check_entries(const int8_t *A, int64_t rows, int64_t cols) {
  for (int64_t i = 0; i < rows * cols; ++i)
    if (A[i] < -1 || A[i] > 1) return 1 + i;
  return 0;
}

/* ---- the same definition on `nthreads` column stripes (timing harness only) ---- */

typedef struct {
  const int8_t *A;
  int64_t rows, cols, batch, c_begin, c_end;
  const void *v;
  void *out;
  int is_f32;
} stripe_job;

static void *stripe_main(void *arg) {
  stripe_job *j = (stripe_job *)arg;
  if (j->is_f32)
    rsr_oracle_matvec_f32_cols(j->A, j->rows, j->cols, (const float *)j->v, j->batch, (double *)j->out,
                               j->c_begin, j->c_end);
  else
    rsr_oracle_matvec_i8_cols(j->A, j->rows, j->cols, (const int8_t *)j->v, j->batch, (int64_t *)j->out,
                              j->c_begin, j->c_end);
  return NULL;
}

/* Returns the number of threads actually used (>= 1), or -1 if a thread could not be started. */
static int run_stripes(const int8_t *A, int64_t rows, int64_t cols, const void *v, int64_t batch, void *out,
                       int nthreads, int is_f32) {
  if (nthreads < 1) nthreads = 1;
  if ((int64_t)nthreads > cols) nthreads = (int)(cols > 0 ? cols : 1);
  pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
  stripe_job *job = (stripe_job *)malloc(sizeof(stripe_job) * (size_t)nthreads);
  if (!tid || !job) { free(tid); free(job); return -1; }
  int started = 0, failed = 0;
  for (int t = 0; t < nthreads; ++t) {
    job[t].A = A; job[t].rows = rows; job[t].cols = cols; job[t].batch = batch;
    job[t].c_begin = cols * t / nthreads; job[t].c_end = cols * (t + 1) / nthreads;
    job[t].v = v; job[t].out = out; job[t].is_f32 = is_f32;
    if (pthread_create(&tid[t], NULL, stripe_main, &job[t]) != 0) { failed = 1; break; }
    ++started;
  }
  for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
  free(tid); free(job);
  return failed ? -1 : started;
}

int rsr_oracle_matvec_f32_mt(const int8_t *A, int64_t rows, int64_t cols, const float *v, int64_t batch,
                             double *out, int nthreads) {
  return run_stripes(A, rows, cols, v, batch, out, nthreads, 1);
}

int rsr_oracle_matvec_i8_mt(const int8_t *A, int64_t rows, int64_t cols, const int8_t *v, int64_t batch,
                            int64_t *out, int nthreads) {
  return run_stripes(A, rows, cols, v, batch, out, nthreads, 0);
}
