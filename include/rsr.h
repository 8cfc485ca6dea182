/*
 * rsr.h - C ABI of the MI355X (gfx950) library for the Redundant Segment Reduction
 * vector x matrix product  out = v . A  with a fixed binary {0,1} or ternary {-1,0,1}
 * weight matrix A (arXiv 2411.06360), in its RSR++ form.
 *
 * The two phases follow the paper's statement of the problem (Section 2.2): the weight
 * matrix is known in advance and is preprocessed once (Section 3, Algorithm 1); activation
 * vectors arrive later and are multiplied with the preprocessed index (Section 4,
 * Algorithms 2 and 3).  A is rows x cols, v multiplies from the left: len(v) = rows,
 * len(out) = cols (the n x m footnote of Section 2.2).
 *
 * Conventions
 *   - Plain C types only.  Every pointer argument says whether it is HOST or DEVICE memory.
 *   - All functions return RSR_OK (0) or a negative rsr_status, except rsr_preprocess which
 *     returns NULL on failure and rsr_last_error which returns a string.  After any failure
 *     rsr_last_error() describes it (thread-local, valid until the next call on that thread).
 *   - No exceptions cross this boundary.  The library keeps no global state besides the
 *     error string; handles are independent of each other.
 *   - A handle belongs to the HIP device that was current when rsr_preprocess was called.
 *     Calls on one handle from several host threads must be serialised by the caller.
 */
#ifndef RSR_H_
#define RSR_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rsr_status {
  RSR_OK = 0,
  RSR_ERR_INVALID_ARGUMENT = -1, /* null pointer, size out of range, entry outside {-1,0,1}, bad handle */
  RSR_ERR_UNSUPPORTED = -2,      /* valid request this build cannot serve (an index too large for its 32-bit offsets) */
  RSR_ERR_HIP = -3,              /* a HIP runtime call failed; the message carries hipGetErrorString */
  RSR_ERR_OUT_OF_MEMORY = -4     /* host allocation failed */
} rsr_status;

typedef struct rsr_handle rsr_handle; /* opaque; owns the device-resident index of one matrix */

/*
 * rsr_preprocess - Algorithm 1 (Section 3.4) for a binary matrix, applied to both halves of
 * the split A = B(1) - B(2) of Proposition 2.1 when A is ternary.
 *
 *   A     HOST pointer, row-major rows x cols int8, entries in {0,1} (binary) or {-1,0,1}
 *         (ternary).  The kind is inferred: any -1 makes the matrix ternary (two parts,
 *         B(1) = [A == 1] and B(2) = [A == -1]); otherwise there is one part, B = A.
 *         A is only read during the call and is not retained.
 *   rows  1 .. 65534   (row indices are stored in 16 bits; one value is reserved).  A matrix with
 *         more than 32768 rows is indexed as two row tiles of equal height, each with its own
 *         permutations and segmentations; a product then takes one launch per tile and the
 *         tiles' results add up (the product is linear in the rows).  rsr_export_block returns
 *         the index of the whole matrix either way.
 *   cols  >= 1
 *   k     block width, 1 .. 16.  Column block i holds columns i*k .. min((i+1)*k, cols)-1
 *         (Definition 3.1); the last block may be narrower.
 *
 * For every part and every k-column block the call builds the row permutation that sorts the
 * rows by their binary value, first column most significant (Definition 3.2; equal rows stay in
 * ascending row order) and the boundaries of the groups of equal rows (the full segmentation,
 * Section 3.3), packs them for the GPU and uploads them to the current HIP device.
 * The packed form is a layout choice, not a different index: rsr_export_block returns the
 * permutation and the full segmentation in the paper's form.  Rows whose value in a block is 0
 * contribute nothing to that block (row 0 of Bin_[k] is all zeros) and are not stored.
 *
 * Returns a handle, or NULL on error (invalid argument, entry outside {-1,0,1}, HIP failure,
 * out of memory).  Synchronous: the tables are resident on the device when it returns.
 */
rsr_handle *rsr_preprocess(const int8_t *A, int64_t rows, int64_t cols, int k);

/*
 * rsr_preprocess_device - Algorithm 1 (Section 3.4) run on the GPU, for a matrix that is already in
 * device memory (weights loaded there): row values per column block (Definition 3.2), the stable
 * counting sort that yields the permutation (the bucket sort in the proof of Theorem 3.6), the full
 * segmentation (Section 3.3) and the packing all happen on the device; the host only turns per-window
 * entry counts into the schedule.  The handle is used exactly like one from rsr_preprocess and encodes
 * the same index (rsr_export_block returns identical tables).  Both builders order the rows inside
 * every group of equal rows so that the gathers of the product spread over the LDS banks; their
 * searches differ, so the two packed streams may differ in that order (and float results in their
 * summation order), not in the index or in the speed of the product.
 *
 *   A     DEVICE pointer, row-major rows x cols int8 in {-1,0,1}; read during the call only.
 *   rows, cols, k   as for rsr_preprocess.
 * Returns a handle, or NULL on error.  Synchronous; allocates temporary device memory of about
 * 4 bytes per row and column block and part, plus 4 * 2^k bytes per column block and part.
 */
rsr_handle *rsr_preprocess_device(const int8_t *A, int64_t rows, int64_t cols, int k);

/*
 * rsr_matvec - the RSR++ product (Section 4: segmented sums of Eq. SS2, then the fold of
 * Section 4.3 / Algorithm 3 per block; ternary result = (v . B(1)) - (v . B(2)),
 * Proposition 2.1), for float activations with float accumulation.
 *
 *   v      DEVICE pointer, row-major [batch][rows] float, 4-byte aligned; read only.
 *   out    DEVICE pointer, row-major [batch][cols] float; every element is overwritten.
 *          Must not overlap v.  Both stay owned by the caller.
 *   batch  >= 1 independent vectors sharing the index (lane b of out = v[b] . A).
 *   stream a hipStream_t passed as void* (NULL = the default stream).
 *
 * Asynchronous: the work is enqueued on `stream` and the call returns without synchronising;
 * it allocates no memory and is safe to capture in a HIP graph.  The order of the float
 * additions differs from a row-by-row sum but is fixed (no floating-point atomics), so a result
 * is reproducible from run to run; it satisfies |out - exact| <= 1e-5 * sum_i |v_i| for
 * finite inputs of ordinary magnitude.
 *
 * Errors: RSR_ERR_INVALID_ARGUMENT (null pointer, batch < 1 or > 65535), RSR_ERR_HIP (launch
 * failure).  Every row count that rsr_preprocess accepts is served.
 */
int rsr_matvec(rsr_handle *h, const float *v, float *out, int batch, void *stream);

/*
 * rsr_matvec_i8 - the same product for int8 activations with int32 accumulation; the result
 * is exact (|sum| <= 128 * rows < 2^31) and identical from run to run.
 *
 *   v    DEVICE pointer, row-major [batch][rows] int8.
 *   out  DEVICE pointer, row-major [batch][cols] int32, 4-byte aligned; fully overwritten.
 * Other arguments, asynchrony and errors as for rsr_matvec.
 */
int rsr_matvec_i8(rsr_handle *h, const int8_t *v, int32_t *out, int batch, void *stream);

/*
 * rsr_matvec_multi / rsr_matvec_multi_i8 - several products v_j . A_j as ONE launch: the products
 * are independent (Section 2.2 states the problem for one matrix; a transformer layer applies several
 * fixed matrices per step, Section 5.3) and share the device, each with its own handle, activations
 * and results.  Use it for matrices whose inputs are ready together (the q/k/v projections of one
 * activation, gate and up), where separate launches would each pay the start of a kernel.
 *
 *   jobs    HOST pointer to njobs records (read during the call only); in job j, `h` is a handle,
 *           `v` a DEVICE pointer [batch][rows_j] (float, or int8 for _i8) and `out` a DEVICE pointer
 *           [batch][cols_j] (float, or int32), as for rsr_matvec.  Buffers of different jobs must
 *           not overlap, except that several jobs may read the same v.
 *   njobs   1 .. 8
 *   batch   >= 1, the same for every job
 *   stream  as for rsr_matvec
 *
 * Asynchronous, allocates nothing, results bit-identical to separate rsr_matvec calls.
 * Errors: RSR_ERR_INVALID_ARGUMENT (null pointers, njobs or batch out of range, handles of different
 * devices), RSR_ERR_UNSUPPORTED (a handle with more than 32768 rows: use rsr_matvec), RSR_ERR_HIP.
 */
typedef struct rsr_job {
  rsr_handle *h;
  const void *v;
  void *out;
} rsr_job;
int rsr_matvec_multi(const rsr_job *jobs, int njobs, int batch, void *stream);
int rsr_matvec_multi_i8(const rsr_job *jobs, int njobs, int batch, void *stream);

/*
 * rsr_matvec_acc / rsr_matvec_acc_i8 - out += scale * (v . A): the product of rsr_matvec, scaled,
 * added to what `out` holds instead of replacing it.  This is the combining step of a weighted sum
 * of binary or ternary matrices, which is how Proposition 2.1 builds a ternary product from two
 * binary ones and how Appendix "Generalization" extends the method to matrices with more bits per
 * entry (rsr_qbit.h does that with these calls).
 *   v, out, batch, stream   as for rsr_matvec / rsr_matvec_i8; `out` must hold valid numbers
 *   scale                   finite float; any int32 for _i8 (the caller keeps the sums within int32)
 * Float: out[c] = out[c] + scale * p[c], with p the product as rsr_matvec computes it (rounded),
 * then one fused multiply-add or a rounded multiplication and a rounded addition.  int8: exact.
 * Asynchronous, allocates nothing.
 * Errors as rsr_matvec; RSR_ERR_INVALID_ARGUMENT for a scale that is not finite.
 */
int rsr_matvec_acc(rsr_handle *h, const float *v, float *out, float scale, int batch, void *stream);
int rsr_matvec_acc_i8(rsr_handle *h, const int8_t *v, int32_t *out, int32_t scale, int batch, void *stream);

/*
 * rsr_set_step2 - which form of step 2 (the product of the segmented sums u with Bin_[k]) later
 * rsr_matvec / rsr_matvec_i8 calls on this handle use:
 *   RSR_STEP2_FOLD   the RSR++ halving fold of Section 4.3 / Algorithm 3, O(2^k) (the default);
 *   RSR_STEP2_PLAIN  step 2 of Algorithm 2 as printed: the plain product u . Bin_[k], O(k 2^k).
 * Both give the same product (bit-identical for int8; the float sums are taken in another order).
 * The plain form exists to measure what the fold is worth (Appendix F.2); rsr_matvec_multi always folds.
 */
enum { RSR_STEP2_FOLD = 0, RSR_STEP2_PLAIN = 1 };
int rsr_set_step2(rsr_handle *h, int step2);

/*
 * rsr_model_k - the block width that minimises the paper's cost of RSR++, (rows + 2^k) / k per
 * column (Section 4.3, the optimal-k equation for RSR++), over k_min .. k_max.  A formula, no device
 * work; returns k, or a negative rsr_status.
 *
 * rsr_autotune_k - the empirical choice (the paper picks k by measurement too, Appendix F.1): for every
 * k in k_min .. k_max the matrix is preprocessed on the current device and `reps` products of `batch`
 * float vectors are timed (after warm-up calls, with events on the default stream).
 *   A, rows, cols   as for rsr_preprocess (HOST)
 *   cold            nonzero: rotate over enough copies of the index (at most 16) that a call does not
 *                   find its tables in the last-level cache; zero: one copy, called back to back
 *   best_k          HOST out: the k with the shortest product
 *   us_per_k        HOST out or NULL: k_max - k_min + 1 durations in microseconds per product
 * Synchronous; allocates and frees device memory of its own.  Returns RSR_OK or a negative status.
 */
int rsr_model_k(int64_t rows, int k_min, int k_max);
int rsr_autotune_k(const int8_t *A, int64_t rows, int64_t cols, int batch, int k_min, int k_max,
                   int reps, int cold, int *best_k, double *us_per_k);

/* rsr_destroy - frees the device tables and the handle.  NULL is allowed.  The caller must make
 * sure that no enqueued product still uses the handle (synchronise the stream first). */
void rsr_destroy(rsr_handle *h);

/* rsr_last_error - message of the last failure on the calling thread ("" if none). */
const char *rsr_last_error(void);

/*
 * rsr_info - sizes of the index as stored on the device (Theorem 3.6 bounds them by
 * O(rows*cols/k) words).  The byte counts are what one product reads from device memory and are
 * the figures a bandwidth measurement must use.
 */
typedef struct rsr_info_t {
  int64_t rows, cols;
  int32_t k;                /* block width asked for */
  int32_t parts;            /* 1 = binary, 2 = ternary (B(1), B(2)) */
  int64_t nblocks;          /* ceil(cols / k) */
  int32_t last_block_width; /* cols - (nblocks-1)*k, in 1..k */
  int32_t lo_bits, hi_bits; /* how the k value bits are split for the two-level fold */
  int64_t stored_rows;      /* row indices stored over all blocks and parts (value-0 rows left out) */
  int64_t segments;         /* stored groups of equal rows (long groups are cut into several) */
  int64_t work_units;       /* scheduling units (part of the segments of 512 consecutive row values) */
  int64_t index_bytes;      /* row indices of the packed permutation, padding included */
  int64_t segment_bytes;    /* value ids of the segments, padding included */
  int64_t schedule_bytes;   /* unit descriptors and per-block unit ranges */
  int64_t table_bytes;      /* index_bytes + segment_bytes + schedule_bytes */
  int32_t device;           /* HIP device ordinal that holds the tables */
  int32_t compute_units;    /* of that device */
  int32_t row_tiles;        /* 1, or 2 for more than 32768 rows: launches per product */
  int32_t reserved;
} rsr_info_t;

int rsr_info(const rsr_handle *h, rsr_info_t *info); /* info: HOST pointer */

/*
 * rsr_export_block - the index of one column block in the paper's form, decoded from the
 * tables resident on the device (they are copied back to the host on first use).
 *
 *   part   0 = B(1) (or B for a binary matrix), 1 = B(2)
 *   block  0 .. nblocks-1
 *   sigma  HOST pointer to `rows` int32, or NULL.  sigma[p] = the row at sorted position p,
 *          counted from 0: rows ascend by value, equal rows by row number (Definition 3.2,
 *          Example 3.3; add 1 for the paper's numbering).
 *   L      HOST pointer to 2^w + 1 int32, or NULL, where w is the width of this block
 *          (k, or last_block_width for the last block).  L[j] = number of rows whose value
 *          is below j, so L[0..2^w-1] is the full segmentation of Section 3.3 counted from 0,
 *          and L[2^w] = rows closes the last group.
 *
 * Meant for tests and tooling; not a fast path.
 */
int rsr_export_block(rsr_handle *h, int part, int64_t block, int32_t *sigma, int32_t *L);

/* ------------------------------------------------------------------------------------------
 * Host-only entry points: the index builder without a device.  They run the same code as
 * rsr_preprocess up to, but not including, the upload, so that the tables can be checked on a
 * machine with no GPU.  They compute no product.
 * ------------------------------------------------------------------------------------------ */
typedef struct rsr_host_index rsr_host_index; /* opaque; owns host memory only */

/* Arguments and errors as rsr_preprocess; no HIP call is made.  NULL on error. */
rsr_host_index *rsr_host_pack(const int8_t *A, int64_t rows, int64_t cols, int k);

/* NULL is allowed. */
void rsr_host_free(rsr_host_index *x);

/* As rsr_info; device = -1 and compute_units = 0. */
int rsr_host_info(const rsr_host_index *x, rsr_info_t *info);

/* As rsr_export_block, decoding the host copy of the packed tables. */
int rsr_host_export_block(const rsr_host_index *x, int part, int64_t block, int32_t *sigma, int32_t *L);

/*
 * rsr_host_streams - read-only views of the packed streams of one row tile exactly as they would
 * be uploaded (layout: see csrc/rsr_format.h).  Pointers are HOST memory owned by x and valid until
 * rsr_host_free.  Any output pointer may be NULL.
 *   tile                  0 .. row_tiles-1
 *   stream / n_stream     uint16 elements of the unit streams (row indices, then flag words)
 *   units / n_units       32-byte unit descriptors
 *   blk_unit              nblocks + 1 uint32 offsets into units
 *   tile_row0 / tile_rows first row and height of the tile (row indices count from tile_row0)
 */
int rsr_host_streams(const rsr_host_index *x, int tile, const uint16_t **stream, int64_t *n_stream,
                     const void **units, int64_t *n_units, const uint32_t **blk_unit,
                     int64_t *tile_row0, int64_t *tile_rows);

#ifdef __cplusplus
}
#endif
#endif /* RSR_H_ */
