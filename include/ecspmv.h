/*
 * ecspmv.h -- C ABI of the MI355X-native batch-1 SpMV  y = W x  over EC-CSR.
 *
 * EC-CSR (paper, Section 6) stores a pruned FP16 weight matrix as dense g-grained blocks
 * found by hierarchical block extraction (Section 4, Algorithms 1 and 2) plus the
 * residual 1-grained rows, with 8-bit or 4-bit delta-encoded column indices (Section 6.2; EC-CSR-8 and
 * EC-CSR-4 of Section 8.2); 16-bit absolute columns can be asked for instead, for the ablation of Section 8.3.
 * ecspmv_build_* runs the offline phase on the host (Sections 4, 5, 6); ecspmv_run is the
 * online phase (Section 7): one HIP kernel launch on a caller-supplied stream.
 *
 * Conventions
 *  - Every function returns an int status: ECSPMV_OK (0) or a negative ECSPMV_ERR_* code.
 *    Nothing throws, aborts or prints.  Output arguments are untouched on error.
 *  - "host" / "device" in an argument's comment says which memory the pointer addresses.
 *  - FP16 data crosses the ABI as uint16_t IEEE 754 binary16 bit patterns.
 *  - A matrix entry is stored iff its bits are neither +0 nor -0 (bits & 0x7FFF != 0).
 *  - The handle owns host memory only.  The caller owns W, x, y and the device buffers and
 *    must keep a device image alive and unchanged while runs on it are in flight.
 *  - Streams are passed as void* (a hipStream_t; NULL = the default stream).
 *  - ecspmv_build_* may be called from several threads at once; a handle is read-only after
 *    ecspmv_upload and may then be used from several threads / streams, provided the runs
 *    write different y.
 */
#ifndef ECSPMV_H
#define ECSPMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ECSPMV_OK                 0
#define ECSPMV_ERR_INVALID       -1  /* NULL pointer, bad size, ld < n, unsorted / duplicate / out-of-range CSR column */
#define ECSPMV_ERR_UNSUPPORTED   -2  /* n > 65535, delta_bits not 4, 8 or 16, max_granularity not in {1,2,4,8,16}, too many rows,
                                        an option or call that does not exist for this kind of image */
#define ECSPMV_ERR_NOMEM         -3  /* host allocation failed */
#define ECSPMV_ERR_HIP           -4  /* a HIP call failed; ecspmv_last_hip_error() has its code */
#define ECSPMV_ERR_NOT_UPLOADED  -5  /* ecspmv_run before ecspmv_upload */
#define ECSPMV_ERR_TOO_SMALL     -6  /* caller's buffer is smaller than required */
#define ECSPMV_ERR_INTERNAL      -7  /* anything else that went wrong inside a host-side call (e.g. a worker thread could
                                        not be started); the handle or output is not produced */

typedef struct ecspmv_matrix ecspmv_matrix;     /* opaque: the host-side EC-CSR image of one matrix */
typedef struct ecspmv_csr ecspmv_csr;           /* opaque: plain CSR (comparison kernel) */

/* Options of the offline phase.  NULL, or a zeroed struct with struct_size set, gives the
 * defaults.  Fields beyond struct_size are taken as 0 (= default).
 * The paper leaves the clipping threshold of Section 5, the smallest useful block and the number of levels open.
 * Here they are not options: blocks are clipped into fixed units of 64 columns and residual rows into units of 16
 * entries (what a quarter of a wavefront, resp. a lane, handles per step), a block is useful from one unit on, and
 * the number of levels follows from max_granularity.  What can be chosen instead is how the launch is cut
 * (num_panels, threads_per_wg). */
typedef struct ecspmv_build_opts {
    uint32_t struct_size;     /* sizeof(ecspmv_build_opts) as the caller compiled it */
    int32_t  delta_bits;      /* width of a delta index (Section 6.2, range R_P = 2^bits): 8 (EC-CSR-8) or 4
                                 (EC-CSR-4, Section 8.2: zero fillers every 15 columns, blocks only where 64 shared
                                 columns follow one another within 15); 0 = 8.  16 = index compression off: every
                                 index is the 16-bit column itself, no fillers, no range limit on blocks (the first
                                 step of the ablation of Section 8.3, through the same kernel; FP16 values and one
                                 right-hand side only) */
    int32_t  max_granularity; /* largest block granularity g (rows per block, Section 4); 0 = 8 (4 for FP32 values);
                                 1 = no extraction */
    int32_t  max_rounds;      /* cap on extraction rounds per level (Algorithm 1, inner loop); 0 = 64 */
    int32_t  num_panels;      /* row panels = workgroups of the SpMV launch; 0 = auto (256; fewer for small m; more
                                 where few long rows would put more partial sums into a panel than LDS holds) */
    int32_t  num_threads;     /* host threads for the offline phase; 0 = hardware concurrency, at most 16 */
    int32_t  threads_per_wg;  /* workgroup size of the SpMV launch, multiple of 64 in [64,1024]; 0 = chosen at
                                 launch: 1024 for a lone SpMV, 512 inside a batch */
    uint64_t flags;           /* ECSPMV_FLAG_* */
} ecspmv_build_opts;

#define ECSPMV_FLAG_GLOBAL_MATCHING  1ull /* one panel for extraction: row matching over all rows as in Algorithm 2
                                             (the launch then has a single workgroup: for studies on small inputs) */
#define ECSPMV_FLAG_NO_REORDER       2ull /* keep blocks in extraction order instead of longest-first (Section 5) */
#define ECSPMV_FLAG_KEEP_SMALL_SETS  4ull /* keep a coarsest block set even if it holds under 1 % of the stored entries.
                                             Without the flag such a set is dropped (max_granularity is halved and the
                                             matrix encoded again): every set costs the launch a pipeline stage. */

#define ECSPMV_FLAG_CLUSTER_ROWS     8ull /* Before the panels are cut, bring rows that share columns together: the
                                             multi-level aggregation of Algorithm 1 (greedy row matching, Algorithm 2)
                                             is run over ALL rows, one matching round per level, up to groups of
                                             max_granularity rows; panels are cut from the rows listed group by group
                                             and y is stored through a row index table (the paper's row_indices,
                                             Section 6.1).  Blocks whose rows lie far apart in W are found this way
                                             (the paper matches over the whole matrix, Section 4); the price is build
                                             time quadratic in the number of rows. */

/* What ecspmv_stats reports (Section 8.2 storage study, Table 2 padding). */
typedef struct ecspmv_stats_t {
    uint32_t struct_size;
    int64_t  m, n, nnz;                /* stored entries of W */
    int64_t  image_bytes;              /* whole device image */
    int64_t  value_bytes;              /* values (FP16, or FP32 for an _f32 build) incl. padding */
    int64_t  delta_bytes;              /* delta indices (one or half a byte each) incl. padding */
    int64_t  meta_bytes;               /* headers, bases, row/slot tables */
    int64_t  slack_bytes;              /* alignment gaps and per-panel slack up to the common panel stride */
    int64_t  csr32_bytes;              /* 6*nnz + 4*(m+1): int32 columns + FP16 values + int32 row pointers (8*nnz with FP32 values) */
    int64_t  csr16_bytes;              /* 4*nnz + 4*(m+1): the same with int16 columns (6*nnz with FP32 values) */
    int64_t  nnz_by_g[5];              /* stored entries held at granularity 1, 2, 4, 8, 16 */
    int64_t  units_by_g[5];            /* [0] = residual lane units (16 elements), [t>=1] = 64-column units of g = 2^t */
    int64_t  pad_elements;             /* explicit zeros: gap fillers + row-tail alignment (residual rows only) */
    int64_t  gap_pad_elements;         /* of those, zeros inserted because a column gap exceeded the largest delta (255 or 15) */
    int32_t  num_panels, threads_per_wg;
    int64_t  panel_stride, meta_stride, lds_bytes;
    int64_t  max_panel_bytes, min_panel_bytes;
    double   x_access_cost;            /* sum over stored entries of 1/g(e): the paper's x-access objective with L = 1 */
    double   build_seconds;
    int64_t  delta_hist[9];            /* residual deltas: 0, 1, 2-3, 4-7, ..., 64-127, 128-255 */
    int32_t  delta_bits, value_bits;   /* delta width the image was built with; 16 (FP16) or 32 (FP32) values */
} ecspmv_stats_t;

/* ---- offline phase (host) -------------------------------------------------------------------------- */

/* Sections 4 (hierarchical block extraction, Algorithms 1 and 2), 5 (clipping, ordering) and 6 (EC-CSR encoding).
 * Build from a dense row-major FP16 matrix.  W: host, m rows of n entries, row stride ld >= n (elements).
 * Caller keeps W.  *out receives a new handle (free with ecspmv_destroy).  m, n >= 1; n <= 65535. */
int ecspmv_build_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld,
                       const ecspmv_build_opts *opts, ecspmv_matrix **out);

/* The same from CSR (the form pruned weights usually come in).
 * rowptr: host, m+1 entries, rowptr[0] = 0, non-decreasing; col: host, strictly increasing
 * within a row, in [0, n); val: host FP16 bits (entries equal to +-0 are dropped). */
int ecspmv_build_csr(const int64_t *rowptr, const int32_t *col, const uint16_t *val,
                     int64_t m, int64_t n, const ecspmv_build_opts *opts, ecspmv_matrix **out);

/* The same for FP32 values (the paper's other precision: its evaluation, Sections 8.1 and 8.2, covers FP32 and FP16): W, and later x and y of ecspmv_run, are
 * float.  An entry is stored iff it is neither +0 nor -0.  The image keeps 4-byte values; everything else (block
 * extraction, delta indices, layout) is unchanged.  csr32_bytes / csr16_bytes of the stats then count 4-byte values. */
int ecspmv_build_dense_f32(const float *W, int64_t m, int64_t n, int64_t ld,
                           const ecspmv_build_opts *opts, ecspmv_matrix **out);
int ecspmv_build_csr_f32(const int64_t *rowptr, const int32_t *col, const float *val,
                         int64_t m, int64_t n, const ecspmv_build_opts *opts, ecspmv_matrix **out);

void ecspmv_destroy(ecspmv_matrix *A);          /* NULL is a no-op */

/* The figures of the paper's storage study (Section 8.2: bytes against CSR-32 / CSR-16; Table 2: padding) and of its
 * objective (Section 4: x-access cost) for this image.  Fill *st (st->struct_size must be set by the caller). */
int ecspmv_stats(const ecspmv_matrix *A, ecspmv_stats_t *st);

/* Decode the image back to coordinate triples by walking it the way the kernel does (columns by the recurrence of
 * Section 6.2, I_k = I_0 + sum of deltas; values through the inverse of the permutation of Section 6.3.2), dropping
 * padding.
 * Call with rows = cols = vals = NULL to get *nnz; then with host arrays of *nnz entries each (capacity
 * passed in *nnz).  Output order is image order (not sorted). */
int ecspmv_decode(const ecspmv_matrix *A, int64_t *nnz, int32_t *rows, int32_t *cols, uint16_t *vals);
/* The same for a matrix built with ecspmv_build_*_f32 (each of the two refuses the other kind: ECSPMV_ERR_INVALID). */
int ecspmv_decode_f32(const ecspmv_matrix *A, int64_t *nnz, int32_t *rows, int32_t *cols, float *vals);

/* The block sets (Algorithm 1's output): for every extracted unit, its granularity, its g original rows and
 * its 64 columns.  Call with NULLs to get the counts (*n_units, *n_rows = sum of g over units).
 * g: n_units entries; unit_rows: concatenated row lists; unit_cols: 64 entries per unit.  Host arrays. */
int ecspmv_block_sets(const ecspmv_matrix *A, int64_t *n_units, int64_t *n_rows,
                      int32_t *g, int32_t *unit_rows, int32_t *unit_cols);

/* ---- device image ---------------------------------------------------------------------------------- */

/* Library plumbing, no passage of the paper: size of the device image in bytes (a multiple of 256). */
int ecspmv_device_bytes(const ecspmv_matrix *A, size_t *bytes);

/* Library plumbing, no passage of the paper: copy the image into host memory (host_dst: host, >=
 * ecspmv_device_bytes): for inspection, tests and caching.  Layout of the bytes (version 3; all little-endian):
 *   [image header, 256 B: magic "ECSR", version, m, n, num_panels, threads_per_wg, panel_stride, meta_stride,
 *    max_slots, lds_bytes (uint32 each), image_bytes, nnz (uint64), delta_bits, value_bits (uint32)]
 *   [panel 0] ... [panel P-1], panel_stride bytes apart, then 4 KB of zeros.
 *   panel = [header, 32 uint32: first row, rows, block slots, residual lane units, residual row segments, byte
 *            offsets of the tables and arrays that follow, units per granularity]
 *           [tables: first slot of each row (uint16), first residual lane unit of each row (uint32), output row of
 *            each row (uint32: the paper's row_indices), per block unit its base column and the slots of its rows
 *            (uint16), per residual chunk a 64-bit mask of lanes that start a row segment, per row segment its
 *            base column]
 *           [residual chunks: 64 lane units of 16 entries each: their indices, then their values, 128 bits per lane
 *            and load]
 *           [per granularity 16, 8, 4, 2: the units' indices (64 per unit), then their values (g per column,
 *            permuted so that a 16-lane group loads 128 bits per lane)].
 * The authoritative description, with every offset, is the format header that ships with the library's sources. */
int ecspmv_export_image(const ecspmv_matrix *A, void *host_dst, size_t bytes);

/* Library plumbing, no passage of the paper (which builds the format once, ahead of inference: Section 8.1).
 * Copy the image into d_buf (device, 256-byte aligned, >= ecspmv_device_bytes, allocated and owned by the
 * caller) on `stream`, and remember d_buf in the handle.  Returns after the copy has completed. */
int ecspmv_upload(ecspmv_matrix *A, void *d_buf, size_t bytes, void *stream);

/* ---- online phase ---------------------------------------------------------------------------------- */

/* The online phase (Section 7; the product is the one of Sections 1 and 2.2: Y = W X with a single column).
 * y = W x (overwrites y; every one of the m entries is written).  d_x: device, n FP16, 2-byte aligned
 * (16-byte alignment takes the faster staging path).  d_y: device, m FP16.  x and y must not overlap.
 * For a matrix built with ecspmv_build_*_f32, x and y are FP32 (4-byte aligned).
 * Asynchronous on `stream`: exactly one kernel launch, no allocation (host or device), no memset, no host
 * synchronisation, nothing that can throw.
 * x must be finite: padding zeros are multiplied with x entries. */
int ecspmv_run(const ecspmv_matrix *A, const void *d_x, void *d_y, void *stream);

/* No passage of the paper (its kernel is launched once per matrix): the same for `count` independent SpMVs in one
 * kernel launch per 16 matrices (a launch also ends where the
 * delta width or the value width changes from one matrix to the next): y_i = W_i x_i.  As, d_xs, d_ys:
 * host arrays of `count` handles / device pointers.  The SpMVs must not depend on one another (no y_i may be an
 * x_j of the same call).  Meant for the projections of a decoder layer that do not depend on one another:
 * workgroups of the next matrix start while the last ones of the previous matrix drain, which removes the launch
 * and ramp-up cost between small SpMVs.  Every y_i has the bits a lone ecspmv_run would give. */
int ecspmv_run_batch(const ecspmv_matrix *const *As, const void *const *d_xs, void *const *d_ys, int32_t count,
                     void *stream);

/* Y = W X for nb right-hand sides at once (the paper's problem statement, Section 2.1: Y (M,N) = W (M,K) X (K,N), here
 * with N = nb in {1, 2, 4, 8}; the paper leaves small N > 1 as future work, Section 10).  d_X: device, n rows of nb
 * FP16 (row-major: the nb values that belong to one column of W are adjacent), d_Y: device, m rows of nb FP16; every
 * entry of Y is written.  The deltas are decoded once and every stored entry of W is read once for all nb products.
 * One kernel launch, asynchronous on `stream`, no allocation.  nb = 1 is ecspmv_run.  Where 2*n*nb bytes of X plus
 * 4*nb bytes per partial sum do not fit the LDS of a compute unit, the call runs as 2 or 4 launches of nb/2 or nb/4
 * right-hand sides each (same X, Y and results; the image is then read once per launch).
 * For a matrix built with ecspmv_build_*_f32, X and Y are FP32 (and 4*n*nb bytes of X count for LDS).
 * ECSPMV_ERR_UNSUPPORTED if the image holds a 16-grained block set, or an 8-grained one with FP32 values (the default
 * build options produce neither), or if not even two right-hand sides fit LDS; ECSPMV_ERR_INVALID for other nb. */
int ecspmv_run_multi(const ecspmv_matrix *A, const void *d_X, void *d_Y, int32_t nb, void *stream);

/* ---- comparison: plain CSR (int32 column index + FP16 value per entry, one wavefront per row) ------- */
/* The CSR-32 format the paper's Section 8.2 measures storage against, with a kernel of its own (not one of the
 * paper's comparison libraries). */

int ecspmv_csr_build_dense(const uint16_t *W, int64_t m, int64_t n, int64_t ld, ecspmv_csr **out);
void ecspmv_csr_destroy(ecspmv_csr *C);
int ecspmv_csr_device_bytes(const ecspmv_csr *C, size_t *bytes);
int ecspmv_csr_upload(ecspmv_csr *C, void *d_buf, size_t bytes, void *stream);
int ecspmv_csr_run(const ecspmv_csr *C, const void *d_x, void *d_y, void *stream);

/* ---- measurement aid: streaming-read ceiling -------------------------------------------------------- */

/* Reads `bytes` (multiple of 16) from d_buf (device, 16-byte aligned) with 128-bit loads from `num_wg`
 * workgroups of 1024 threads and writes one 32-bit checksum per workgroup to d_out (device, num_wg words).
 * One launch, asynchronous on `stream`. */
int ecspmv_stream_read(const void *d_buf, size_t bytes, void *d_out, int32_t num_wg, void *stream);

/* The same bytes read the way a launch of the SpMV kernel reads an image: workgroup w of `num_wg` workgroups of
 * `threads_per_wg` (256, 512 or 1024) threads reads the w-th contiguous slice of the buffer, two 128-bit loads in
 * flight per lane.  The fastest plain read found for 20-50 MB in a launch of its own: the time of this launch is the
 * floor under a lone SpMV launch that reads as many bytes.  d_out: device, num_wg words.  One launch, asynchronous. */
int ecspmv_stream_read_sliced(const void *d_buf, size_t bytes, void *d_out, int32_t num_wg, int32_t threads_per_wg,
                              void *stream);

/* `count` launches, one after the other on `stream`, of `num_wg` workgroups of `threads_per_wg` (a multiple of 64,
 * <= 1024) threads that read nothing and store one word per workgroup to d_out (device, num_wg words): what a launch
 * costs by itself when launches follow one another on a stream (submitted from one host loop, so that the host is
 * not what is timed).  Asynchronous. */
int ecspmv_empty_launch(void *d_out, int32_t num_wg, int32_t threads_per_wg, int32_t count, void *stream);

/* ---- errors ---------------------------------------------------------------------------------------- */

const char *ecspmv_strerror(int status);
int ecspmv_last_hip_error(void);                /* hipError_t of the most recent failed HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* ECSPMV_H */
