/*
 * cnr.h -- C ABI of libcnr: the GPU hot path of an incremental, quantized checkpoint encoder for
 * embedding tables (Check-N-Run, arXiv 2010.08679), written for AMD MI355X (gfx950).
 *
 * The path, in call order:
 *   cnr_clear_bitmap   start a new tracking window (Section 5.1: a new baseline, or every
 *                      interval under the consecutive-increment policy)
 *   cnr_mark_touched   once per training iteration and table: record which rows were looked up
 *                      (Section 5.1.1, tracking bit-vector)
 *   cnr_compact_dirty  at checkpoint time: the list of rows whose bit is set, i.e. the
 *                      incremental view (Section 5.1)
 *   cnr_quantize_rows  gather those rows and quantize each one with uniform per-row
 *                      quantization F_Q (Section 5.2, Approach 1), the range being the row's
 *                      min/max, the symmetric range, or the greedy-searched one (Approach 3);
 *                      codes are packed densely in the same kernel
 *   cnr_pack           dense packing alone, for codes produced one per byte
 *   cnr_restore_rows   resume: de-quantize (x = scale * x_q + zero_point) and write the rows
 *                      back over a stale baseline table (Sections 5.1 and 6.2)
 * Around the path:
 *   cnr_*_batch        every stage for several tables per call (Sections 2.1, 4.1)
 *   cnr_compact_dirty_noalloc   the compaction for callers that cannot allocate: no scratch argument
 *   cnr_quant_error    the l2 error metric of Section 5.2
 *   cnr_select_greedy_params   greedy parameters by profiling a sample (Section 5.2)
 *   cnr_host_writer_*, cnr_encode_to_host   chunked encode into host memory with the copy of one
 *                      chunk overlapping the encode of the next (Sections 4.4, 5.2)
 *   cnr_restore_from_host   the way back: the restore reads pinned host memory itself over the host
 *                      link, or takes it chunk by chunk with the copy overlapping the restore
 *   cnr_policy_*       the incremental-checkpoint policies (Section 5.1), host only
 *   cnr_select_bits    the code width for an expected number of resumes (Section 6.2.1), host only
 *
 * General rules
 *   - Every pointer argument is a DEVICE pointer owned by the caller unless its comment says
 *     "host".  The library allocates nothing on the hot path; cnr_create allocates a few bytes of
 *     device and pinned host memory for the error counters, cnr_destroy frees them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues work on it and returns at once; the status returned covers argument checks and
 *     launch failures.  Conditions found on the device (look-up indices outside the table, more
 *     dirty rows than `capacity`, a row id outside the table) never fault: the offending item is
 *     skipped, a counter / flag in the context is updated, and cnr_poll_errors reports it.
 *   - Row counts that are only known on the device (the output of cnr_compact_dirty) are passed
 *     on as device pointers, so that a checkpoint needs no host synchronisation between its
 *     stages.  `n_max` bounds the count from the host side (it sizes the launch and the output
 *     buffers); the kernels process min(*n_dev, n_max) rows.
 *   - A context belongs to one device and must not be used from two host threads at once.
 *   - No C++ type, exception or torch object crosses this boundary.
 *
 * Data layout
 *   table     float [n_rows][dim], row-major, 16-byte aligned base, dim % 4 == 0
 *   bitmap    uint32 [cnr_bitmap_words(n_rows)]; row i is bit (i & 31) of word (i >> 5);
 *             8-byte aligned base; bits at positions >= n_rows are ignored
 *   row_ids   uint32 [n], strictly ascending when produced by cnr_compact_dirty; 16-byte aligned
 *             base where cnr_quantize_rows or cnr_restore_rows reads it
 *   scale,    float [n]: scale = (hi - lo) / (2^bits - 1) and bias = lo (the zero_point) of
 *   bias      row_ids[k]'s range [lo, hi]; 16-byte aligned base where cnr_restore_rows reads them
 *   packed    uint8 [n][cnr_packed_row_bytes(dim, bits)], rows back to back without padding; per
 *             row one little-endian bit stream in which element j occupies stream bits
 *             [j*bits, (j+1)*bits), least-significant code bit first (stream bit t is bit
 *             (t & 7) of byte (t >> 3)); 16-byte aligned base
 *   codes_u8  uint8 [n][dim], one code per byte; 16-byte aligned base where cnr_quantize_rows
 *             writes it
 */
#ifndef CNR_H
#define CNR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cnr_ctx cnr_ctx; /* opaque */

typedef enum {
    CNR_OK = 0,
    CNR_E_INVALID = 1,     /* NULL where a pointer is required, bad enum value, n_rows >= 2^32 */
    CNR_E_BITS = 2,        /* bits not in {2, 3, 4, 8} */
    CNR_E_DIM = 3,         /* dim == 0, dim % 4 != 0, dim > CNR_MAX_DIM, or dim*bits % 8 != 0 */
    CNR_E_ALIGN = 4,       /* a base pointer is not aligned as the layout section requires */
    CNR_E_CAPACITY = 5,    /* device: more dirty rows than `capacity` (poll only) */
    CNR_E_INDEX_RANGE = 6, /* device: look-up indices outside [0, n_rows) were skipped (poll only) */
    CNR_E_ROW_ID = 7,      /* device: a row id >= n_rows was skipped (poll only) */
    CNR_E_HIP = 8,         /* a HIP runtime call failed; see cnr_last_hip_error */
    CNR_E_TOO_LARGE = 9,   /* a size beyond the fixed maximum of an entry point that allocates nothing */
    CNR_E_HOST_MEMORY = 10 /* a host buffer that a kernel was to access itself is not pinned, device-accessible memory */
} cnr_status;

typedef enum { CNR_IDX_I32 = 0, CNR_IDX_I64 = 1 } cnr_index_type;

typedef enum {
    CNR_RANGE_MINMAX = 0,   /* asymmetric: [min x, max x]            (Section 5.2, Approach 1) */
    CNR_RANGE_GREEDY = 1,   /* adaptive asymmetric, greedy search    (Section 5.2, Approach 3) */
    CNR_RANGE_SYMMETRIC = 2 /* [-max|x|, +max|x|]                    (Section 5.2, Approach 1) */
} cnr_range_mode;

/* Parameters of the greedy range search (Section 5.2, Approach 3).  step_size is the row's
 * original range divided by num_bins; the search performs
 *     n_iter = min(ceil(ratio * num_bins - 1e-4), num_bins - 1)
 * iterations, i.e. it stops once the removed part reaches `ratio` of the original range and
 * never lets the range collapse.  Each iteration tries [lo + step, hi] and [lo, hi - step], keeps
 * the one with the smaller squared l2 error (the lower bound moves only on a strictly smaller
 * error); the result is the range of the iteration with the smallest error, the un-shrunk range
 * included (an earlier iteration wins ties). */
typedef struct {
    uint32_t num_bins;
    float ratio;
} cnr_greedy_params;

#define CNR_MAX_DIM 4096u

/* Flags reported by cnr_poll_errors. */
#define CNR_FLAG_CAPACITY 1u
#define CNR_FLAG_ROW_ID 2u

/* ---- context ---------------------------------------------------------------------------- */

/* Creates a context on HIP device `device` (host call; allocates the error counters).
 * *out receives the context (host pointer, owned by the caller until cnr_destroy). */
cnr_status cnr_create(cnr_ctx **out, int device);
cnr_status cnr_destroy(cnr_ctx *ctx);

/* Sizes (pure host arithmetic, no GPU involved). */
size_t cnr_bitmap_words(uint64_t n_rows);               /* ceil(n_rows / 32) */
size_t cnr_packed_row_bytes(uint32_t dim, int bits);    /* dim*bits/8; 0 if not a whole number */
size_t cnr_scratch_bytes(uint64_t n_rows);              /* scratch cnr_compact_dirty needs */
size_t cnr_mark_scratch_bytes(uint64_t n_rows);         /* optional scratch of cnr_mark_touched: one byte per
                                                           row, at least 5 MiB for a table of 1.3 M rows or
                                                           more, four bytes per row below that; never
                                                           decreases as n_rows grows */
uint32_t cnr_greedy_iterations(uint32_t num_bins, float ratio); /* n_iter as defined above */

/* ---- tracking (Section 5.1.1) ----------------------------------------------------------- */

/* Zeroes bitmap[0 .. cnr_bitmap_words(n_rows)) with a fill kernel (safe under graph capture). */
cnr_status cnr_clear_bitmap(cnr_ctx *ctx, uint32_t *bitmap, uint64_t n_rows, void *stream);

/* For every t < n_indices with 0 <= indices[t] < n_rows sets bit indices[t] of `bitmap`
 * (in place; bits accumulate over calls until the bitmap is cleared).  Duplicates are expected.
 * Indices outside the table are skipped and counted in the context.
 *   indices  int32 or int64 [n_indices] as `type` says; naturally aligned
 *   n_rows   < 2^32
 *   scratch  NULL, or cnr_mark_scratch_bytes(n_rows) bytes, 16-byte aligned, ALL ZERO before the
 *            first call that uses it (hipMemset once after allocating); every call leaves it all
 *            zero again, so one buffer sized for the largest table can serve all tables marked on
 *            the same stream.  With a scratch buffer, long index streams are marked without one
 *            device-scope atomic per index: through bitmap slices held in on-chip memory whose
 *            partial bitmaps pass through the scratch (tables of up to about 21 M rows, when
 *            several tables are marked in one call), or through one flag byte per row with
 *            repeated look-ups dropped on chip (larger tables, and one or two tables marked
 *            alone), each followed by a fold into the bitmap.  Short streams, and all streams
 *            when scratch is NULL, use atomic ORs on the bitmap directly.  The resulting bitmap is
 *            the same whichever way. */
cnr_status cnr_mark_touched(cnr_ctx *ctx, uint32_t *bitmap, uint64_t n_rows, const void *indices,
                            uint64_t n_indices, cnr_index_type type, void *scratch, void *stream);

/* ---- incremental view (Section 5.1) ------------------------------------------------------ */

/* Writes the ascending list of set-bit positions below n_rows to row_ids and their number to
 * *n_dirty_dev.  If there are more than `capacity`, only the first `capacity` ids are written,
 * *n_dirty_dev still receives the full count and CNR_FLAG_CAPACITY is raised in the context.
 *   row_ids      uint32 [capacity]
 *   n_dirty_dev  uint64 [1] (device)
 *   scratch      cnr_scratch_bytes(n_rows) bytes, 8-byte aligned, contents irrelevant */
cnr_status cnr_compact_dirty(cnr_ctx *ctx, const uint32_t *bitmap, uint64_t n_rows,
                             uint32_t *row_ids, uint64_t capacity, uint64_t *n_dirty_dev,
                             void *scratch, void *stream);

/* cnr_compact_dirty for callers that cannot allocate device memory and have none to pass as scratch:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and device-side conditions as cnr_compact_dirty, minus `scratch`: the per-tile counts of the
 * compaction go to a fixed array that is part of the loaded library's device image
 * (CNR_NOALLOC_SCRATCH_BYTES on every GPU the library runs on, held until the process ends), whose
 * address on the context's device cnr_create looked up once.  The call allocates and frees nothing.
 *   n_rows   at most CNR_NOALLOC_MAX_ROWS, else CNR_E_TOO_LARGE is returned and nothing is launched
 * Every context of one GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * contexts, two host threads) race and give wrong lists; calls on one stream are ordered and safe.
 * The array keeps the last call's contents; nothing in it has to start at zero (the count kernel
 * writes every entry the scatter kernel reads). */
#define CNR_NOALLOC_MAX_ROWS (1ull << 30)
#define CNR_NOALLOC_SCRATCH_BYTES ((CNR_NOALLOC_MAX_ROWS / 16384u) * 4u + 8u)
cnr_status cnr_compact_dirty_noalloc(cnr_ctx *ctx, const uint32_t *bitmap, uint64_t n_rows,
                                     uint32_t *row_ids, uint64_t capacity, uint64_t *n_dirty_dev,
                                     void *stream);

/* ---- quantization (Section 5.2) ---------------------------------------------------------- */

/* For k < n = min(*n_dev, n_max): gathers row r = row_ids[k] (r = k when row_ids is NULL) of
 * `table`, finds X_min / X_max, selects the range [lo, hi] by `mode`, and quantizes the row with
 * F_Q(x, lo, hi) at `bits` bits: scale = (hi - lo) / (2^bits - 1), code = round-half-even
 * ((clip(x, lo, hi) - lo) / scale) in fp32, all codes 0 when scale == 0.
 *   n_dev     uint64 [1] device pointer, or NULL meaning n = n_max
 *   greedy    host pointer, read during the call; required for CNR_RANGE_GREEDY only
 *   scale, bias        float [n_max], required
 *   row_min, row_max   float [n_max] or NULL: X_min / X_max before any shrinking (-0.0 reported
 *                      as +0.0)
 *   codes_u8  uint8 [n_max][dim] or NULL: the codes one per byte
 *   packed    uint8 [n_max][cnr_packed_row_bytes] or NULL: the codes packed (fused path)
 * Rows must hold finite values with |x| < FLT_MAX / 2; anything else gives unspecified codes
 * (never a fault).  A row id >= n_rows is skipped and CNR_FLAG_ROW_ID raised. */
cnr_status cnr_quantize_rows(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                             const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                             int bits, cnr_range_mode mode, const cnr_greedy_params *greedy,
                             float *scale, float *bias, float *row_min, float *row_max,
                             uint8_t *codes_u8, uint8_t *packed, void *stream);

/* Packs codes_u8 [n][dim] (values < 2^bits) into `packed` as laid out above. */
cnr_status cnr_pack(cnr_ctx *ctx, const uint8_t *codes_u8, const uint64_t *n_dev, uint64_t n_max,
                    uint32_t dim, int bits, uint8_t *packed, void *stream);

/* ---- restore (Sections 5.1, 5.2, 6.2) ----------------------------------------------------- */

/* For k < n = min(*n_dev, n_max): table[row_ids[k]][j] = scale[k] * code_kj + bias[k] (fp32, one
 * rounding for the product and one for the sum) for all j; rows not listed keep their contents.
 * row_ids == NULL means row k.  Row ids must not repeat.  A row id >= n_rows is skipped and
 * CNR_FLAG_ROW_ID raised. */
cnr_status cnr_restore_rows(cnr_ctx *ctx, float *table, uint64_t n_rows, uint32_t dim,
                            const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                            int bits, const uint8_t *packed, const float *scale,
                            const float *bias, void *stream);

/* ---- error metric (Section 5.2: l2 error of a quantized vector, mean l2 error of a checkpoint) - */

/* For k < n = min(*n_dev, n_max): err[k] = || X_k - Q_k ||_2, where X_k is row row_ids[k] (row k
 * when row_ids is NULL) of `table` and Q_k the same row as cnr_restore_rows would write it from
 * (packed, scale, bias); element differences, their squares and the sum are taken in fp64.  When
 * mean_out is not NULL, *mean_out receives (1/n) * sum_k err[k], added up in a fixed order (0 when
 * n == 0).  Rows with an id >= n_rows get err 0 and raise CNR_FLAG_ROW_ID.
 *   err       double [n_max], required
 *   mean_out  double [1] (device) or NULL */
cnr_status cnr_quant_error(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                           const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max, int bits,
                           const uint8_t *packed, const float *scale, const float *bias, double *err,
                           double *mean_out, void *stream);

/* ---- greedy parameters by profiling (Section 5.2, "Parameter selection") ------------------------
 *
 * Quantizes the rows `sample_ids` of `table` (a uniform sample of the checkpoint drawn by the caller;
 * the paper samples 0.001 % of it) with min/max quantization and with the greedy search at every
 * num_bins of `bins_grid` (ratio 1), keeps the num_bins at which the improvement of the mean l2
 * error tapers off, then does the same over `ratio_grid` at that num_bins.  "Tapers off" is read as:
 * with I(p) = 1 - E(p) / E_minmax, the first p of the grid with I(p) >= (1 - taper) * max I (the
 * first grid value when nothing improves on min/max).  Grids are taken in the order given.
 * Synchronizes `stream` once per grid point (each mean is read back).
 *   sample_ids  device uint32 [n_sample], 16-byte aligned
 *   bins_grid   host uint32 [n_bins], ratio_grid host float [n_ratios]; at most CNR_SELECT_MAX_GRID each
 *   taper       in [0, 1), e.g. 0.05
 *   scratch     device, cnr_select_scratch_bytes(n_sample, dim, bits) bytes, 16-byte aligned
 *   chosen      host out
 *   report      host out or NULL: double [1 + n_bins + n_ratios]: the mean l2 error of min/max, of
 *               each num_bins, of each ratio */
#define CNR_SELECT_MAX_GRID 64u
size_t cnr_select_scratch_bytes(uint64_t n_sample, uint32_t dim, int bits);
cnr_status cnr_select_greedy_params(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                                    const uint32_t *sample_ids, uint64_t n_sample, int bits,
                                    const uint32_t *bins_grid, uint32_t n_bins, const float *ratio_grid,
                                    uint32_t n_ratios, double taper, void *scratch, cnr_greedy_params *chosen,
                                    double *report, void *stream);

/* ---- several tables per launch (Section 2.1: a GPU holds many embedding tables; Section 4.1: a
 *      checkpoint covers every table of the GPU's shard) ------------------------------------------
 *
 * One cnr_table_job describes the buffers of one table; the *_batch calls take a host array of
 * them (read during the call) and do for every job what the single-table call of the same name
 * does.  Where a call is short -- the per-iteration mark of a few ten thousand indices, the clear,
 * the compaction -- the jobs run side by side in one launch per kernel (and per CNR_MAX_BATCH
 * jobs), which is what the batch calls are for; the encode and restore kernels, which are bound by
 * memory bandwidth and sweep a table best with the whole GPU, take up to CNR_MAX_BATCH jobs per
 * launch as well and work through them one after the other without a gap (small tables, rows of at
 * most 64 MB at `capacity`, and large ones in launches of their own kind; the greedy search and
 * row lengths other than 16, 32, 64, 128 and 256 one job per launch).  Results are identical to
 * those of the single-table calls.  Buffers of different jobs
 * of one call must not overlap (mark scratch included: one per job).  Every field has the meaning, layout and alignment of the
 * argument of the same name of the single-table call; a call reads only the fields listed for it.
 *   cnr_clear_bitmap_batch    bitmap, n_rows
 *   cnr_mark_touched_batch    bitmap, n_rows, indices, n_indices, mark_scratch (all jobs one index type)
 *   cnr_compact_dirty_batch   bitmap, n_rows, row_ids, capacity, n_dirty_dev, compact_scratch
 *   cnr_quantize_rows_batch   table, n_rows, row_ids, n_dirty_dev (as n_dev, may be NULL), capacity
 *                             (as n_max), scale, bias, row_min, row_max, codes_u8, packed; all jobs
 *                             share dim, bits, mode and the greedy parameters
 *   cnr_restore_rows_batch    table (written), n_rows, row_ids, n_dirty_dev, capacity, packed, scale,
 *                             bias; all jobs share dim and bits
 * Argument errors are reported for the whole call before anything is launched. */
#define CNR_MAX_BATCH 16u

typedef struct {
    float *table;
    uint64_t n_rows;
    uint32_t *bitmap;
    const void *indices;
    uint64_t n_indices;
    void *mark_scratch;
    uint32_t *row_ids;
    uint64_t capacity;
    uint64_t *n_dirty_dev;
    void *compact_scratch;
    float *scale, *bias, *row_min, *row_max;
    uint8_t *codes_u8, *packed;
} cnr_table_job;

cnr_status cnr_clear_bitmap_batch(cnr_ctx *ctx, const cnr_table_job *jobs /* host */, uint32_t n_jobs,
                                  void *stream);
cnr_status cnr_mark_touched_batch(cnr_ctx *ctx, const cnr_table_job *jobs /* host */, uint32_t n_jobs,
                                  cnr_index_type type, void *stream);
cnr_status cnr_compact_dirty_batch(cnr_ctx *ctx, const cnr_table_job *jobs /* host */, uint32_t n_jobs,
                                   void *stream);
cnr_status cnr_quantize_rows_batch(cnr_ctx *ctx, const cnr_table_job *jobs /* host */, uint32_t n_jobs,
                                   uint32_t dim, int bits, cnr_range_mode mode,
                                   const cnr_greedy_params *greedy /* host */, void *stream);
cnr_status cnr_restore_rows_batch(cnr_ctx *ctx, const cnr_table_job *jobs /* host */, uint32_t n_jobs,
                                  uint32_t dim, int bits, void *stream);

/* ---- chunked encode into host memory (Sections 4.4 and 5.2: the optimized checkpoint is built chunk
 *      by chunk, and a finished chunk is handed on while the next one is quantized) ----------------
 *
 * A writer owns two device staging sets of chunk_rows rows (row ids, scale, bias, packed codes), a
 * copy stream of default priority and the events that order it against the caller's stream.
 * cnr_host_writer_create allocates them (cnr_host_writer_device_bytes tells how much device memory),
 * cnr_host_writer_destroy waits for the copy stream and frees them; nothing is allocated in between.
 *
 * cnr_encode_to_host quantizes rows row_ids[0 .. n) of `table` (min/max, symmetric or greedy range, as
 * cnr_quantize_rows does) chunk by chunk on `stream` and copies every finished chunk, and the matching
 * slice of row_ids, into the host buffers; with `overlap` != 0 the copies run on the writer's stream
 * while the next chunk is encoded, else on `stream` itself.  It only enqueues work; the host buffers
 * are complete after cnr_host_writer_wait (which synchronizes both streams).  One call at a time per
 * writer.  With CNR_HOST_DIRECT nothing is staged: one encode kernel on `stream` stores scale, bias and
 * codes into the host buffers over the host link, and the id list is copied on the writer's stream
 * meanwhile; the host buffers must then be pinned, device-accessible memory, 16-byte aligned
 * (CNR_E_HOST_MEMORY, CNR_E_ALIGN).  Rows of up to 64 elements leave a wave as one contiguous block and
 * this way is then slightly faster than the staged one; longer rows leave in pieces that the link does
 * not merge (a fifth slower at 128 elements), and the staged way is the better one.
 *   n               host value: the number of rows (read it back from cnr_compact_dirty's count first)
 *   row_ids         device, uint32 [n], 16-byte aligned; NULL means rows 0 .. n-1 of the table (a
 *                   full checkpoint)
 *   host_row_ids    host uint32 [n] (ignored when row_ids is NULL)
 *   host_scale, host_bias   host float [n]
 *   host_packed     host uint8 [n][cnr_packed_row_bytes(dim, bits)]
 *                   Pinned host memory lets the copies overlap; pageable memory works but serializes.
 *   chunk_rows      a multiple of 16
 *
 * cnr_restore_from_host is the way back (Section 5.1: resume = baseline + incremental checkpoint;
 * Section 6.2: the checkpoint is de-quantized when it is loaded): the same staging sets take the n
 * rows of a checkpoint from host memory chunk by chunk, and every chunk is de-quantized and
 * written over `table` as cnr_restore_rows does; with `overlap` == CNR_HOST_OVERLAP the copy of one
 * chunk runs on the writer's stream while the chunk before it is restored on `stream`, with
 * CNR_HOST_SERIAL the copies run on `stream` too.  The copies start after everything enqueued on
 * `stream` before the call.  With CNR_HOST_DIRECT nothing is copied and nothing staged: one restore
 * kernel on `stream` reads ids, scale, bias and codes from the host buffers over the host link while
 * it writes the rows (each byte crosses the link once and is never written to device memory first);
 * the host buffers must then be pinned, device-accessible memory (hipHostMalloc and what wraps it),
 * 16-byte aligned, else CNR_E_HOST_MEMORY or CNR_E_ALIGN is returned and nothing is launched.
 * The call only enqueues work; the host buffers may be reused after cnr_host_writer_wait.
 *   host_row_ids    host uint32 [n]; NULL means rows 0 .. n-1 of the table (a full checkpoint)
 *   host_scale, host_bias, host_packed   as cnr_encode_to_host wrote them
 *   overlap         a cnr_host_path (CNR_E_INVALID for any other value) */
typedef struct cnr_host_writer cnr_host_writer; /* opaque */

typedef enum cnr_host_path {
    CNR_HOST_SERIAL = 0,  /* copies on the caller's stream, in order with the kernels */
    CNR_HOST_OVERLAP = 1, /* copies on the writer's stream, overlapping the kernels of the neighbouring chunk */
    CNR_HOST_DIRECT = 2   /* no copies of the data: the kernel reads or writes the pinned host buffers itself */
} cnr_host_path;

size_t cnr_host_writer_device_bytes(uint32_t dim, int bits, uint64_t chunk_rows);
cnr_status cnr_host_writer_create(cnr_ctx *ctx, uint32_t dim, int bits, uint64_t chunk_rows, cnr_host_writer **out);
cnr_status cnr_host_writer_destroy(cnr_host_writer *w);
cnr_status cnr_encode_to_host(cnr_host_writer *w, const float *table, uint64_t n_rows, const uint32_t *row_ids,
                              uint64_t n, cnr_range_mode mode, const cnr_greedy_params *greedy /* host */,
                              uint32_t *host_row_ids, float *host_scale, float *host_bias, uint8_t *host_packed,
                              int overlap, void *stream);
cnr_status cnr_restore_from_host(cnr_host_writer *w, float *table, uint64_t n_rows,
                                 const uint32_t *host_row_ids, const float *host_scale, const float *host_bias,
                                 const uint8_t *host_packed, uint64_t n, int overlap, void *stream);
cnr_status cnr_host_writer_wait(cnr_host_writer *w, void *stream);

/* ---- device-side conditions ---------------------------------------------------------------- */

/* Waits for `stream`, then reports and resets what the kernels recorded since the last poll.
 *   n_bad_indices  host uint64 [1] or NULL: look-up indices skipped by cnr_mark_touched
 *   flags          host uint32 [1] or NULL: CNR_FLAG_* bits
 * Returns CNR_OK when nothing was recorded, else CNR_E_CAPACITY, CNR_E_ROW_ID or
 * CNR_E_INDEX_RANGE (in that order of precedence). */
cnr_status cnr_poll_errors(cnr_ctx *ctx, void *stream, uint64_t *n_bad_indices, uint32_t *flags);

const char *cnr_status_str(cnr_status s);
/* hipError_t of the last failed HIP call on this context (0 if none), as an int. */
int cnr_last_hip_error(const cnr_ctx *ctx);

/* ---- checkpoint policy (Section 5.1; host only, no GPU involved) --------------------------------- */

/* sizes[0..i) = S_1..S_i, the sizes of the incremental checkpoints since the last full one as
 * fractions of a full checkpoint.  Returns 1 when a full checkpoint should be taken at interval
 * i+1, i.e. when F_c = 1 + S_1 + ... + S_i <= I_c = (i + 1) * S_i, else 0 (also for i == 0). */
int cnr_full_checkpoint_due(const double *sizes /* host */, uint32_t i);

/* The three incremental policies of Section 5.1 as a small state machine the trainer consults at
 * the end of every checkpoint interval.
 *   one-shot      every incremental checkpoint holds the rows modified since the baseline: the
 *                 tracking bitmap is never cleared; resume = baseline + latest incremental
 *   consecutive   every incremental checkpoint holds the rows modified in the last interval: the
 *                 bitmap is cleared after each checkpoint; resume = baseline + all incrementals in
 *                 order
 *   intermittent  one-shot, but a new full baseline is taken when cnr_full_checkpoint_due says so
 *                 on the history S_1..S_i of incremental sizes since the last full one (the
 *                 decision at interval i+1 uses the history only, as in the paper; the size measured
 *                 at interval i+1 is recorded afterwards when the checkpoint is incremental)
 * The struct is plain data owned by the caller (host). */
typedef enum { CNR_POLICY_ONE_SHOT = 0, CNR_POLICY_CONSECUTIVE = 1, CNR_POLICY_INTERMITTENT = 2 } cnr_policy_kind;

#define CNR_POLICY_MAX_HISTORY 256u

typedef struct {
    int kind;                               /* cnr_policy_kind */
    uint32_t n_history;                     /* i: incremental checkpoints since the last full one */
    double history[CNR_POLICY_MAX_HISTORY]; /* S_1 .. S_i */
} cnr_policy;

typedef struct {
    int take_full;    /* 1: write a full checkpoint (new baseline) now; 0: write the dirty rows */
    int clear_bitmap; /* 1: clear the tracking bitmap after this checkpoint */
} cnr_policy_decision;

cnr_status cnr_policy_init(cnr_policy *p /* host */, cnr_policy_kind kind);
/* dirty_fraction = n_dirty / n_rows as cnr_compact_dirty just measured it (the size the incremental
 * checkpoint would have, as a fraction of a full one).  When the history is full the intermittent
 * policy takes a full checkpoint. */
cnr_policy_decision cnr_policy_next(cnr_policy *p /* host */, double dirty_fraction);

/* Dynamic bit-width selection (Section 6.2.1): the narrowest code width that keeps the accuracy
 * loss under the paper's threshold for the number of times the job is expected to resume from a
 * quantized checkpoint: 2 bits for at most one resume, 3 bits for at most 3, 4 bits for at most
 * 20, 8 bits beyond that; and 8 bits from the moment the resumes seen so far exceed the
 * expectation.  Host only.  Returns 2, 3, 4 or 8 (a value cnr_quantize_rows takes as `bits`). */
int cnr_select_bits(uint32_t expected_resumes, uint32_t observed_resumes);

#ifdef __cplusplus
}
#endif
#endif /* CNR_H */
