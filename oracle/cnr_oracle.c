/*
 * cnr_oracle.c -- plain CPU reference for the Check-N-Run checkpoint-encoder hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * GPU library has to compute.  It shares no code, header, table or helper with the GPU path
 * and must never be called from it.  Only the test-suite, the smoke check and the CPU-baseline
 * leg of the benchmark load it.
 *
 * What each function follows (Check-N-Run, arXiv 2010.08679):
 *   mark / clear      Section 5.1.1 "Efficient Tracking": one bit per local embedding vector,
 *                     set when the vector is looked up in the forward pass.
 *   compact           Section 5.1 "One-Shot Incremental Checkpoint": the incremental view holds
 *                     exactly the vectors whose bit is set.
 *   quantize (naive)  Section 5.2, Approach 1: scale = (x_max - x_min) / (2^N - 1),
 *                     zero_point = x_min, x_q = round((x - zero_point) / scale), with x_min and
 *                     x_max the smallest and largest element of the vector (asymmetric), or
 *                     +-max|x| (symmetric).
 *   quantize (greedy) Section 5.2, Approach 3: step_size = (X_max - X_min) / num_bins; every
 *                     iteration evaluates F_Q(x, x_min + step, x_max) and
 *                     F_Q(x, x_min, x_max - step), keeps the bound whose quantization has the
 *                     lower l2 error, and the final range is the one of the iteration with the
 *                     lowest error; `ratio` bounds the fraction of the range walked.
 *   de-quantize       Section 5.2, Approach 1: x = scale * x_q + zero_point.
 *   l2 error          Section 5.2: ||X - Q||_2 per vector, mean over the m vectors.
 *
 * Arithmetic: the table is fp32 and the stored parameters are fp32, and the integer code is a
 * decision taken on floating-point values, so every step that leads to a code is done in fp32
 * with each operation rounded once (round-to-nearest-even, no fused multiply-add: build with
 * -ffp-contract=off and without -ffast-math).  Error sums that only rank candidate ranges, and
 * the reported l2 metric, are accumulated in fp64.
 *
 * Readings taken where the text is silent (each is also listed in the design notes):
 *   - "round" is round-half-to-even.
 *   - A constant vector (x_max == x_min) gets scale 0 and all codes 0; it de-quantizes to x_min.
 *   - -0.0 is canonicalised to +0.0 in the row minimum / maximum.
 *   - The greedy loop runs n_iter = min(ceil(ratio * num_bins - 1e-4), num_bins - 1) iterations:
 *     it stops once the removed part reaches ratio * range, and never collapses the range to
 *     zero width.  The un-shrunk range is candidate number zero.  The lower bound moves only on
 *     a strictly smaller error; the best range is replaced only on a strictly smaller error.
 *     Bounds are updated cumulatively in fp32.
 *   - Packed layout: per row a little-endian bit stream, element j in stream bits
 *     [j*b, (j+1)*b), least significant code bit first; rows back to back, no padding.
 *   - Bitmap: row i is bit (i & 31) of 32-bit word (i >> 5).  Indices outside [0, n_rows) are
 *     skipped and counted.
 *
 * Every function is pinned by tests that do not go through this file's formulas: set/np.unique
 * brute force (mark, compact), numpy min/max (range), nearest-grid-point brute force and the
 * scale/2 error bound (codes), hand-written byte patterns (pack), exact rational brute force
 * over the shrink lattice (greedy).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CNRO_RANGE_MINMAX = 0, CNRO_RANGE_GREEDY = 1, CNRO_RANGE_SYMMETRIC = 2 };

/* ------------------------------------------------------------------ tracking bit-vector */

uint64_t cnro_bitmap_words(uint64_t n_rows) { return (n_rows + 31u) / 32u; }

void cnro_clear(uint32_t *bitmap, uint64_t n_rows) {
    memset(bitmap, 0, cnro_bitmap_words(n_rows) * sizeof(uint32_t));
}

/* Sets the bit of every looked-up row.  Returns how many indices fell outside [0, n_rows). */
uint64_t cnro_mark_touched(uint32_t *bitmap, uint64_t n_rows, const void *indices,
                           uint64_t n_indices, int index_is_i64) {
    uint64_t skipped = 0;
    for (uint64_t t = 0; t < n_indices; ++t) {
        int64_t i = index_is_i64 ? ((const int64_t *)indices)[t]
                                 : (int64_t)((const int32_t *)indices)[t];
        if (i < 0 || (uint64_t)i >= n_rows) {
            ++skipped;
            continue;
        }
        bitmap[i >> 5] |= (uint32_t)1 << (i & 31);
    }
    return skipped;
}

/* Ascending list of rows whose bit is set.  Writes at most `capacity` ids, returns the full
 * count. */
uint64_t cnro_compact_dirty(const uint32_t *bitmap, uint64_t n_rows, uint32_t *row_ids,
                            uint64_t capacity) {
    uint64_t n = 0;
    for (uint64_t r = 0; r < n_rows; ++r) {
        if ((bitmap[r >> 5] >> (r & 31)) & 1u) {
            if (n < capacity) row_ids[n] = (uint32_t)r;
            ++n;
        }
    }
    return n;
}

/* ------------------------------------------------------------------ uniform quantization */

static int valid_bits(int bits) { return bits == 2 || bits == 3 || bits == 4 || bits == 8; }

/* scale of F_Q(., lo, hi) at N bits */
static float fq_scale(float lo, float hi, int bits) {
    float range = hi - lo;
    return range / (float)((1 << bits) - 1);
}

/* code of one element under F_Q(., lo, hi) */
static int fq_code(float x, float lo, float hi, float scale, int qmax) {
    if (scale == 0.0f) return 0;
    float c = x;
    if (c < lo) c = lo;
    if (c > hi) c = hi;
    float t = (c - lo) / scale;
    int q = (int)nearbyintf(t);
    if (q < 0) q = 0;
    if (q > qmax) q = qmax;
    return q;
}

/* x = scale * x_q + zero_point: one multiplication, then one addition */
static float fq_value(int q, float scale, float bias) {
    float p = scale * (float)q;
    return p + bias;
}

/* squared l2 error of quantizing one vector with F_Q(., lo, hi) */
static double fq_sq_error(const float *x, uint32_t dim, float lo, float hi, int bits) {
    const int qmax = (1 << bits) - 1;
    const float scale = fq_scale(lo, hi, bits);
    double acc = 0.0;
    for (uint32_t j = 0; j < dim; ++j) {
        int q = fq_code(x[j], lo, hi, scale, qmax);
        float d = x[j] - fq_value(q, scale, lo);
        acc += (double)d * (double)d;
    }
    return acc;
}

static uint32_t greedy_iterations(uint32_t num_bins, float ratio) {
    if (num_bins < 2) return 0;
    double want = ceil((double)ratio * (double)num_bins - 1e-4);
    if (want < 0.0) want = 0.0;
    double cap = (double)(num_bins - 1);
    return (uint32_t)(want < cap ? want : cap);
}

/* Adaptive range: greedy shrink of [X_min, X_max], one step_size at a time. */
static void greedy_range(const float *x, uint32_t dim, float X_min, float X_max, int bits,
                         uint32_t num_bins, float ratio, float *lo_out, float *hi_out) {
    float best_lo = X_min, best_hi = X_max;
    float range = X_max - X_min;
    uint32_t n_iter = greedy_iterations(num_bins, ratio);
    if (range == 0.0f || n_iter == 0) {
        *lo_out = best_lo;
        *hi_out = best_hi;
        return;
    }
    float step_size = range / (float)num_bins;
    float x_min = X_min, x_max = X_max;
    double best_err = fq_sq_error(x, dim, x_min, x_max, bits);
    for (uint32_t it = 0; it < n_iter; ++it) {
        float cand_min = x_min + step_size;
        float cand_max = x_max - step_size;
        double err_min = fq_sq_error(x, dim, cand_min, x_max, bits);
        double err_max = fq_sq_error(x, dim, x_min, cand_max, bits);
        double err;
        if (err_min < err_max) {
            x_min = cand_min;
            err = err_min;
        } else {
            x_max = cand_max;
            err = err_max;
        }
        if (err < best_err) {
            best_err = err;
            best_lo = x_min;
            best_hi = x_max;
        }
    }
    *lo_out = best_lo;
    *hi_out = best_hi;
}

typedef struct {
    const float *table;
    uint32_t dim;
    const uint32_t *row_ids;
    uint64_t k_begin, k_end;
    int bits, mode;
    uint32_t num_bins;
    float ratio;
    float *scale, *bias, *row_min, *row_max;
    uint8_t *codes;
} quant_job;

static void quantize_range_of_rows(const quant_job *job) {
    const uint32_t dim = job->dim;
    const int qmax = (1 << job->bits) - 1;
    for (uint64_t k = job->k_begin; k < job->k_end; ++k) {
        uint64_t r = job->row_ids ? (uint64_t)job->row_ids[k] : k;
        const float *x = job->table + r * (uint64_t)dim;
        float X_min = x[0], X_max = x[0];
        for (uint32_t j = 1; j < dim; ++j) {
            if (x[j] < X_min) X_min = x[j];
            if (x[j] > X_max) X_max = x[j];
        }
        X_min = X_min + 0.0f; /* -0.0 -> +0.0 */
        X_max = X_max + 0.0f;
        if (job->row_min) job->row_min[k] = X_min;
        if (job->row_max) job->row_max[k] = X_max;

        float lo = X_min, hi = X_max;
        if (job->mode == CNRO_RANGE_GREEDY) {
            greedy_range(x, dim, X_min, X_max, job->bits, job->num_bins, job->ratio, &lo, &hi);
        } else if (job->mode == CNRO_RANGE_SYMMETRIC) {
            float a = fabsf(X_min) > fabsf(X_max) ? fabsf(X_min) : fabsf(X_max);
            lo = -a + 0.0f;
            hi = a;
        }
        float scale = fq_scale(lo, hi, job->bits);
        if (job->scale) job->scale[k] = scale;
        if (job->bias) job->bias[k] = lo;
        if (job->codes) {
            uint8_t *c = job->codes + k * (uint64_t)dim;
            for (uint32_t j = 0; j < dim; ++j) c[j] = (uint8_t)fq_code(x[j], lo, hi, scale, qmax);
        }
    }
}

static void *quantize_thread(void *arg) {
    quantize_range_of_rows((const quant_job *)arg);
    return NULL;
}

/* Runs fn over [0, n) split into n_threads contiguous pieces. */
static void split_rows(uint64_t n, int n_threads, void *(*fn)(void *), void *jobs, size_t job_size,
                       void (*set_range)(void *, uint64_t, uint64_t)) {
    if (n_threads < 1) n_threads = 1;
    if ((uint64_t)n_threads > n) n_threads = n ? (int)n : 1;
    pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)n_threads);
    uint64_t per = (n + (uint64_t)n_threads - 1) / (uint64_t)n_threads;
    for (int t = 0; t < n_threads; ++t) {
        uint64_t b = per * (uint64_t)t, e = b + per;
        if (b > n) b = n;
        if (e > n) e = n;
        set_range((char *)jobs + job_size * (size_t)t, b, e);
    }
    if (n_threads == 1) {
        fn(jobs);
    } else {
        for (int t = 0; t < n_threads; ++t)
            pthread_create(&tid[t], NULL, fn, (char *)jobs + job_size * (size_t)t);
        for (int t = 0; t < n_threads; ++t) pthread_join(tid[t], NULL);
    }
    free(tid);
}

static void quant_set_range(void *job, uint64_t b, uint64_t e) {
    ((quant_job *)job)->k_begin = b;
    ((quant_job *)job)->k_end = e;
}

/*
 * Gathers rows row_ids[0..n) (rows 0..n-1 when row_ids is NULL) of a row-major fp32 table and
 * quantizes each to `bits` bits.  Any output pointer may be NULL.  codes is [n][dim], one code
 * per byte.  Returns 0, or -1 on an unsupported bit-width / mode / empty dim.
 */
int cnro_quantize_rows(const float *table, uint32_t dim, const uint32_t *row_ids, uint64_t n,
                       int bits, int mode, uint32_t num_bins, float ratio, float *scale,
                       float *bias, float *row_min, float *row_max, uint8_t *codes,
                       int n_threads) {
    if (!valid_bits(bits) || dim == 0) return -1;
    if (mode != CNRO_RANGE_MINMAX && mode != CNRO_RANGE_GREEDY && mode != CNRO_RANGE_SYMMETRIC)
        return -1;
    if (n == 0) return 0;
    if (n_threads < 1) n_threads = 1;
    quant_job *jobs = (quant_job *)malloc(sizeof(quant_job) * (size_t)n_threads);
    for (int t = 0; t < n_threads; ++t) {
        quant_job j = {table, dim, row_ids, 0, 0, bits, mode, num_bins, ratio,
                       scale, bias, row_min, row_max, codes};
        jobs[t] = j;
    }
    split_rows(n, n_threads, quantize_thread, jobs, sizeof(quant_job), quant_set_range);
    free(jobs);
    return 0;
}

/* Number of greedy iterations the parameters ask for (exposed so tests can pin the reading). */
uint32_t cnro_greedy_iterations(uint32_t num_bins, float ratio) {
    return greedy_iterations(num_bins, ratio);
}

/* Squared l2 error of F_Q(x, lo, hi) on one vector (exposed for the greedy pins). */
double cnro_fq_sq_error(const float *x, uint32_t dim, float lo, float hi, int bits) {
    return fq_sq_error(x, dim, lo, hi, bits);
}

/* ------------------------------------------------------------------ dense bit packing */

uint64_t cnro_packed_row_bytes(uint32_t dim, int bits) {
    return ((uint64_t)dim * (uint64_t)bits) / 8u;
}

int cnro_pack(const uint8_t *codes, uint64_t n, uint32_t dim, int bits, uint8_t *packed) {
    if (!valid_bits(bits) || ((uint64_t)dim * (uint64_t)bits) % 8u) return -1;
    const uint64_t row_bytes = cnro_packed_row_bytes(dim, bits);
    memset(packed, 0, n * row_bytes);
    for (uint64_t k = 0; k < n; ++k) {
        uint8_t *out = packed + k * row_bytes;
        for (uint32_t j = 0; j < dim; ++j) {
            unsigned code = codes[k * (uint64_t)dim + j];
            for (int t = 0; t < bits; ++t) {
                uint64_t pos = (uint64_t)j * (uint64_t)bits + (uint64_t)t;
                if ((code >> t) & 1u) out[pos >> 3] |= (uint8_t)(1u << (pos & 7u));
            }
        }
    }
    return 0;
}

int cnro_unpack(const uint8_t *packed, uint64_t n, uint32_t dim, int bits, uint8_t *codes) {
    if (!valid_bits(bits) || ((uint64_t)dim * (uint64_t)bits) % 8u) return -1;
    const uint64_t row_bytes = cnro_packed_row_bytes(dim, bits);
    for (uint64_t k = 0; k < n; ++k) {
        const uint8_t *in = packed + k * row_bytes;
        for (uint32_t j = 0; j < dim; ++j) {
            unsigned code = 0;
            for (int t = 0; t < bits; ++t) {
                uint64_t pos = (uint64_t)j * (uint64_t)bits + (uint64_t)t;
                code |= (unsigned)((in[pos >> 3] >> (pos & 7u)) & 1u) << t;
            }
            codes[k * (uint64_t)dim + j] = (uint8_t)code;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ de-quantize / restore */

/* out[k][j] = scale[k] * codes[k][j] + bias[k] */
void cnro_dequantize(const uint8_t *codes, const float *scale, const float *bias, uint64_t n,
                     uint32_t dim, float *out) {
    for (uint64_t k = 0; k < n; ++k)
        for (uint32_t j = 0; j < dim; ++j)
            out[k * (uint64_t)dim + j] = fq_value(codes[k * (uint64_t)dim + j], scale[k], bias[k]);
}

typedef struct {
    float *table;
    uint32_t dim;
    const uint32_t *row_ids;
    uint64_t k_begin, k_end;
    int bits;
    const uint8_t *packed;
    const float *scale, *bias;
} restore_job;

static void *restore_thread(void *arg) {
    const restore_job *job = (const restore_job *)arg;
    const uint64_t row_bytes = cnro_packed_row_bytes(job->dim, job->bits);
    for (uint64_t k = job->k_begin; k < job->k_end; ++k) {
        const uint8_t *in = job->packed + k * row_bytes;
        uint64_t r = job->row_ids ? (uint64_t)job->row_ids[k] : k;
        float *dst = job->table + r * (uint64_t)job->dim;
        for (uint32_t j = 0; j < job->dim; ++j) {
            unsigned code = 0;
            for (int t = 0; t < job->bits; ++t) {
                uint64_t pos = (uint64_t)j * (uint64_t)job->bits + (uint64_t)t;
                code |= (unsigned)((in[pos >> 3] >> (pos & 7u)) & 1u) << t;
            }
            dst[j] = fq_value((int)code, job->scale[k], job->bias[k]);
        }
    }
    return NULL;
}

static void restore_set_range(void *job, uint64_t b, uint64_t e) {
    ((restore_job *)job)->k_begin = b;
    ((restore_job *)job)->k_end = e;
}

/* Overwrites rows row_ids[0..n) of `table` with the de-quantized checkpoint rows; every other
 * row is left as it is.  row_ids must not repeat (threads would race otherwise). */
int cnro_restore_rows(float *table, uint64_t n_rows, uint32_t dim, const uint32_t *row_ids,
                      uint64_t n, int bits, const uint8_t *packed, const float *scale,
                      const float *bias, int n_threads) {
    if (!valid_bits(bits) || ((uint64_t)dim * (uint64_t)bits) % 8u) return -1;
    if (row_ids)
        for (uint64_t k = 0; k < n; ++k)
            if ((uint64_t)row_ids[k] >= n_rows) return -2;
    if (n == 0) return 0;
    if (n_threads < 1) n_threads = 1;
    restore_job *jobs = (restore_job *)malloc(sizeof(restore_job) * (size_t)n_threads);
    for (int t = 0; t < n_threads; ++t) {
        restore_job j = {table, dim, row_ids, 0, 0, bits, packed, scale, bias};
        jobs[t] = j;
    }
    split_rows(n, n_threads, restore_thread, jobs, sizeof(restore_job), restore_set_range);
    free(jobs);
    return 0;
}

/* ------------------------------------------------------------------ error metric */

/* err[k] = || a[k] - b[k] ||_2 in fp64; returns the mean over the n vectors (0 when n == 0). */
double cnro_row_l2(const float *a, const float *b, uint64_t n, uint32_t dim, double *err) {
    double total = 0.0;
    for (uint64_t k = 0; k < n; ++k) {
        double acc = 0.0;
        for (uint32_t j = 0; j < dim; ++j) {
            double d = (double)a[k * (uint64_t)dim + j] - (double)b[k * (uint64_t)dim + j];
            acc += d * d;
        }
        double e = sqrt(acc);
        if (err) err[k] = e;
        total += e;
    }
    return n ? total / (double)n : 0.0;
}

/* ------------------------------------------------------------------ checkpoint policy */

/*
 * Intermittent incremental policy (Section 5.1): S[0..i) holds S_1..S_i, the sizes of the
 * incremental checkpoints taken since the last full one, as fractions of the full checkpoint
 * (S_0 = 1).  A full checkpoint is taken at interval i+1 iff
 *     F_c = 1 + S_1 + ... + S_i  <=  I_c = (i + 1) * S_i.
 * Returns 1 for "take a full checkpoint", 0 for "take another incremental one".  With no
 * history (i == 0) there is nothing to compare and the answer is 0.
 */
int cnro_full_checkpoint_due(const double *S, uint32_t i) {
    if (i == 0) return 0;
    double F_c = 1.0;
    for (uint32_t t = 0; t < i; ++t) F_c += S[t];
    double I_c = (double)(i + 1) * S[i - 1];
    return F_c <= I_c ? 1 : 0;
}
