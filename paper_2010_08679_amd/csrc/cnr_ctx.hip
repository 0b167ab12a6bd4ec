// Context, size helpers, bitmap clear, error polling and the host-side checkpoint policy.
#include <math.h>
#include <new>

#include "cnr_common.h"

cnr_status cnr_hip_status(cnr_ctx *ctx, hipError_t e) {
    if (e == hipSuccess) return CNR_OK;
    if (ctx) ctx->last_hip_error = (int)e;
    return CNR_E_HIP;
}

cnr_status cnr_enter(cnr_ctx *ctx) {
    if (!ctx) return CNR_E_INVALID;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return cnr_hip_status(ctx, e);
    if (cur != ctx->device) return cnr_hip_status(ctx, hipSetDevice(ctx->device));
    return CNR_OK;
}

__global__ void __launch_bounds__(kBlock) fill_u32_kernel(uint32_t *p, uint64_t n, uint32_t v) {
    uint64_t i = (uint64_t)wg_x() * kBlock + tid_x();
    const uint64_t stride = (uint64_t)grid_x() * kBlock;
    for (; i < n; i += stride) p[i] = v;
}

extern "C" {

cnr_status cnr_create(cnr_ctx **out, int device) {
    if (!out) return CNR_E_INVALID;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return CNR_E_HIP;
    cnr_ctx *ctx = new (std::nothrow) cnr_ctx();
    if (!ctx) return CNR_E_INVALID;
    ctx->device = device;
    ctx->last_hip_error = 0;
    ctx->dev_err = nullptr;
    ctx->host_err = nullptr;
    ctx->host_scalar = nullptr;
    ctx->static_scratch = nullptr;
    hipError_t e = hipSetDevice(device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess) {
        ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        e = hipMalloc((void **)&ctx->dev_err, sizeof(cnr_dev_errors));
    }
    if (e == hipSuccess) {
        e = hipHostMalloc((void **)&ctx->host_err, sizeof(cnr_dev_errors) + sizeof(double), hipHostMallocDefault);
        if (e == hipSuccess) ctx->host_scalar = reinterpret_cast<double *>(ctx->host_err + 1);
    }
    if (e == hipSuccess) e = hipMemset(ctx->dev_err, 0, sizeof(cnr_dev_errors));
    if (e == hipSuccess && cnr_bind_static_scratch(ctx) != CNR_OK) e = (hipError_t)ctx->last_hip_error;
    if (e != hipSuccess) {
        if (ctx->dev_err) (void)hipFree(ctx->dev_err);
        if (ctx->host_err) (void)hipHostFree(ctx->host_err);
        delete ctx;
        return CNR_E_HIP;
    }
    *out = ctx;
    return CNR_OK;
}

cnr_status cnr_destroy(cnr_ctx *ctx) {
    if (!ctx) return CNR_E_INVALID;
    cnr_status st = cnr_enter(ctx);
    hipError_t e1 = hipFree(ctx->dev_err);
    hipError_t e2 = hipHostFree(ctx->host_err);
    delete ctx;
    if (st != CNR_OK) return st;
    return (e1 == hipSuccess && e2 == hipSuccess) ? CNR_OK : CNR_E_HIP;
}

size_t cnr_bitmap_words(uint64_t n_rows) { return (size_t)((n_rows + 31u) / 32u); }

size_t cnr_packed_row_bytes(uint32_t dim, int bits) {
    if (!cnr_valid_bits(bits)) return 0;
    uint64_t total = (uint64_t)dim * (uint64_t)bits;
    return (total % 8u) ? 0 : (size_t)(total / 8u);
}

size_t cnr_scratch_bytes(uint64_t n_rows) {
    uint64_t blocks = (n_rows + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    if (blocks < 1) blocks = 1;
    return (size_t)(blocks * sizeof(uint32_t) + 8u);
}

uint32_t cnr_greedy_iterations(uint32_t num_bins, float ratio) {
    if (num_bins < 2) return 0;
    double want = ceil((double)ratio * (double)num_bins - 1e-4);
    if (!(want > 0.0)) return 0;
    double cap = (double)(num_bins - 1);
    return (uint32_t)(want < cap ? want : cap);
}

cnr_status cnr_poll_errors(cnr_ctx *ctx, void *stream, uint64_t *n_bad_indices, uint32_t *flags) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    hipStream_t s = as_stream(stream);
    hipError_t e = hipMemcpyAsync(ctx->host_err, ctx->dev_err, sizeof(cnr_dev_errors),
                                  hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return cnr_hip_status(ctx, e);
    const cnr_dev_errors got = *ctx->host_err;
    if (got.n_bad_indices || got.flags) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(kBlock), 0, s, (uint32_t *)ctx->dev_err,
                           (uint64_t)(sizeof(cnr_dev_errors) / sizeof(uint32_t)), 0u);
        st = cnr_launch_status(ctx);
        if (st != CNR_OK) return st;
    }
    if (n_bad_indices) *n_bad_indices = got.n_bad_indices;
    if (flags) *flags = got.flags;
    if (got.flags & CNR_FLAG_CAPACITY) return CNR_E_CAPACITY;
    if (got.flags & CNR_FLAG_ROW_ID) return CNR_E_ROW_ID;
    if (got.n_bad_indices) return CNR_E_INDEX_RANGE;
    return CNR_OK;
}

const char *cnr_status_str(cnr_status s) {
    switch (s) {
        case CNR_OK: return "ok";
        case CNR_E_INVALID: return "invalid argument";
        case CNR_E_BITS: return "bit-width must be 2, 3, 4 or 8";
        case CNR_E_DIM: return "unsupported row dimension for this bit-width";
        case CNR_E_ALIGN: return "misaligned base pointer";
        case CNR_E_CAPACITY: return "more dirty rows than the row-id buffer holds";
        case CNR_E_INDEX_RANGE: return "look-up indices outside the table were skipped";
        case CNR_E_ROW_ID: return "row id outside the table was skipped";
        case CNR_E_HIP: return "HIP runtime error";
        case CNR_E_TOO_LARGE: return "size beyond the fixed maximum of a call that allocates nothing";
        case CNR_E_HOST_MEMORY: return "host buffer is not pinned, device-accessible memory";
    }
    return "unknown status";
}

int cnr_last_hip_error(const cnr_ctx *ctx) { return ctx ? ctx->last_hip_error : 0; }

int cnr_full_checkpoint_due(const double *sizes, uint32_t i) {
    if (!sizes || i == 0) return 0;
    double future_if_full = 1.0;
    for (uint32_t t = 0; t < i; ++t) future_if_full += sizes[t];
    const double future_if_incremental = (double)(i + 1) * sizes[i - 1];
    return future_if_full <= future_if_incremental ? 1 : 0;
}

cnr_status cnr_policy_init(cnr_policy *p, cnr_policy_kind kind) {
    if (!p || (kind != CNR_POLICY_ONE_SHOT && kind != CNR_POLICY_CONSECUTIVE && kind != CNR_POLICY_INTERMITTENT))
        return CNR_E_INVALID;
    p->kind = (int)kind;
    p->n_history = 0;
    for (uint32_t t = 0; t < CNR_POLICY_MAX_HISTORY; ++t) p->history[t] = 0.0;
    return CNR_OK;
}

cnr_policy_decision cnr_policy_next(cnr_policy *p, double dirty_fraction) {
    cnr_policy_decision d = {0, 0};
    if (!p) return d;
    switch (p->kind) {
        case CNR_POLICY_CONSECUTIVE:
            d.clear_bitmap = 1;
            return d;
        case CNR_POLICY_INTERMITTENT:
            if (p->n_history >= CNR_POLICY_MAX_HISTORY || cnr_full_checkpoint_due(p->history, p->n_history)) {
                d.take_full = 1;
                d.clear_bitmap = 1;
                p->n_history = 0;
            } else {
                p->history[p->n_history++] = dirty_fraction;
            }
            return d;
        default:  // one-shot: the bitmap keeps accumulating since the baseline
            return d;
    }
}

int cnr_select_bits(uint32_t expected_resumes, uint32_t observed_resumes) {
    if (observed_resumes > expected_resumes) return 8;
    if (expected_resumes <= 1) return 2;
    if (expected_resumes <= 3) return 3;
    if (expected_resumes <= 20) return 4;
    return 8;
}

}  // extern "C"
