// Choice of the greedy search parameters by profiling a sample of the checkpoint (Section 5.2,
// "Parameter selection"): quantize the sampled rows with a grid of parameter values, compute the
// mean l2 error of each, keep the value at which the improvement over plain min/max quantization
// tapers off.  Quantization and errors run in the library's kernels; what happens here on the host
// is the comparison of a dozen means.
#include "cnr_common.h"

namespace {

size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

// Layout of the caller's scratch: scale | bias | packed | err | mean, each 16-byte aligned.
struct SelectScratch {
    float *scale, *bias;
    uint8_t *packed;
    double *err, *mean;
    size_t bytes;
};

SelectScratch carve(void *base, uint64_t n, uint32_t dim, int bits) {
    SelectScratch s;
    uint8_t *p = static_cast<uint8_t *>(base);
    size_t off = 0;
    s.scale = reinterpret_cast<float *>(p + off); off += align16(n * sizeof(float));
    s.bias = reinterpret_cast<float *>(p + off); off += align16(n * sizeof(float));
    s.packed = p + off; off += align16(n * cnr_packed_row_bytes(dim, bits));
    s.err = reinterpret_cast<double *>(p + off); off += align16(n * sizeof(double));
    s.mean = reinterpret_cast<double *>(p + off); off += 16;
    s.bytes = off;
    return s;
}

// Index of the smallest grid value whose improvement 1 - E / E_naive is within `taper` (relative) of
// the best improvement on the grid; the first one when nothing improves on min/max.
uint32_t taper_choice(const double *errors, uint32_t n, double naive, double taper) {
    double best = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
        const double gain = naive > 0.0 ? 1.0 - errors[i] / naive : 0.0;
        if (i == 0 || gain > best) best = gain;
    }
    if (!(best > 0.0)) return 0;
    for (uint32_t i = 0; i < n; ++i) {
        const double gain = naive > 0.0 ? 1.0 - errors[i] / naive : 0.0;
        if (gain >= (1.0 - taper) * best) return i;
    }
    return n - 1;
}

}  // namespace

extern "C" {

size_t cnr_select_scratch_bytes(uint64_t n_sample, uint32_t dim, int bits) {
    if (cnr_packed_row_bytes(dim, bits) == 0) return 0;
    return carve(nullptr, n_sample, dim, bits).bytes;
}

cnr_status cnr_select_greedy_params(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                                    const uint32_t *sample_ids, uint64_t n_sample, int bits,
                                    const uint32_t *bins_grid, uint32_t n_bins, const float *ratio_grid,
                                    uint32_t n_ratios, double taper, void *scratch, cnr_greedy_params *chosen,
                                    double *report, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (!chosen || !bins_grid || !ratio_grid || n_bins == 0 || n_ratios == 0 || n_sample == 0 || !scratch ||
        !(taper >= 0.0 && taper < 1.0))
        return CNR_E_INVALID;
    if (n_bins > CNR_SELECT_MAX_GRID || n_ratios > CNR_SELECT_MAX_GRID) return CNR_E_INVALID;
    if ((uintptr_t)scratch % 16) return CNR_E_ALIGN;
    const SelectScratch s = carve(scratch, n_sample, dim, bits);
    hipStream_t hs = as_stream(stream);

    // mean l2 error of the sample under one quantizer, read back through pinned memory
    auto mean_error = [&](cnr_range_mode mode, const cnr_greedy_params *gp, double *out) -> cnr_status {
        cnr_status r = cnr_quantize_rows(ctx, table, n_rows, dim, sample_ids, nullptr, n_sample, bits, mode, gp, s.scale,
                                         s.bias, nullptr, nullptr, nullptr, s.packed, stream);
        if (r != CNR_OK) return r;
        r = cnr_quant_error(ctx, table, n_rows, dim, sample_ids, nullptr, n_sample, bits, s.packed, s.scale, s.bias,
                            s.err, s.mean, stream);
        if (r != CNR_OK) return r;
        hipError_t e = hipMemcpyAsync(ctx->host_scalar, s.mean, sizeof(double), hipMemcpyDeviceToHost, hs);
        if (e == hipSuccess) e = hipStreamSynchronize(hs);
        if (e != hipSuccess) return cnr_hip_status(ctx, e);
        *out = *ctx->host_scalar;
        return CNR_OK;
    };

    double naive = 0.0;
    if ((st = mean_error(CNR_RANGE_MINMAX, nullptr, &naive)) != CNR_OK) return st;
    if (report) report[0] = naive;
    double errors[CNR_SELECT_MAX_GRID];
    for (uint32_t i = 0; i < n_bins; ++i) {  // num_bins first, at ratio 1
        const cnr_greedy_params gp = {bins_grid[i], 1.0f};
        if ((st = mean_error(CNR_RANGE_GREEDY, &gp, &errors[i])) != CNR_OK) return st;
        if (report) report[1 + i] = errors[i];
    }
    chosen->num_bins = bins_grid[taper_choice(errors, n_bins, naive, taper)];
    for (uint32_t i = 0; i < n_ratios; ++i) {  // then the ratio, at that num_bins
        const cnr_greedy_params gp = {chosen->num_bins, ratio_grid[i]};
        if ((st = mean_error(CNR_RANGE_GREEDY, &gp, &errors[i])) != CNR_OK) return st;
        if (report) report[1 + n_bins + i] = errors[i];
    }
    chosen->ratio = ratio_grid[taper_choice(errors, n_ratios, naive, taper)];
    return CNR_OK;
}

}  // extern "C"
