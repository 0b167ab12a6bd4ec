// Gather + per-row uniform quantization F_Q + dense packing (Section 5.2, Approaches 1 and 3).
//
// Arithmetic contract (what makes the output comparable bit for bit with a plain CPU statement of
// the formulas): fp32 throughout, one rounding per operation (the build disables contraction into
// fused multiply-adds), correctly rounded division, round-half-even, fp32 denormals kept.  Error
// sums that only rank candidate ranges are accumulated in fp64.
#include "cnr_common.h"

namespace {

enum { kModeMinMax = CNR_RANGE_MINMAX, kModeGreedy = CNR_RANGE_GREEDY, kModeSymmetric = CNR_RANGE_SYMMETRIC };

// Code of one element as a float in [0, qmax] (F_Q of Section 5.2: clip, subtract the zero point,
// divide by the scale, round).
__device__ __forceinline__ float fq_code_f(float x, float lo, float hi, float scale, float qmaxf) {
    const float c = fminf(fmaxf(x, lo), hi);
    const float t = (c - lo) / scale;
    float q = fminf(fmaxf(rintf(t), 0.0f), qmaxf);
    return scale == 0.0f ? 0.0f : q;
}

// x = scale * x_q + zero_point, product and sum rounded separately.
__device__ __forceinline__ float fq_value(float qf, float scale, float bias) {
    const float p = scale * qf;
    return p + bias;
}

__device__ __forceinline__ double fq_sq_err(float x, float lo, float hi, float scale, float qmaxf) {
    const float d = x - fq_value(fq_code_f(x, lo, hi, scale, qmaxf), scale, lo);
    return (double)d * (double)d;
}

// 4x4 transpose inside each quad of lanes: on return r[i] of quad lane j holds what r[j] of quad
// lane i held.
__device__ __forceinline__ void quad_transpose(uint32_t (&r)[4], int j) {
#pragma unroll
    for (int n = 0; n < 4; n += 2) {
        const uint32_t send = (j & 1) ? r[n] : r[n + 1];
        const uint32_t recv = (uint32_t)dpp_i<0xB1>((int)send);
        if (j & 1) r[n] = recv; else r[n + 1] = recv;
    }
#pragma unroll
    for (int n = 0; n < 2; ++n) {
        const uint32_t send = (j & 2) ? r[n] : r[n + 2];
        const uint32_t recv = (uint32_t)dpp_i<0x4E>((int)send);
        if (j & 2) r[n] = recv; else r[n + 2] = recv;
    }
}

// ---------------------------------------------------------------------------------------------
// Fast path, dim = 64 * M.
//
// Sixteen lanes share a row: lane l of the group holds, for every 64-element chunk c of the row,
// the four consecutive elements 64c + 4l .. 64c + 4l + 3, so one 16-byte load per lane reads 256
// contiguous bytes per group, and all reductions over a row stay inside one 16-lane DPP row.  Each
// group works on four consecutive dirty rows at once (so a wave has sixteen rows = 4 KB * M in
// flight before it reduces anything), which is also what lets the packed codes leave through full
// words: after quantizing, a 4x4 transpose inside each quad of lanes hands lane j the codes of
// sixteen consecutive elements of row j.
// ---------------------------------------------------------------------------------------------
template <int M, int BITS, bool GREEDY>
__global__ void __launch_bounds__(kBlock)
quantize_rows16_kernel(const float *__restrict__ table, uint64_t n_rows,
                       const uint32_t *__restrict__ row_ids, const uint64_t *__restrict__ n_dev,
                       uint64_t n_max, int mode, uint32_t n_iter, float num_bins_f,
                       float *__restrict__ scale_out, float *__restrict__ bias_out,
                       float *__restrict__ min_out, float *__restrict__ max_out,
                       uint8_t *__restrict__ codes_out, uint8_t *__restrict__ packed_out,
                       cnr_dev_errors *err) {
    constexpr int DIM = 64 * M;
    constexpr int QMAX = (1 << BITS) - 1;
    constexpr float QMAXF = (float)QMAX;
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;  // packed bytes per row

    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane >> 4;  // group of 16 lanes
    const int l = lane & 15;  // lane in group
    const int q = l >> 2;     // quad in group
    const int j = l & 3;      // lane in quad
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    const uint64_t wave_id = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;

    for (uint64_t batch = wave_id; batch * 16u < n; batch += n_waves) {
        const uint64_t k0 = batch * 16u + 4u * (uint64_t)g;  // this group's rows: k0 .. k0+3

        // ---- gather
        unsigned skip = 0;  // bit u: row k0+u is past the end or has an id outside the table
        uint64_t src[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint64_t k = k0 + u;
            if (k >= n) { skip |= 1u << u; k = n - 1; }
            uint64_t r = row_ids ? (uint64_t)row_ids[k] : k;
            if (r >= n_rows) {
                if (!(skip & (1u << u)) && l == 0) raise_flag(err, CNR_FLAG_ROW_ID);
                skip |= 1u << u;
                r = 0;
            }
            src[u] = r * (uint64_t)DIM + 4u * (uint64_t)l;
        }
        float4 x[4][M];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < M; ++c)
                x[u][c] = *reinterpret_cast<const float4 *>(table + src[u] + 64 * c);

        // ---- row minimum / maximum
        float X_min[4], X_max[4], lo[4], hi[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float mn = x[u][0].x, mx = x[u][0].x;
#pragma unroll
            for (int c = 0; c < M; ++c) {
                mn = fminf(fminf(mn, x[u][c].x), fminf(x[u][c].y, fminf(x[u][c].z, x[u][c].w)));
                mx = fmaxf(fmaxf(mx, x[u][c].x), fmaxf(x[u][c].y, fmaxf(x[u][c].z, x[u][c].w)));
            }
            X_min[u] = row16_min(mn) + 0.0f;  // -0.0 -> +0.0
            X_max[u] = row16_max(mx) + 0.0f;
            lo[u] = X_min[u];
            hi[u] = X_max[u];
            if (mode == kModeSymmetric) {
                const float a = fmaxf(fabsf(X_min[u]), fabsf(X_max[u]));
                lo[u] = -a + 0.0f;
                hi[u] = a;
            }
        }

        // ---- greedy range search (Approach 3): shrink from whichever side hurts less, remember
        // the best range seen
        if constexpr (GREEDY) {
            float cur_lo[4], cur_hi[4], step[4];
            double best[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                cur_lo[u] = lo[u];
                cur_hi[u] = hi[u];
                step[u] = (hi[u] - lo[u]) / num_bins_f;
                const float s0 = (hi[u] - lo[u]) / QMAXF;
                double e = 0.0;
#pragma unroll
                for (int c = 0; c < M; ++c) {
                    e += fq_sq_err(x[u][c].x, lo[u], hi[u], s0, QMAXF);
                    e += fq_sq_err(x[u][c].y, lo[u], hi[u], s0, QMAXF);
                    e += fq_sq_err(x[u][c].z, lo[u], hi[u], s0, QMAXF);
                    e += fq_sq_err(x[u][c].w, lo[u], hi[u], s0, QMAXF);
                }
                best[u] = row16_sum(e);
            }
            for (uint32_t it = 0; it < n_iter; ++it) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float c_lo = cur_lo[u] + step[u];
                    const float c_hi = cur_hi[u] - step[u];
                    const float s_lo = (cur_hi[u] - c_lo) / QMAXF;
                    const float s_hi = (c_hi - cur_lo[u]) / QMAXF;
                    double e_lo = 0.0, e_hi = 0.0;
#pragma unroll
                    for (int c = 0; c < M; ++c) {
                        e_lo += fq_sq_err(x[u][c].x, c_lo, cur_hi[u], s_lo, QMAXF);
                        e_lo += fq_sq_err(x[u][c].y, c_lo, cur_hi[u], s_lo, QMAXF);
                        e_lo += fq_sq_err(x[u][c].z, c_lo, cur_hi[u], s_lo, QMAXF);
                        e_lo += fq_sq_err(x[u][c].w, c_lo, cur_hi[u], s_lo, QMAXF);
                        e_hi += fq_sq_err(x[u][c].x, cur_lo[u], c_hi, s_hi, QMAXF);
                        e_hi += fq_sq_err(x[u][c].y, cur_lo[u], c_hi, s_hi, QMAXF);
                        e_hi += fq_sq_err(x[u][c].z, cur_lo[u], c_hi, s_hi, QMAXF);
                        e_hi += fq_sq_err(x[u][c].w, cur_lo[u], c_hi, s_hi, QMAXF);
                    }
                    e_lo = row16_sum(e_lo);
                    e_hi = row16_sum(e_hi);
                    const bool move_lo = e_lo < e_hi;
                    cur_lo[u] = move_lo ? c_lo : cur_lo[u];
                    cur_hi[u] = move_lo ? cur_hi[u] : c_hi;
                    const double e = move_lo ? e_lo : e_hi;
                    if (e < best[u]) {
                        best[u] = e;
                        lo[u] = cur_lo[u];
                        hi[u] = cur_hi[u];
                    }
                }
            }
        }

        // ---- quantize with the selected range, pack this lane's four codes per (row, chunk)
        float sc[4];
        uint32_t h[M][4];  // [chunk][row]: 4*BITS bits each
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            sc[u] = (hi[u] - lo[u]) / QMAXF;
#pragma unroll
            for (int c = 0; c < M; ++c) {
                const uint32_t q0 = (uint32_t)fq_code_f(x[u][c].x, lo[u], hi[u], sc[u], QMAXF);
                const uint32_t q1 = (uint32_t)fq_code_f(x[u][c].y, lo[u], hi[u], sc[u], QMAXF);
                const uint32_t q2 = (uint32_t)fq_code_f(x[u][c].z, lo[u], hi[u], sc[u], QMAXF);
                const uint32_t q3 = (uint32_t)fq_code_f(x[u][c].w, lo[u], hi[u], sc[u], QMAXF);
                h[c][u] = q0 | (q1 << BITS) | (q2 << (2 * BITS)) | (q3 << (3 * BITS));
                if (codes_out && !(skip & (1u << u)))
                    *reinterpret_cast<uint32_t *>(codes_out + (k0 + u) * (uint64_t)DIM + 64 * c + 4 * l) =
                        q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
            }
        }

        // ---- per-row parameters: lanes 0-3 of a group write scale, 4-7 bias, 8-11 min, 12-15 max
        {
            float *dst = q == 0 ? scale_out : q == 1 ? bias_out : q == 2 ? min_out : max_out;
            float v = 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float mine = q == 0 ? sc[u] : q == 1 ? lo[u] : q == 2 ? X_min[u] : X_max[u];
                v = j == u ? mine : v;
            }
            if (dst && !((skip >> j) & 1u)) dst[k0 + j] = v;
        }

        // ---- packed codes: after the quad transpose lane j owns 16 consecutive elements
        // (64c + 16q ..) of row k0 + j
        if (packed_out) {
            const bool live = !((skip >> j) & 1u);
            uint8_t *row = packed_out + (k0 + (uint64_t)j) * P;
#pragma unroll
            for (int c = 0; c < M; ++c) {
                uint32_t t[4] = {h[c][0], h[c][1], h[c][2], h[c][3]};
                quad_transpose(t, j);
                if constexpr (BITS == 8) {
                    if (live)
                        *reinterpret_cast<uint4 *>(row + 64 * c + 16 * q) = make_uint4(t[0], t[1], t[2], t[3]);
                } else if constexpr (BITS == 4) {
                    if (live)
                        *reinterpret_cast<uint2 *>(row + 32 * c + 8 * q) =
                            make_uint2(t[0] | (t[1] << 16), t[2] | (t[3] << 16));
                } else if constexpr (BITS == 2) {
                    if (live)
                        *reinterpret_cast<uint32_t *>(row + 16 * c + 4 * q) =
                            t[0] | (t[1] << 8) | (t[2] << 16) | (t[3] << 24);
                } else {  // 3 bits: 48 bits per lane; even quads append the next quad's 48 bits
                    const uint32_t w0 = t[0] | (t[1] << 12) | (t[2] << 24);  // stream bits 0..31
                    const uint32_t w1 = (t[2] >> 8) | (t[3] << 4);           // stream bits 32..47
                    const uint32_t n0 = __shfl_down(w0, 4);
                    const uint32_t n1 = __shfl_down(w1, 4);
                    if (live && !(q & 1)) {
                        uint32_t *dst = reinterpret_cast<uint32_t *>(row + 24 * c + 12 * (q >> 1));
                        dst[0] = w0;
                        dst[1] = w1 | (n0 << 16);
                        dst[2] = (n0 >> 16) | (n1 << 16);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Any other dim (dim % 4 == 0, dim * bits % 8 == 0): one wavefront per row, lanes stride over the
// row, which is re-read from cache for each pass.  Output bytes are produced one per lane-visit
// from the codes they cover, so no staging or barrier is needed.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_min(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ double row_sq_err(const float *__restrict__ x, uint32_t dim, int lane,
                                             float lo, float hi, float qmaxf) {
    const float s = (hi - lo) / qmaxf;
    double e = 0.0;
    for (uint32_t t = lane; t < dim; t += kWave) e += fq_sq_err(x[t], lo, hi, s, qmaxf);
    return wave_sum(e);
}

template <int BITS>
__global__ void __launch_bounds__(kBlock)
quantize_rows_generic_kernel(const float *__restrict__ table, uint64_t n_rows, uint32_t dim,
                             const uint32_t *__restrict__ row_ids, const uint64_t *__restrict__ n_dev,
                             uint64_t n_max, int mode, uint32_t n_iter, float num_bins_f,
                             float *__restrict__ scale_out, float *__restrict__ bias_out,
                             float *__restrict__ min_out, float *__restrict__ max_out,
                             uint8_t *__restrict__ codes_out, uint8_t *__restrict__ packed_out,
                             cnr_dev_errors *err) {
    constexpr int QMAX = (1 << BITS) - 1;
    constexpr float QMAXF = (float)QMAX;
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    const uint64_t P = (uint64_t)dim * BITS / 8;
    for (uint64_t k = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; k < n; k += n_waves) {
        const uint64_t r = row_ids ? (uint64_t)row_ids[k] : k;
        if (r >= n_rows) {  // uniform over the wave
            if (lane == 0) raise_flag(err, CNR_FLAG_ROW_ID);
            continue;
        }
        const float *__restrict__ x = table + r * (uint64_t)dim;
        float mn = x[0], mx = x[0];
        for (uint32_t t = lane; t < dim; t += kWave) {
            mn = fminf(mn, x[t]);
            mx = fmaxf(mx, x[t]);
        }
        const float X_min = wave_min(mn) + 0.0f, X_max = wave_max(mx) + 0.0f;
        float lo = X_min, hi = X_max;
        if (mode == kModeSymmetric) {
            const float a = fmaxf(fabsf(X_min), fabsf(X_max));
            lo = -a + 0.0f;
            hi = a;
        } else if (mode == kModeGreedy) {
            float cur_lo = lo, cur_hi = hi;
            const float step = (hi - lo) / num_bins_f;
            double best = row_sq_err(x, dim, lane, lo, hi, QMAXF);
            for (uint32_t it = 0; it < n_iter; ++it) {
                const float c_lo = cur_lo + step, c_hi = cur_hi - step;
                const double e_lo = row_sq_err(x, dim, lane, c_lo, cur_hi, QMAXF);
                const double e_hi = row_sq_err(x, dim, lane, cur_lo, c_hi, QMAXF);
                const bool move_lo = e_lo < e_hi;
                if (move_lo) cur_lo = c_lo; else cur_hi = c_hi;
                const double e = move_lo ? e_lo : e_hi;
                if (e < best) {
                    best = e;
                    lo = cur_lo;
                    hi = cur_hi;
                }
            }
        }
        const float s = (hi - lo) / QMAXF;
        if (lane == 0) {
            scale_out[k] = s;
            bias_out[k] = lo;
            if (min_out) min_out[k] = X_min;
            if (max_out) max_out[k] = X_max;
        }
        if (codes_out)
            for (uint32_t t = lane; t < dim; t += kWave)
                codes_out[k * (uint64_t)dim + t] = (uint8_t)fq_code_f(x[t], lo, hi, s, QMAXF);
        if (packed_out) {
            uint8_t *out = packed_out + k * P;
            for (uint64_t b = lane; b < P; b += kWave) {
                const uint32_t first = (uint32_t)((8 * b) / BITS);
                const uint32_t last = (uint32_t)((8 * b + 7) / BITS);
                uint32_t byte = 0;
                for (uint32_t e = first; e <= last; ++e) {
                    const uint32_t code = (uint32_t)fq_code_f(x[e], lo, hi, s, QMAXF);
                    const int shift = (int)(e * BITS) - (int)(8 * b);  // stream position of code bit 0
                    byte |= shift >= 0 ? (code << shift) : (code >> -shift);
                }
                out[b] = (uint8_t)byte;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Stand-alone dense packing of one-code-per-byte input: one output byte per thread-visit.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ void __launch_bounds__(kBlock)
pack_kernel(const uint8_t *__restrict__ codes, const uint64_t *__restrict__ n_dev, uint64_t n_max,
            uint32_t dim, uint8_t *__restrict__ packed) {
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const uint64_t P = (uint64_t)dim * BITS / 8;
    const uint64_t total = n * P;
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    for (uint64_t o = (uint64_t)blockIdx.x * kBlock + threadIdx.x; o < total; o += stride) {
        const uint64_t k = o / P, b = o - k * P;
        const uint8_t *row = codes + k * (uint64_t)dim;
        const uint32_t first = (uint32_t)((8 * b) / BITS);
        const uint32_t last = (uint32_t)((8 * b + 7) / BITS);
        uint32_t byte = 0;
        for (uint32_t e = first; e <= last; ++e) {
            const uint32_t code = row[e] & ((1u << BITS) - 1u);
            const int shift = (int)(e * BITS) - (int)(8 * b);
            byte |= shift >= 0 ? (code << shift) : (code >> -shift);
        }
        packed[o] = (uint8_t)byte;
    }
}

struct QuantArgs {
    const float *table;
    uint64_t n_rows;
    uint32_t dim;
    const uint32_t *row_ids;
    const uint64_t *n_dev;
    uint64_t n_max;
    int mode;
    uint32_t n_iter;
    float num_bins_f;
    float *scale, *bias, *row_min, *row_max;
    uint8_t *codes, *packed;
};

template <int M, int BITS, bool GREEDY>
void launch_rows16(cnr_ctx *ctx, const QuantArgs &a, hipStream_t s) {
    const unsigned grid = cnr_grid(ctx, a.n_max, 16u * kWavesPerBlock, 8);
    hipLaunchKernelGGL((quantize_rows16_kernel<M, BITS, GREEDY>), dim3(grid), dim3(kBlock), 0, s, a.table,
                       a.n_rows, a.row_ids, a.n_dev, a.n_max, a.mode, a.n_iter, a.num_bins_f, a.scale,
                       a.bias, a.row_min, a.row_max, a.codes, a.packed, ctx->dev_err);
}

template <int M, int BITS>
void launch_rows16_mode(cnr_ctx *ctx, const QuantArgs &a, hipStream_t s) {
    if (a.mode == kModeGreedy && a.n_iter > 0)
        launch_rows16<M, BITS, true>(ctx, a, s);
    else
        launch_rows16<M, BITS, false>(ctx, a, s);
}

template <int BITS>
void launch_bits(cnr_ctx *ctx, const QuantArgs &a, hipStream_t s) {
    if (a.dim == 64) return launch_rows16_mode<1, BITS>(ctx, a, s);
    if (a.dim == 128) return launch_rows16_mode<2, BITS>(ctx, a, s);
    if (a.dim == 256) return launch_rows16_mode<4, BITS>(ctx, a, s);
    const unsigned grid = cnr_grid(ctx, a.n_max, kWavesPerBlock, 8);
    hipLaunchKernelGGL((quantize_rows_generic_kernel<BITS>), dim3(grid), dim3(kBlock), 0, s, a.table,
                       a.n_rows, a.dim, a.row_ids, a.n_dev, a.n_max, a.mode, a.n_iter, a.num_bins_f,
                       a.scale, a.bias, a.row_min, a.row_max, a.codes, a.packed, ctx->dev_err);
}

}  // namespace

extern "C" {

cnr_status cnr_quantize_rows(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                             const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                             int bits, cnr_range_mode mode, const cnr_greedy_params *greedy,
                             float *scale, float *bias, float *row_min, float *row_max,
                             uint8_t *codes_u8, uint8_t *packed, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (mode != CNR_RANGE_MINMAX && mode != CNR_RANGE_GREEDY && mode != CNR_RANGE_SYMMETRIC) return CNR_E_INVALID;
    if (mode == CNR_RANGE_GREEDY && !greedy) return CNR_E_INVALID;
    if (n_max == 0) return CNR_OK;
    if (!table || !scale || !bias || n_rows == 0 || n_rows >= (1ull << 32)) return CNR_E_INVALID;
    if (((uintptr_t)table % 16) || ((uintptr_t)packed % 16) || ((uintptr_t)codes_u8 % 4) ||
        ((uintptr_t)scale % 4) || ((uintptr_t)bias % 4) || ((uintptr_t)row_min % 4) ||
        ((uintptr_t)row_max % 4) || ((uintptr_t)row_ids % 4) || ((uintptr_t)n_dev % 8))
        return CNR_E_ALIGN;
    QuantArgs a;
    a.table = table; a.n_rows = n_rows; a.dim = dim; a.row_ids = row_ids; a.n_dev = n_dev; a.n_max = n_max;
    a.mode = (int)mode;
    a.n_iter = mode == CNR_RANGE_GREEDY ? cnr_greedy_iterations(greedy->num_bins, greedy->ratio) : 0;
    a.num_bins_f = mode == CNR_RANGE_GREEDY ? (float)greedy->num_bins : 1.0f;
    a.scale = scale; a.bias = bias; a.row_min = row_min; a.row_max = row_max;
    a.codes = codes_u8; a.packed = packed;
    hipStream_t s = as_stream(stream);
    switch (bits) {
        case 2: launch_bits<2>(ctx, a, s); break;
        case 3: launch_bits<3>(ctx, a, s); break;
        case 4: launch_bits<4>(ctx, a, s); break;
        default: launch_bits<8>(ctx, a, s); break;
    }
    return cnr_launch_status(ctx);
}

cnr_status cnr_pack(cnr_ctx *ctx, const uint8_t *codes_u8, const uint64_t *n_dev, uint64_t n_max,
                    uint32_t dim, int bits, uint8_t *packed, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (n_max == 0) return CNR_OK;
    if (!codes_u8 || !packed) return CNR_E_INVALID;
    if ((uintptr_t)n_dev % 8) return CNR_E_ALIGN;
    const uint64_t bytes = n_max * cnr_packed_row_bytes(dim, bits);
    const unsigned grid = cnr_grid(ctx, bytes, kBlock, 16);
    hipStream_t s = as_stream(stream);
    switch (bits) {
        case 2: hipLaunchKernelGGL(pack_kernel<2>, dim3(grid), dim3(kBlock), 0, s, codes_u8, n_dev, n_max, dim, packed); break;
        case 3: hipLaunchKernelGGL(pack_kernel<3>, dim3(grid), dim3(kBlock), 0, s, codes_u8, n_dev, n_max, dim, packed); break;
        case 4: hipLaunchKernelGGL(pack_kernel<4>, dim3(grid), dim3(kBlock), 0, s, codes_u8, n_dev, n_max, dim, packed); break;
        default: hipLaunchKernelGGL(pack_kernel<8>, dim3(grid), dim3(kBlock), 0, s, codes_u8, n_dev, n_max, dim, packed); break;
    }
    return cnr_launch_status(ctx);
}

}  // extern "C"
