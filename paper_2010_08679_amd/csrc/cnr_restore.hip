// Restore: unpack, de-quantize (x = scale * x_q + zero_point, Section 5.2 Approach 1) and scatter
// whole rows over a stale baseline table (Section 5.1: resume = baseline + latest incremental).
#include "cnr_common.h"

namespace {

// Bits [pos, pos + BITS*4) of a row's packed stream, pos = 4 * first_element * BITS, returned with
// the first element's code in the low bits.  `p` points at the row's first packed byte.
template <int BITS>
__device__ __forceinline__ uint32_t load_four_codes(const uint8_t *__restrict__ p, uint32_t first_element) {
    if constexpr (BITS == 8) {
        return *reinterpret_cast<const uint32_t *>(p + first_element);
    } else if constexpr (BITS == 4) {
        return *reinterpret_cast<const uint16_t *>(p + first_element / 2);
    } else if constexpr (BITS == 2) {
        return p[first_element / 4];
    } else {
        const uint32_t bit = first_element * 3;  // multiple of 12: starts on a byte or a nibble
        const uint32_t two = (uint32_t)p[bit >> 3] | ((uint32_t)p[(bit >> 3) + 1] << 8);
        return (two >> (bit & 7u)) & 0xFFFu;
    }
}

// Fast path, dim = 64 * M: same lane-to-element mapping as the encoder (sixteen lanes per row, lane
// l owns elements 64c + 4l .. + 3 of every chunk c, four rows per group in flight), so the fp32
// rows leave as 16-byte stores that cover 256 contiguous bytes per group.
template <int M, int BITS>
__global__ void __launch_bounds__(kBlock)
restore_rows16_kernel(float *__restrict__ table, uint64_t n_rows, const uint32_t *__restrict__ row_ids,
                      const uint64_t *__restrict__ n_dev, uint64_t n_max,
                      const uint8_t *__restrict__ packed, const float *__restrict__ scale,
                      const float *__restrict__ bias, cnr_dev_errors *err) {
    constexpr int DIM = 64 * M;
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane >> 4;
    const int l = lane & 15;
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    const uint64_t wave_id = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    for (uint64_t batch = wave_id; batch * 16u < n; batch += n_waves) {
        const uint64_t k0 = batch * 16u + 4u * (uint64_t)g;
        uint32_t h[4][M];
        float s[4], b[4];
        uint64_t dst[4];
        bool live[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint64_t k = k0 + u;
            live[u] = k < n;
            if (!live[u]) k = n - 1;
            const uint64_t r = row_ids ? (uint64_t)row_ids[k] : k;
            if (r >= n_rows) {
                if (live[u] && l == 0) raise_flag(err, CNR_FLAG_ROW_ID);
                live[u] = false;
            }
            dst[u] = r * (uint64_t)DIM + 4u * (uint64_t)l;
            s[u] = scale[k];
            b[u] = bias[k];
#pragma unroll
            for (int c = 0; c < M; ++c) h[u][c] = load_four_codes<BITS>(packed + k * P, 64 * c + 4 * l);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!live[u]) continue;
#pragma unroll
            for (int c = 0; c < M; ++c) {
                const uint32_t w = h[u][c];
                float4 v;
                v.x = s[u] * (float)(w & MASK) + b[u];
                v.y = s[u] * (float)((w >> BITS) & MASK) + b[u];
                v.z = s[u] * (float)((w >> (2 * BITS)) & MASK) + b[u];
                v.w = s[u] * (float)((w >> (3 * BITS)) & MASK) + b[u];
                store_stream<f32x4>(table + dst[u] + 64 * c, f32x4{v.x, v.y, v.z, v.w});
            }
        }
    }
}

// Any other dim: one wavefront per row, lanes stride over the elements.
template <int BITS>
__global__ void __launch_bounds__(kBlock)
restore_rows_generic_kernel(float *__restrict__ table, uint64_t n_rows, uint32_t dim,
                            const uint32_t *__restrict__ row_ids, const uint64_t *__restrict__ n_dev,
                            uint64_t n_max, const uint8_t *__restrict__ packed,
                            const float *__restrict__ scale, const float *__restrict__ bias,
                            cnr_dev_errors *err) {
    constexpr uint32_t MASK = (1u << BITS) - 1u;
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
        if (r >= n_rows) {
            if (lane == 0) raise_flag(err, CNR_FLAG_ROW_ID);
            continue;
        }
        const uint8_t *__restrict__ in = packed + k * P;
        const float s = scale[k], b = bias[k];
        float *__restrict__ out = table + r * (uint64_t)dim;
        for (uint32_t e = lane; e < dim; e += kWave) {
            const uint64_t bit = (uint64_t)e * BITS;
            uint32_t two = in[bit >> 3];
            if (((bit & 7u) + BITS) > 8u) two |= (uint32_t)in[(bit >> 3) + 1] << 8;
            const uint32_t code = (two >> (bit & 7u)) & MASK;
            out[e] = s * (float)code + b;
        }
    }
}

template <int M, int BITS>
void launch_restore16(cnr_ctx *ctx, hipStream_t st, float *table, uint64_t n_rows, const uint32_t *row_ids,
                      const uint64_t *n_dev, uint64_t n_max, const uint8_t *packed, const float *scale,
                      const float *bias) {
    const unsigned grid = cnr_grid(ctx, n_max, 16u * kWavesPerBlock,
                                   cnr_resident_blocks_per_cu<restore_rows16_kernel<M, BITS>>());
    hipLaunchKernelGGL((restore_rows16_kernel<M, BITS>), dim3(grid), dim3(kBlock), 0, st, table, n_rows,
                       row_ids, n_dev, n_max, packed, scale, bias, ctx->dev_err);
}

template <int BITS>
void launch_restore(cnr_ctx *ctx, hipStream_t st, float *table, uint64_t n_rows, uint32_t dim,
                    const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                    const uint8_t *packed, const float *scale, const float *bias) {
    if (dim == 64)
        launch_restore16<1, BITS>(ctx, st, table, n_rows, row_ids, n_dev, n_max, packed, scale, bias);
    else if (dim == 128)
        launch_restore16<2, BITS>(ctx, st, table, n_rows, row_ids, n_dev, n_max, packed, scale, bias);
    else if (dim == 256)
        launch_restore16<4, BITS>(ctx, st, table, n_rows, row_ids, n_dev, n_max, packed, scale, bias);
    else
        hipLaunchKernelGGL((restore_rows_generic_kernel<BITS>), dim3(cnr_grid(ctx, n_max, kWavesPerBlock, 8)),
                           dim3(kBlock), 0, st, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale,
                           bias, ctx->dev_err);
}

}  // namespace

extern "C" cnr_status cnr_restore_rows(cnr_ctx *ctx, float *table, uint64_t n_rows, uint32_t dim,
                                       const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                                       int bits, const uint8_t *packed, const float *scale,
                                       const float *bias, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (n_max == 0) return CNR_OK;
    if (!table || !packed || !scale || !bias || n_rows == 0 || n_rows >= (1ull << 32)) return CNR_E_INVALID;
    if (((uintptr_t)table % 16) || ((uintptr_t)packed % 16) || ((uintptr_t)scale % 4) ||
        ((uintptr_t)bias % 4) || ((uintptr_t)row_ids % 4) || ((uintptr_t)n_dev % 8))
        return CNR_E_ALIGN;
    hipStream_t s = as_stream(stream);
    switch (bits) {
        case 2: launch_restore<2>(ctx, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias); break;
        case 3: launch_restore<3>(ctx, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias); break;
        case 4: launch_restore<4>(ctx, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias); break;
        default: launch_restore<8>(ctx, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias); break;
    }
    return cnr_launch_status(ctx);
}
