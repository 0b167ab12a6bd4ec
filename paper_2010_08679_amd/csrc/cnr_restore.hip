// Restore: unpack, de-quantize (x = scale * x_q + zero_point, Section 5.2 Approach 1) and scatter
// whole rows over a stale baseline table (Section 5.1: resume = baseline + latest incremental).
#include "cnr_common.h"

namespace {

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

// Shape of the kernel for rows of DIM = 16 * Q floats: LR lanes per group of four rows (16, or the
// row's 4 * Q units of 16 bytes when it is shorter than 64 floats), M chunks of 64 floats per row.
template <int Q>
struct RestoreShape {
    static constexpr int DIM = 16 * Q;
    static constexpr int LR = Q >= 4 ? 16 : 4 * Q;
    static constexpr int M = Q >= 4 ? Q / 4 : 1;
    static constexpr int ROWS = 4 * (kWave / LR);  // rows per wave and pass
};

// How the packed codes of a pass reach the lanes.  Quad lane j of quad q needs the codes of the 16
// consecutive elements 64c + 16q .. of row k0 + j, for every chunk c: 2 * BITS bytes per chunk.
//   direct  one load per lane, straight from memory: rows of one chunk at 2, 4 or 8 bits, where the
//           lanes of a wave together read every byte of the pass's codes exactly once;
//   staged  rows of several chunks (one load per chunk would have the wave pass over the same lines
//           once per chunk) and every row at 3 bits (a lane's 6 bytes straddle dword boundaries): the
//           codes of the pass's ROWS rows are contiguous in memory, ROWS * P bytes, so the wave fetches
//           them 16 bytes per lane, each line once, parks them in its own piece of LDS and every lane
//           picks its words from there.  (Measured on 4 M rows of 128 floats with cold inputs: 3 bits
//           495 -> 456 us, the other widths 2 % faster; on rows of 64 floats 3 bits 410 -> 373 us.)
template <int Q, int BITS>
struct CodeFetch {
    using S = RestoreShape<Q>;
    static constexpr int P = S::DIM * BITS / 8;                  // packed bytes per row
    static constexpr bool STAGED = S::M >= 2 || BITS == 3;
    static constexpr int BLOCK = S::ROWS * P;                    // packed bytes per pass, a multiple of 16
    static constexpr int LOADS = STAGED ? (BLOCK + 1023) / 1024 : 1;   // 16-byte loads per lane and pass
    static constexpr int STAGE_BYTES = STAGED ? LOADS * 1024 : 0;      // LDS per wave
    static constexpr int WORDS = BITS == 8 ? 4 : BITS == 4 ? 2 : BITS == 3 ? 2 : 1;  // per lane and chunk
};

// What one group of LR lanes needs to restore its four rows k0 .. k0+3: ids, scales and biases (the
// same 16 bytes for every lane of the group, one load each) and the packed codes, as this lane's words
// (direct) or as this lane's 16-byte units of the pass's block (staged).
template <int Q, int BITS>
struct RestoreInput {
    uint4 ids;
    float4 scale, bias;
    u32x4 raw[CodeFetch<Q, BITS>::LOADS];
};

template <int Q, int BITS>
__device__ __forceinline__ void fetch_restore_input(const uint32_t *__restrict__ row_ids,
                                                    const uint8_t *__restrict__ packed,
                                                    const float *__restrict__ scale,
                                                    const float *__restrict__ bias, uint64_t n_max, uint64_t pass_row0,
                                                    int lane, int g, int q, int j, RestoreInput<Q, BITS> &in) {
    using F = CodeFetch<Q, BITS>;
    constexpr uint64_t P = F::P;
    const uint64_t k0 = pass_row0 + 4u * (uint64_t)g;
    if (k0 + 3 < n_max) {  // every buffer holds n_max rows: whole 16-byte loads
        in.ids = row_ids ? *reinterpret_cast<const uint4 *>(row_ids + k0)
                         : make_uint4((uint32_t)k0, (uint32_t)k0 + 1, (uint32_t)k0 + 2, (uint32_t)k0 + 3);
        in.scale = *reinterpret_cast<const float4 *>(scale + k0);
        in.bias = *reinterpret_cast<const float4 *>(bias + k0);
    } else {
        uint32_t id[4] = {0, 0, 0, 0};
        float sc[4] = {0, 0, 0, 0}, bi[4] = {0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k0 + u < n_max) {
                id[u] = row_ids ? row_ids[k0 + u] : (uint32_t)(k0 + u);
                sc[u] = scale[k0 + u];
                bi[u] = bias[k0 + u];
            }
        in.ids = make_uint4(id[0], id[1], id[2], id[3]);
        in.scale = make_float4(sc[0], sc[1], sc[2], sc[3]);
        in.bias = make_float4(bi[0], bi[1], bi[2], bi[3]);
    }
    if constexpr (F::STAGED) {
        // the buffer holds n_max rows: the pass's block, or what is left of the buffer
        const uint64_t left = n_max - pass_row0;  // >= 1
        const uint32_t bytes = left < (uint64_t)F::S::ROWS ? (uint32_t)(left * P) : (uint32_t)F::BLOCK;
        const uint8_t *src = packed + pass_row0 * P;
#pragma unroll
        for (int i = 0; i < F::LOADS; ++i) {
            const uint32_t off = (uint32_t)(i * kWave + lane) * 16u;
            u32x4 v = {0, 0, 0, 0};
            if (off + 16u <= bytes) {
                v = load_stream<u32x4>(src + off);
            } else if (off < bytes) {  // the buffer ends inside this unit (P is even): halfword by halfword
                uint32_t h[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    h[t] = off + 2u * t < bytes ? (uint32_t)*reinterpret_cast<const uint16_t *>(src + off + 2 * t) : 0u;
                v = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
            }
            in.raw[i] = v;
        }
    } else {  // one chunk per row, 2 * BITS bytes per lane
        const bool row_in_buffer = k0 + (uint64_t)j < n_max;
        const uint8_t *src = packed + (k0 + (uint64_t)j) * P + 2 * BITS * q;
        u32x4 v = {0, 0, 0, 0};
        if constexpr (BITS == 8) {
            if (row_in_buffer) v = load_stream<u32x4>(src);
        } else if constexpr (BITS == 4) {
            if (row_in_buffer) {
                const u32x2 t = load_stream<u32x2>(src);
                v.x = t.x; v.y = t.y;
            }
        } else {
            if (row_in_buffer) v.x = load_stream<uint32_t>(src);
        }
        in.raw[0] = v;
    }
}

// This lane's words of chunk c: from its registers (direct), or from the wave's LDS stage, which
// park_codes filled with the pass's block.  w[0 .. WORDS) = 16 * BITS code bits of the elements
// 64c + 16q .. of row k0 + j, first element lowest; at 3 bits they start at bit 16 * (q & 1) of w[0].
template <int Q, int BITS>
__device__ __forceinline__ void park_codes(unsigned char *stage, int lane, const RestoreInput<Q, BITS> &in) {
    using F = CodeFetch<Q, BITS>;
    if constexpr (F::STAGED) {
        __builtin_amdgcn_wave_barrier();  // the reads of the pass before are done (LDS is in order per wave)
#pragma unroll
        for (int i = 0; i < F::LOADS; ++i) *reinterpret_cast<u32x4 *>(stage + (i * kWave + lane) * 16) = in.raw[i];
        __builtin_amdgcn_wave_barrier();
    }
}
template <int Q, int BITS>
__device__ __forceinline__ void chunk_words(const unsigned char *stage, int c, int g, int q, int j,
                                            const RestoreInput<Q, BITS> &in, uint32_t (&w)[CodeFetch<Q, BITS>::WORDS]) {
    using F = CodeFetch<Q, BITS>;
    if constexpr (!F::STAGED) {
        w[0] = in.raw[0].x;
        if constexpr (F::WORDS >= 2) w[1] = in.raw[0].y;
        if constexpr (F::WORDS >= 4) { w[2] = in.raw[0].z; w[3] = in.raw[0].w; }
    } else {
        const unsigned char *row = stage + (4 * g + j) * F::P;
        if constexpr (BITS == 8) {
            const uint4 v = *reinterpret_cast<const uint4 *>(row + 64 * c + 16 * q);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else if constexpr (BITS == 4) {
            const uint2 v = *reinterpret_cast<const uint2 *>(row + 32 * c + 8 * q);
            w[0] = v.x; w[1] = v.y;
        } else if constexpr (BITS == 2) {
            w[0] = *reinterpret_cast<const uint32_t *>(row + 16 * c + 4 * q);
        } else if constexpr (Q == 1) {  // 3 bits, rows of 6 bytes: at a two-byte boundary
            const uint16_t *h = reinterpret_cast<const uint16_t *>(row);
            w[0] = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
            w[1] = h[2];
        } else {
            // 3 bits: a quad's 48 bits start at byte 24c + 6q of the row, which is a dword boundary for
            // even quads and two bytes past one for odd quads: the two dwords around them
            const uint32_t *d = reinterpret_cast<const uint32_t *>(row + 24 * c + 6 * q - 2 * (q & 1));
            w[0] = d[0];
            w[1] = d[1];
        }
    }
}

// Fast path, dim = 16 * Q in {16, 32, 64, 128, 256}: the mirror image of the encoder.  LR lanes share
// a row, four rows per group; every lane gets the codes of 16 consecutive elements of one row and
// chunk (CodeFetch) and a 4x4 transpose inside each quad turns them into "lane l owns elements
// 64c + 4l .. + 3 of each of the four rows", so the fp32 rows leave as 16-byte streaming stores that
// cover up to 256 contiguous bytes per row.  The input of the next batch is requested before the
// current batch is de-quantized and stored.
struct RestoreJob {
    float *table;
    uint64_t n_rows;
    const uint32_t *row_ids;
    const uint64_t *n_dev;
    uint64_t n_max;
    const uint8_t *packed;
    const float *scale, *bias;
    uint32_t n_waves;  // waves of the grid
};
template <int Q, int BITS>
__device__ __forceinline__ void restore_table(const RestoreJob &a, cnr_dev_errors *err,
                                              unsigned char *stage /* this wave's STAGE_BYTES of LDS */) {
    using S = RestoreShape<Q>;
    using F = CodeFetch<Q, BITS>;
    constexpr int DIM = S::DIM, M = S::M, LR = S::LR;
    constexpr uint64_t ROWS = S::ROWS;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    float *__restrict__ table = a.table;
    const uint32_t *__restrict__ row_ids = a.row_ids;
    const uint64_t *__restrict__ n_dev = a.n_dev;
    const uint8_t *__restrict__ packed = a.packed;
    const float *__restrict__ scale = a.scale, *__restrict__ bias = a.bias;
    const uint64_t n_rows = a.n_rows, n_max = a.n_max;
    const uint64_t n = live_rows(n_dev, n_max);
    const int lane = tid_x() & (kWave - 1);
    const int g = lane / LR;
    const int l = lane % LR;
    const int q = l >> 2;
    const int j = l & 3;
    const uint32_t n_waves = a.n_waves;
    uint64_t batch = wave_in_grid();
    if (batch * ROWS >= n) return;
    RestoreInput<Q, BITS> cur, nxt;
    fetch_restore_input<Q, BITS>(row_ids, packed, scale, bias, n_max, batch * ROWS, lane, g, q, j, cur);
    for (;;) {
        const uint64_t next = batch + n_waves;
        const bool has_next = next * ROWS < n;  // uniform over the wave
        if (has_next) fetch_restore_input<Q, BITS>(row_ids, packed, scale, bias, n_max, next * ROWS, lane, g, q, j, nxt);
        park_codes<Q, BITS>(stage, lane, cur);

        const uint64_t k0 = batch * ROWS + 4u * (uint64_t)g;
        const uint32_t rid[4] = {cur.ids.x, cur.ids.y, cur.ids.z, cur.ids.w};
        const float s[4] = {cur.scale.x, cur.scale.y, cur.scale.z, cur.scale.w};
        const float b[4] = {cur.bias.x, cur.bias.y, cur.bias.z, cur.bias.w};
#pragma unroll
        for (int c = 0; c < M; ++c) {
            uint32_t w[F::WORDS];
            chunk_words<Q, BITS>(stage, c, g, q, j, cur, w);
            // t[i] = 4*BITS code bits of elements 64c + 16q + 4i .. + 3 of row k0 + j
            uint32_t t[4];
            if constexpr (BITS == 8) {
                t[0] = w[0]; t[1] = w[1]; t[2] = w[2]; t[3] = w[3];
            } else if constexpr (BITS == 4) {
                t[0] = w[0] & 0xFFFFu; t[1] = w[0] >> 16;
                t[2] = w[1] & 0xFFFFu; t[3] = w[1] >> 16;
            } else if constexpr (BITS == 2) {
                t[0] = w[0] & 0xFFu; t[1] = (w[0] >> 8) & 0xFFu;
                t[2] = (w[0] >> 16) & 0xFFu; t[3] = w[0] >> 24;
            } else {  // the 48 bits start at bit 16 of w[0] in odd quads
                const uint32_t lo32 = (q & 1) ? ((w[0] >> 16) | (w[1] << 16)) : w[0];
                const uint32_t hi16 = (q & 1) ? (w[1] >> 16) : (w[1] & 0xFFFFu);
                t[0] = lo32 & 0xFFFu; t[1] = (lo32 >> 12) & 0xFFFu;
                t[2] = (lo32 >> 24) | ((hi16 & 0xFu) << 8); t[3] = hi16 >> 4;
            }
            quad_transpose(t, j);  // now t[u] = codes of elements 64c + 4l .. + 3 of row k0 + u
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool live = k0 + u < n && rid[u] < n_rows;
                if (!live) continue;
                const uint32_t cw = t[u];
                f32x4 v;
                v.x = s[u] * (float)(cw & MASK) + b[u];
                v.y = s[u] * (float)((cw >> BITS) & MASK) + b[u];
                v.z = s[u] * (float)((cw >> (2 * BITS)) & MASK) + b[u];
                v.w = s[u] * (float)((cw >> (3 * BITS)) & MASK) + b[u];
                float *dst = table + (uint64_t)rid[u] * DIM + 64 * c + 4 * l;
                if constexpr (M == 1 && BITS <= 4)  // one instruction writes the whole row: straight to memory
                    store_stream_through(dst, v);
                else
                    store_stream<f32x4>(dst, v);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k0 + u < n && rid[u] >= n_rows && l == 0) raise_flag(err, CNR_FLAG_ROW_ID);

        if (!has_next) break;
        cur = nxt;
        batch = next;
    }
}

// One launch takes up to CNR_MAX_BATCH tables (grid y = table; a slice of a long list counts as a
// table), swept one after the other because workgroups are handed out x first, as for the encode.
struct RestoreBatch {
    RestoreJob job[CNR_MAX_BATCH];
};
// The register budget is pinned to eight waves per SIMD (64 registers), which every shape meets without
// spilling except rows of 256 floats at 8 bits (left to the compiler: 84 registers, five waves): left
// alone, a few shapes land two registers above the step.
template <int Q, int BITS>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(Q == 16 && BITS == 8 ? 5 : 8, 8)))
restore_rows16_kernel(const RestoreBatch b, cnr_dev_errors *err) {
    constexpr int kStage = CodeFetch<Q, BITS>::STAGE_BYTES;
    __shared__ __align__(16) unsigned char stages[kStage ? kWavesPerBlock * kStage : 16];
    const RestoreJob &a = b.job[wg_y()];
    if (wg_x() * kWavesPerBlock >= a.n_waves) return;  // fewer workgroups than the launch's largest table
    restore_table<Q, BITS>(a, err, stages + (tid_x() / kWave) * kStage);
}

// Other row lengths: LPR lanes per row (a power of two, at least the row's number of 16-byte units up
// to 64), 64 / LPR rows per wave and pass; lane j takes the units j, j + LPR, ... of its row: it reads
// the unit's 4 * BITS code bits (one, two or four bytes; at 3 bits the three bytes that hold the
// unit and its pair partner) and stores 16 bytes.
template <int LPR, int BITS>
__global__ void __launch_bounds__(kBlock) restore_strided_kernel(const RestoreJob a, uint32_t dim, cnr_dev_errors *err) {
    constexpr int kRowsPerPass = kWave / LPR;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const uint64_t n = live_rows(a.n_dev, a.n_max);
    const uint32_t n4 = dim / 4;
    const uint64_t P = (uint64_t)dim * BITS / 8;
    const int lane = tid_x() & (kWave - 1);
    const uint32_t j = lane % LPR;
    const uint32_t n_waves = a.n_waves;
    const uint32_t trips = (n4 + LPR - 1) / LPR;
    for (uint64_t pass = wave_in_grid(); pass * kRowsPerPass < n; pass += n_waves) {
        const uint64_t k = pass * kRowsPerPass + lane / LPR;
        const uint64_t kc = k < n ? k : n - 1;  // rows past the end repeat the last one; nothing of theirs is stored
        const uint64_t r = a.row_ids ? (uint64_t)a.row_ids[kc] : kc;
        const bool in_table = r < a.n_rows;
        const bool live = k < n && in_table;
        if (k < n && !in_table && j == 0) raise_flag(err, CNR_FLAG_ROW_ID);
        const uint8_t *in = a.packed + kc * P;
        const float s = a.scale[kc], b = a.bias[kc];
        f32x4 *out = reinterpret_cast<f32x4 *>(a.table + (in_table ? r : 0) * (uint64_t)dim);
        for (uint32_t trip = 0; trip < trips; ++trip) {
            const uint32_t u = j + trip * LPR;
            const bool mine = u < n4;
            const uint32_t uc = mine ? u : 0;
            uint32_t w;  // the unit's four codes, first element lowest
            if constexpr (BITS == 8) {
                w = *reinterpret_cast<const uint32_t *>(in + 4 * uc);
            } else if constexpr (BITS == 4) {
                w = *reinterpret_cast<const uint16_t *>(in + 2 * uc);
            } else if constexpr (BITS == 2) {
                w = in[uc];
            } else {  // units come in pairs (dim % 8 == 0): three bytes hold the even one's 12 bits, then the odd one's
                const uint8_t *i3 = in + 3 * (uc >> 1);
                const uint32_t both = (uint32_t)i3[0] | ((uint32_t)i3[1] << 8) | ((uint32_t)i3[2] << 16);
                w = (uc & 1) ? both >> 12 : both & 0xFFFu;
            }
            f32x4 v;
            v.x = s * (float)(w & MASK) + b;
            v.y = s * (float)((w >> BITS) & MASK) + b;
            v.z = s * (float)((w >> (2 * BITS)) & MASK) + b;
            v.w = s * (float)((w >> (3 * BITS)) & MASK) + b;
            if (mine && live) store_stream<f32x4>(out + u, v);
        }
    }
}

template <int Q, int BITS>
void launch_restore16(cnr_ctx *ctx, hipStream_t st, RestoreBatch &b, uint32_t n) {
    unsigned grid = 1;
    for (uint32_t i = 0; i < n; ++i) {
        const unsigned g = cnr_row_grid(b.job[i].n_max, (uint64_t)RestoreShape<Q>::ROWS * kWavesPerBlock);
        b.job[i].n_waves = g * kWavesPerBlock;
        if (g > grid) grid = g;
    }
    hipLaunchKernelGGL((restore_rows16_kernel<Q, BITS>), dim3(grid, n), dim3(kBlock), 0, st, b, ctx->dev_err);
}
template <int BITS>
void launch_restore16_bits(cnr_ctx *ctx, hipStream_t st, uint32_t dim, RestoreBatch &b, uint32_t n) {
    switch (dim) {
        case 16: return launch_restore16<1, BITS>(ctx, st, b, n);
        case 32: return launch_restore16<2, BITS>(ctx, st, b, n);
        case 64: return launch_restore16<4, BITS>(ctx, st, b, n);
        case 128: return launch_restore16<8, BITS>(ctx, st, b, n);
        default: return launch_restore16<16, BITS>(ctx, st, b, n);
    }
}

template <int LPR, int BITS>
void launch_restore_strided(cnr_ctx *ctx, hipStream_t st, uint32_t dim, RestoreJob &a) {
    const unsigned grid = cnr_row_grid(a.n_max, (uint64_t)(kWave / LPR) * kWavesPerBlock);
    a.n_waves = grid * kWavesPerBlock;
    hipLaunchKernelGGL((restore_strided_kernel<LPR, BITS>), dim3(grid), dim3(kBlock), 0, st, a, dim, ctx->dev_err);
}

// other row lengths: one table per launch
template <int BITS>
void launch_restore(cnr_ctx *ctx, hipStream_t st, uint32_t dim, RestoreJob &a) {
    const uint32_t n4 = dim / 4;
    if (n4 <= 4) return launch_restore_strided<4, BITS>(ctx, st, dim, a);
    if (n4 <= 8) return launch_restore_strided<8, BITS>(ctx, st, dim, a);
    if (n4 <= 16) return launch_restore_strided<16, BITS>(ctx, st, dim, a);
    if (n4 <= 32) return launch_restore_strided<32, BITS>(ctx, st, dim, a);
    return launch_restore_strided<64, BITS>(ctx, st, dim, a);
}

// ---------------------------------------------------------------------------------------------
// Error metric: || X - Q ||_2 per row in fp64, one wavefront per row, any dim; and its mean, added
// up by one workgroup in a fixed order so that the result does not depend on scheduling.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ void __launch_bounds__(kBlock)
quant_error_kernel(const float *__restrict__ table, uint64_t n_rows, uint32_t dim,
                   const uint32_t *__restrict__ row_ids, const uint64_t *__restrict__ n_dev, uint64_t n_max,
                   const uint8_t *__restrict__ packed, const float *__restrict__ scale,
                   const float *__restrict__ bias, double *__restrict__ err_out, cnr_dev_errors *err) {
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const int lane = tid_x() & (kWave - 1);
    const uint64_t n_waves = (uint64_t)grid_x() * kWavesPerBlock;
    const uint64_t P = (uint64_t)dim * BITS / 8;
    for (uint64_t k = (uint64_t)wg_x() * kWavesPerBlock + tid_x() / kWave; k < n; k += n_waves) {
        const uint64_t r = row_ids ? (uint64_t)row_ids[k] : k;
        if (r >= n_rows) {
            if (lane == 0) {
                raise_flag(err, CNR_FLAG_ROW_ID);
                err_out[k] = 0.0;
            }
            continue;
        }
        const uint8_t *__restrict__ in = packed + k * P;
        const float s = scale[k], b = bias[k];
        const float *__restrict__ x = table + r * (uint64_t)dim;
        double acc = 0.0;
        for (uint32_t e = lane; e < dim; e += kWave) {
            const uint64_t bit = (uint64_t)e * BITS;
            uint32_t two = in[bit >> 3];
            if (((bit & 7u) + BITS) > 8u) two |= (uint32_t)in[(bit >> 3) + 1] << 8;
            const float q = s * (float)((two >> (bit & 7u)) & MASK) + b;
            const double d = (double)x[e] - (double)q;
            acc += d * d;
        }
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        if (lane == 0) err_out[k] = sqrt(acc);
    }
}

__global__ void __launch_bounds__(kBlock)
mean_kernel(const double *__restrict__ v, const uint64_t *__restrict__ n_dev, uint64_t n_max,
            double *__restrict__ mean_out) {
    __shared__ double part[kBlock];
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    double acc = 0.0;
    for (uint64_t i = tid_x(); i < n; i += kBlock) acc += v[i];
    part[tid_x()] = acc;
    __syncthreads();
    for (int half = kBlock / 2; half > 0; half >>= 1) {
        if ((int)tid_x() < half) part[tid_x()] += part[tid_x() + half];
        __syncthreads();
    }
    if (tid_x() == 0) *mean_out = n ? part[0] / (double)n : 0.0;
}

}  // namespace

extern "C" cnr_status cnr_quant_error(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                                      const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                                      int bits, const uint8_t *packed, const float *scale,
                                      const float *bias, double *err, double *mean_out, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (((uintptr_t)err % 8) || ((uintptr_t)mean_out % 8) || ((uintptr_t)n_dev % 8) || ((uintptr_t)table % 4) ||
        ((uintptr_t)scale % 4) || ((uintptr_t)bias % 4) || ((uintptr_t)row_ids % 4))
        return CNR_E_ALIGN;
    hipStream_t s = as_stream(stream);
    if (n_max > 0) {
        if (!table || !packed || !scale || !bias || !err || n_rows == 0 || n_rows >= (1ull << 32)) return CNR_E_INVALID;
        const unsigned grid = cnr_grid(ctx, n_max, kWavesPerBlock, 8);
        switch (bits) {
            case 2: hipLaunchKernelGGL(quant_error_kernel<2>, dim3(grid), dim3(kBlock), 0, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias, err, ctx->dev_err); break;
            case 3: hipLaunchKernelGGL(quant_error_kernel<3>, dim3(grid), dim3(kBlock), 0, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias, err, ctx->dev_err); break;
            case 4: hipLaunchKernelGGL(quant_error_kernel<4>, dim3(grid), dim3(kBlock), 0, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias, err, ctx->dev_err); break;
            default: hipLaunchKernelGGL(quant_error_kernel<8>, dim3(grid), dim3(kBlock), 0, s, table, n_rows, dim, row_ids, n_dev, n_max, packed, scale, bias, err, ctx->dev_err); break;
        }
        st = cnr_launch_status(ctx);
        if (st != CNR_OK) return st;
    }
    if (mean_out) {
        hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kBlock), 0, s, err, n_dev, n_max, mean_out);
        st = cnr_launch_status(ctx);
    }
    return st;
}

extern "C" cnr_status cnr_restore_rows_batch(cnr_ctx *ctx, const cnr_table_job *jobs, uint32_t n_jobs,
                                             uint32_t dim, int bits, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (n_jobs && !jobs) return CNR_E_INVALID;
    for (uint32_t i = 0; i < n_jobs; ++i) {
        const cnr_table_job &j = jobs[i];
        if (j.capacity == 0) continue;
        if (!j.table || !j.packed || !j.scale || !j.bias || j.n_rows == 0 || j.n_rows >= (1ull << 32))
            return CNR_E_INVALID;
        if (((uintptr_t)j.table % 16) || ((uintptr_t)j.packed % 16) || ((uintptr_t)j.scale % 16) ||
            ((uintptr_t)j.bias % 16) || ((uintptr_t)j.row_ids % 16) || ((uintptr_t)j.n_dirty_dev % 8))
            return CNR_E_ALIGN;
    }
    hipStream_t s = as_stream(stream);
    const uint64_t prb = (uint64_t)dim * (uint64_t)bits / 8u;
    auto part = [&](const cnr_table_job &j, uint64_t k0, uint64_t m) {  // rows k0 .. k0 + m - 1 of j's list
        RestoreJob a = {};
        if (j.row_ids) {
            a.table = j.table; a.n_rows = j.n_rows; a.row_ids = j.row_ids + k0;
        } else {
            a.table = j.table + k0 * dim; a.n_rows = j.n_rows - k0; a.row_ids = nullptr;
        }
        a.n_dev = j.n_dirty_dev; a.n_max = m;
        a.packed = j.packed + k0 * prb; a.scale = j.scale + k0; a.bias = j.bias + k0;
        return a;
    };
    // launches of up to CNR_MAX_BATCH small tables, then of large ones and slices, as for the encode
    const bool tile_dim = dim == 16 || dim == 32 || dim == 64 || dim == 128 || dim == 256;
    if (tile_dim) {
        for (int large = 0; large < 2; ++large) {
            RestoreBatch b = {};
            uint32_t n = 0;
            auto flush = [&]() -> cnr_status {
                if (n == 0) return CNR_OK;
                switch (bits) {
                    case 2: launch_restore16_bits<2>(ctx, s, dim, b, n); break;
                    case 3: launch_restore16_bits<3>(ctx, s, dim, b, n); break;
                    case 4: launch_restore16_bits<4>(ctx, s, dim, b, n); break;
                    default: launch_restore16_bits<8>(ctx, s, dim, b, n); break;
                }
                n = 0;
                return cnr_launch_status(ctx);
            };
            for (uint32_t i = 0; i < n_jobs; ++i) {
                const cnr_table_job &j = jobs[i];
                if (j.capacity == 0 || (j.capacity * 4ull * dim > kSideBySideBytes) != (large != 0)) continue;
                const bool sliceable = !j.n_dirty_dev && (j.row_ids || j.capacity <= j.n_rows);
                const uint64_t step = sliceable ? cnr_slice_rows(j.capacity, dim) : j.capacity;
                for (uint64_t k0 = 0; k0 < j.capacity; k0 += step) {
                    b.job[n++] = part(j, k0, j.capacity - k0 < step ? j.capacity - k0 : step);
                    if (n == CNR_MAX_BATCH && (st = flush()) != CNR_OK) return st;
                }
            }
            if ((st = flush()) != CNR_OK) return st;
        }
        return CNR_OK;
    }
    for (uint32_t i = 0; i < n_jobs; ++i) {  // other row lengths: one launch per table
        const cnr_table_job &j = jobs[i];
        if (j.capacity == 0) continue;
        RestoreJob a = part(j, 0, j.capacity);
        switch (bits) {
            case 2: launch_restore<2>(ctx, s, dim, a); break;
            case 3: launch_restore<3>(ctx, s, dim, a); break;
            case 4: launch_restore<4>(ctx, s, dim, a); break;
            default: launch_restore<8>(ctx, s, dim, a); break;
        }
        if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
    }
    return CNR_OK;
}

extern "C" cnr_status cnr_restore_rows(cnr_ctx *ctx, float *table, uint64_t n_rows, uint32_t dim,
                                       const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                                       int bits, const uint8_t *packed, const float *scale,
                                       const float *bias, void *stream) {
    cnr_table_job j = {};
    j.table = table;
    j.n_rows = n_rows;
    j.row_ids = const_cast<uint32_t *>(row_ids);
    j.n_dirty_dev = const_cast<uint64_t *>(n_dev);
    j.capacity = n_max;
    j.packed = const_cast<uint8_t *>(packed);
    j.scale = const_cast<float *>(scale);
    j.bias = const_cast<float *>(bias);
    return cnr_restore_rows_batch(ctx, &j, 1, dim, bits, stream);
}
