// Gather + per-row uniform quantization F_Q + dense packing (Section 5.2, Approaches 1 and 3).
//
// Arithmetic contract (what makes the output comparable with a plain CPU statement of the
// formulas): fp32 throughout, one rounding per operation (the build disables contraction into fused
// multiply-adds), round-half-even, fp32 denormals kept; row minimum, maximum, scale and bias are
// bit-exact; codes may differ from the divide-and-round definition by one step where the quotient
// lies within rounding distance of a half-integer (see the bulk kernel).  Error sums that only rank
// candidate ranges are accumulated in fp64.
#include <type_traits>

#include "cnr_common.h"

namespace {

enum { kModeMinMax = CNR_RANGE_MINMAX, kModeGreedy = CNR_RANGE_GREEDY, kModeSymmetric = CNR_RANGE_SYMMETRIC };

// Arguments shared by the quantize kernels.
struct QuantArgs {
    const float *table;
    uint64_t n_rows;
    uint32_t dim;
    const uint32_t *row_ids;
    const uint64_t *n_dev;
    uint64_t n_max;
    int mode;
    uint32_t n_iter;   // greedy iterations
    float num_bins_f;  // greedy num_bins
    float *scale, *bias, *row_min, *row_max;
    uint8_t *codes, *packed;
    cnr_dev_errors *err;
};

// The tables of one launch.  A persistent kernel works through them in order: a workgroup that has
// run out of rows in one table goes on to the next at once, so the GPU is not drained and refilled
// between tables.
struct QuantBatch {
    QuantArgs job[CNR_MAX_BATCH];
    uint32_t n_jobs;
    uint32_t n_waves;  // waves of the grid
};

__device__ __forceinline__ uint64_t row_count(const QuantArgs &a) { return live_rows(a.n_dev, a.n_max); }

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

template <int U>
__device__ __forceinline__ float quad_bcast(float v) {  // value of quad lane U in all four lanes
    return dpp_f<U * 0x55>(v);
}

// ---------------------------------------------------------------------------------------------
// Bulk kernel (min/max and symmetric range), dim = 64 * M.  Bound by HBM.
//
// Sixteen lanes share a row: lane l of the group holds, for every 64-element chunk c of the row,
// the four consecutive elements 64c + 4l .. 64c + 4l + 3, so one 16-byte load per lane reads 256
// contiguous bytes per group, and all reductions over a row stay inside one 16-lane DPP row.  Each
// group works on four consecutive dirty rows at once (a wave has sixteen rows = 4 KB * M in flight),
// which is also what lets the packed codes leave through full words: after quantizing, a 4x4
// transpose inside each quad of lanes hands lane j the codes of sixteen consecutive elements of row
// j.  The loop is software-pipelined: the rows of batch i+1 and the ids of batch i+2 are requested
// before batch i is reduced and quantized.
//
// A wave64 instruction occupies a SIMD for four cycles, so vector-ALU issue competes with HBM here,
// and the per-element work is pared down:
//   - scale and 1/scale are computed once per row, by the one lane of each quad that owns the row,
//     with correctly rounded divisions, and broadcast back inside the quad;
//   - an element's code is round((x - lo) * (1/scale)); adding 1.5 * 2^23 does the rounding
//     (half-to-even) and leaves the integer in the low mantissa bits, so four codes are merged by
//     three shift-adds and one subtraction of the merged constant.  The product differs from the
//     correctly rounded quotient by at most 1.5 ulp, which can move a code only when the quotient
//     sits within that distance of a half-integer (a few elements in a million at 4 bits); at 8
//     bits, where quotients are larger, one FMA residual step on the quotient removes that too;
//   - the reciprocal must be a normal number: rows with a scale outside [2^-100, 2^100] (denormal
//     or near-overflow ranges) are brought there by an exact power-of-two factor applied to both
//     x - lo and the scale, and a wave takes that variant only if one of its sixteen rows needs it.
// A layout with sixteen contiguous elements per lane (the greedy kernel's) needs half the
// instructions but its strided 16-byte loads cost more than they save: 92 us against 81 us per
// 5 M x 64 table with 30 % dirty rows.
// ---------------------------------------------------------------------------------------------
#define CNR_SEL4(a) (j == 0 ? (a)[0] : j == 1 ? (a)[1] : j == 2 ? (a)[2] : (a)[3])

template <int M>
struct RowBatch {
    float4 x[4][M];  // [row of the group][chunk]
    unsigned skip;   // bit u: row k0+u is past the end or has an id outside the table
};

// Row ids of the four rows k0 .. k0+3 of one group.
__device__ __forceinline__ uint4 gather_ids(const QuantArgs &a, uint64_t k0) {
    if (!a.row_ids) return make_uint4((uint32_t)k0, (uint32_t)k0 + 1, (uint32_t)k0 + 2, (uint32_t)k0 + 3);
    if (k0 + 3 < a.n_max)  // the id buffer holds n_max entries: one 16-byte load
        return *reinterpret_cast<const uint4 *>(a.row_ids + k0);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k0 + 0 < a.n_max) v.x = a.row_ids[k0 + 0];
    if (k0 + 1 < a.n_max) v.y = a.row_ids[k0 + 1];
    if (k0 + 2 < a.n_max) v.z = a.row_ids[k0 + 2];
    return v;
}

// Issues the loads of the group's four rows (this lane's elements 64c + 4l .. + 3 of each).
template <int M>
__device__ __forceinline__ void gather_rows(const QuantArgs &a, uint64_t n, uint64_t k0, uint4 ids, int l,
                                            RowBatch<M> &rb) {
    const uint32_t rid[4] = {ids.x, ids.y, ids.z, ids.w};
    rb.skip = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const bool past = k0 + u >= n;
        uint64_t r = rid[u];
        if (past || r >= a.n_rows) {
            if (!past && l == 0) raise_flag(a.err, CNR_FLAG_ROW_ID);
            rb.skip |= 1u << u;
            r = 0;
        }
        const float *src = a.table + r * (uint64_t)(64 * M) + 4u * (uint64_t)l;
#pragma unroll
        for (int c = 0; c < M; ++c) {
            const f32x4 v = load_stream<f32x4>(src + 64 * c);
            rb.x[u][c] = make_float4(v.x, v.y, v.z, v.w);
        }
    }
}

// Reduces, quantizes and stores the four rows of one group.
template <int M, int BITS>
__device__ __forceinline__ void encode_batch(const QuantArgs &a, uint64_t k0, const RowBatch<M> &rb, int l) {
    constexpr int DIM = 64 * M;
    constexpr float QMAXF = (float)((1 << BITS) - 1);
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;  // packed bytes per row
    constexpr float MAGIC = 12582912.0f;              // 1.5 * 2^23: x + MAGIC rounds x to an integer
    constexpr uint32_t MAGIC_BITS = 0x4B400000u;      // bit pattern of MAGIC
    // what four magic-biased codes add up to when merged with shifts of B, 2B, 3B bits
    constexpr uint32_t MERGED_BIAS = MAGIC_BITS * (1u + (1u << BITS) + (1u << (2 * BITS)) + (1u << (3 * BITS)));
    constexpr uint32_t MERGED_BIAS8 = MAGIC_BITS * (1u + (1u << 8) + (1u << 16) + (1u << 24));
    const int q = l >> 2;  // quad in group
    const int j = l & 3;   // lane in quad
    const unsigned skip = rb.skip;
    const float4 (&x)[4][M] = rb.x;

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
        if (a.mode == kModeSymmetric) {
            const float m = fmaxf(fabsf(X_min[u]), fabsf(X_max[u]));
            lo[u] = -m + 0.0f;
            hi[u] = m;
        }
    }

    // ---- per-row parameters, computed by the quad lane that owns the row (lane j <-> row k0+j)
    const float my_lo = CNR_SEL4(lo);
    const float my_scale = (CNR_SEL4(hi) - my_lo) / QMAXF;
    const bool my_live = !((skip >> j) & 1u);
    {   // lanes 0-3 of a group write scale, 4-7 bias, 8-11 min, 12-15 max
        float *dst = q == 0 ? a.scale : q == 1 ? a.bias : q == 2 ? a.row_min : a.row_max;
        const float v = q == 0 ? my_scale : q == 1 ? my_lo : q == 2 ? CNR_SEL4(X_min) : CNR_SEL4(X_max);
        if (dst && my_live) store_stream<float>(dst + k0 + j, v);
    }
    const float my_f = my_scale < 0x1p-100f ? 0x1p120f : my_scale > 0x1p100f ? 0x1p-120f : 1.0f;
    const float my_fscale = my_scale * my_f;
    const float my_inv = my_scale == 0.0f ? 0.0f : 1.0f / my_fscale;  // scale 0: every code 0
    const float inv[4] = {quad_bcast<0>(my_inv), quad_bcast<1>(my_inv), quad_bcast<2>(my_inv),
                          quad_bcast<3>(my_inv)};

    // ---- quantize; h[c][u] = this lane's four codes of (row u, chunk c)
    uint32_t h[M][4];
    auto quantize_by_reciprocal = [&](auto rescale) {
        constexpr bool RESCALE = decltype(rescale)::value;
        float f[4] = {1.0f, 1.0f, 1.0f, 1.0f}, fsc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (RESCALE) {
            f[0] = quad_bcast<0>(my_f); f[1] = quad_bcast<1>(my_f);
            f[2] = quad_bcast<2>(my_f); f[3] = quad_bcast<3>(my_f);
        }
        if constexpr (BITS == 8) {
            fsc[0] = quad_bcast<0>(my_fscale); fsc[1] = quad_bcast<1>(my_fscale);
            fsc[2] = quad_bcast<2>(my_fscale); fsc[3] = quad_bcast<3>(my_fscale);
        }
        // magic-biased code of one element: MAGIC_BITS + round((x - lo) / scale)
        auto biased = [&](float xv, int u) -> uint32_t {
            float d0 = xv - lo[u];
            if constexpr (RESCALE) d0 *= f[u];
            float t = d0 * inv[u];
            if constexpr (BITS == 8) t = fmaf(fmaf(-t, fsc[u], d0), inv[u], t);
            return __float_as_uint(t + MAGIC);
        };
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < M; ++c) {
                const uint32_t b0 = biased(x[u][c].x, u), b1 = biased(x[u][c].y, u);
                const uint32_t b2 = biased(x[u][c].z, u), b3 = biased(x[u][c].w, u);
                uint32_t m = (b3 << BITS) + b2;
                m = (m << BITS) + b1;
                h[c][u] = (m << BITS) + b0 - MERGED_BIAS;
                if (a.codes && !(skip & (1u << u)))
                    *reinterpret_cast<uint32_t *>(a.codes + (k0 + u) * (uint64_t)DIM + 64 * c + 4 * l) =
                        (((((b3 << 8) + b2) << 8) + b1) << 8) + b0 - MERGED_BIAS8;
            }
    };
    if (__builtin_amdgcn_ballot_w64(my_f != 1.0f) != 0)
        quantize_by_reciprocal(std::true_type{});
    else
        quantize_by_reciprocal(std::false_type{});

    // ---- packed codes: after the quad transpose lane j owns 16 consecutive elements
    // (64c + 16q ..) of row k0 + j
    if (a.packed) {
        uint8_t *row = a.packed + (k0 + (uint64_t)j) * P;
#pragma unroll
        for (int c = 0; c < M; ++c) {
            uint32_t t[4] = {h[c][0], h[c][1], h[c][2], h[c][3]};
            quad_transpose(t, j);
            if constexpr (BITS == 8) {
                if (my_live) store_stream<u32x4>(row + 64 * c + 16 * q, u32x4{t[0], t[1], t[2], t[3]});
            } else if constexpr (BITS == 4) {
                if (my_live)
                    store_stream<u32x2>(row + 32 * c + 8 * q, u32x2{t[0] | (t[1] << 16), t[2] | (t[3] << 16)});
            } else if constexpr (BITS == 2) {
                if (my_live)
                    store_stream<uint32_t>(row + 16 * c + 4 * q, t[0] | (t[1] << 8) | (t[2] << 16) | (t[3] << 24));
            } else {  // 3 bits: 48 bits per lane; even quads append the next quad's 48 bits
                const uint32_t w0 = t[0] | (t[1] << 12) | (t[2] << 24);  // stream bits 0..31
                const uint32_t w1 = (t[2] >> 8) | (t[3] << 4);           // stream bits 32..47
                const uint32_t n0 = (uint32_t)dpp_i<0x104>((int)w0);     // row_shl:4 = lane + 4
                const uint32_t n1 = (uint32_t)dpp_i<0x104>((int)w1);
                if (my_live && !(q & 1)) {
                    uint32_t *dst = reinterpret_cast<uint32_t *>(row + 24 * c + 12 * (q >> 1));
                    store_stream<uint32_t>(dst, w0);
                    store_stream<uint32_t>(dst + 1, w1 | (n0 << 16));
                    store_stream<uint32_t>(dst + 2, (n0 >> 16) | (n1 << 16));
                }
            }
        }
    }
}
#undef CNR_SEL4

template <int M, int BITS>
__device__ __forceinline__ void encode_table(const QuantArgs &a, uint32_t n_waves, uint32_t &carry) {
    const uint64_t n = row_count(a);
    const int lane = tid_x() & (kWave - 1);
    const uint64_t g4 = 4u * (uint64_t)(lane >> 4);  // first row of this lane's group within a batch
    const int l = lane & 15;                         // lane in group
    uint64_t batch = first_unit(wave_in_grid(), n_waves, (uint32_t)((n + 15u) / 16u), carry);
    if (batch * 16u >= n) return;

    RowBatch<M> cur, nxt;
    gather_rows<M>(a, n, batch * 16u + g4, gather_ids(a, batch * 16u + g4), l, cur);
    uint64_t next = batch + n_waves;
    uint4 ids_next = make_uint4(0, 0, 0, 0);
    if (next * 16u < n) ids_next = gather_ids(a, next * 16u + g4);
    for (;;) {
        const bool has_next = next * 16u < n;  // uniform over the wave
        if (has_next) gather_rows<M>(a, n, next * 16u + g4, ids_next, l, nxt);
        const uint64_t next2 = next + n_waves;
        if (next2 * 16u < n) ids_next = gather_ids(a, next2 * 16u + g4);
        encode_batch<M, BITS>(a, batch * 16u + g4, cur, l);
        if (!has_next) break;
        cur = nxt;
        batch = next;
        next = next2;
    }
}

template <int M, int BITS>
__global__ void __launch_bounds__(kBlock) quantize_rows16_kernel(const QuantBatch b) {
    uint32_t carry = 0;
    for (uint32_t t = 0; t < b.n_jobs; ++t) encode_table<M, BITS>(b.job[t], b.n_waves, carry);
}

// ---------------------------------------------------------------------------------------------
// Greedy range search (Approach 3), dim = 16 * L with L = 4, 8 or 16 lanes per row.  Bound by
// vector-ALU issue: 1 + 2 * n_iter candidate ranges are tried per row.
//
// Every lane owns sixteen consecutive elements (four 16-byte loads) of one row, L neighbouring lanes
// own the row, a wave handles 64 / L consecutive dirty rows per pass.  A candidate's error is summed
// over a lane's sixteen registers and then over the L lanes with log2(L) DPP exchanges, a quarter of
// the cross-lane work the bulk kernel's layout would need, and a lane's sixteen codes are exactly
// 2 * BITS contiguous bytes of the packed row, so the output needs no transpose.
// A candidate is evaluated with the cheapest sequence that still reproduces F_Q's codes: the scale
// (range / (2^b - 1)) and the quotient (x - lo) / scale are formed by a reciprocal multiply followed
// by one FMA residual correction (q' = q + (a - q*b) * (1/b)), which yields the correctly rounded
// quotient except in cases far too rare to matter for ranking candidates; d*d is exact in fp64, so
// fma(d, d, acc) is the multiply-then-add of the definition.  A wave holding a row whose scale lies
// outside [2^-100, 2^100] divides instead.  The final codes of the chosen range are produced by
// division, exactly as F_Q is written.
// ---------------------------------------------------------------------------------------------
template <int L>
__device__ __forceinline__ float lanes_min(float v) {
    v = fminf(v, dpp_f<0xB1>(v));
    v = fminf(v, dpp_f<0x4E>(v));
    if constexpr (L >= 8) v = fminf(v, dpp_f<0x141>(v));
    if constexpr (L >= 16) v = fminf(v, dpp_f<0x140>(v));
    return v;
}
template <int L>
__device__ __forceinline__ float lanes_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    if constexpr (L >= 8) v = fmaxf(v, dpp_f<0x141>(v));
    if constexpr (L >= 16) v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
template <int L>
__device__ __forceinline__ double lanes_sum(double v) {
    v += dpp_d<0xB1>(v);
    v += dpp_d<0x4E>(v);
    if constexpr (L >= 8) v += dpp_d<0x141>(v);
    if constexpr (L >= 16) v += dpp_d<0x140>(v);
    return v;
}

template <int L, int BITS>
__device__ __forceinline__ void greedy_table(const QuantArgs &a, uint32_t n_waves, uint32_t &carry) {
    constexpr int DIM = 16 * L;
    constexpr int kRowsPerPass = kWave / L;
    constexpr float QMAXF = (float)((1 << BITS) - 1);
    constexpr float INV_QMAX = 1.0f / QMAXF;
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;  // packed bytes per row
    const uint64_t n = row_count(a);
    const int lane = tid_x() & (kWave - 1);
    const int j = lane % L;  // lane within the row
    for (uint64_t pass = first_unit(wave_in_grid(), n_waves, (uint32_t)((n + kRowsPerPass - 1) / kRowsPerPass), carry);
         pass * kRowsPerPass < n; pass += n_waves) {
        const uint64_t k = pass * kRowsPerPass + lane / L;
        // ---- gather
        uint64_t rid = 0;
        bool live = k < n;
        if (live) {
            rid = a.row_ids ? (uint64_t)a.row_ids[k] : k;
            if (rid >= a.n_rows) {
                if (j == 0) raise_flag(a.err, CNR_FLAG_ROW_ID);
                live = false;
                rid = 0;
            }
        }
        float4 x[4];
        {
            const float *src = a.table + rid * (uint64_t)DIM + 16u * (uint64_t)j;
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = *reinterpret_cast<const float4 *>(src + 4 * i);
        }

        // ---- row minimum / maximum
        float mn = fminf(fminf(x[0].x, x[0].y), fminf(x[0].z, x[0].w));
        float mx = fmaxf(fmaxf(x[0].x, x[0].y), fmaxf(x[0].z, x[0].w));
#pragma unroll
        for (int i = 1; i < 4; ++i) {
            mn = fminf(fminf(mn, x[i].x), fminf(x[i].y, fminf(x[i].z, x[i].w)));
            mx = fmaxf(fmaxf(mx, x[i].x), fmaxf(x[i].y, fmaxf(x[i].z, x[i].w)));
        }
        const float X_min = lanes_min<L>(mn) + 0.0f;  // -0.0 -> +0.0
        const float X_max = lanes_max<L>(mx) + 0.0f;
        float lo = X_min, hi = X_max;

        // ---- the search: shrink from whichever side hurts less, remember the best range seen
        auto search = [&](auto fast_tag) {
            constexpr bool FAST = decltype(fast_tag)::value;
            auto add_err = [&](double acc, float xv, float c_lo, float c_hi, float s, float inv) -> double {
                if constexpr (FAST) {
                    const float c = __builtin_amdgcn_fmed3f(xv, c_lo, c_hi);
                    const float d0 = c - c_lo;
                    float t = d0 * inv;
                    t = fmaf(fmaf(-t, s, d0), inv, t);
                    const float d = xv - fq_value(rintf(t), s, c_lo);
                    return fma((double)d, (double)d, acc);
                } else {
                    return acc + fq_sq_err(xv, c_lo, c_hi, s, QMAXF);
                }
            };
            auto row_err = [&](float c_lo, float c_hi) -> double {
                const float range = c_hi - c_lo;
                float s, inv = 0.0f;
                if constexpr (FAST) {
                    const float q0 = range * INV_QMAX;
                    s = fmaf(fmaf(-q0, QMAXF, range), INV_QMAX, q0);
                    const float r0 = __builtin_amdgcn_rcpf(s);
                    inv = s == 0.0f ? 0.0f : fmaf(fmaf(-s, r0, 1.0f), r0, r0);
                } else {
                    s = range / QMAXF;
                }
                double e = 0.0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    e = add_err(e, x[i].x, c_lo, c_hi, s, inv);
                    e = add_err(e, x[i].y, c_lo, c_hi, s, inv);
                    e = add_err(e, x[i].z, c_lo, c_hi, s, inv);
                    e = add_err(e, x[i].w, c_lo, c_hi, s, inv);
                }
                return lanes_sum<L>(e);
            };
            float cur_lo = lo, cur_hi = hi;
            const float step = (hi - lo) / a.num_bins_f;
            double best = row_err(lo, hi);
            for (uint32_t it = 0; it < a.n_iter; ++it) {
                const float c_lo = cur_lo + step;
                const float c_hi = cur_hi - step;
                const double e_lo = row_err(c_lo, cur_hi);
                const double e_hi = row_err(cur_lo, c_hi);
                const bool move_lo = e_lo < e_hi;
                cur_lo = move_lo ? c_lo : cur_lo;
                cur_hi = move_lo ? cur_hi : c_hi;
                const double e = move_lo ? e_lo : e_hi;
                if (e < best) {
                    best = e;
                    lo = cur_lo;
                    hi = cur_hi;
                }
            }
        };
        const float s0 = (hi - lo) * INV_QMAX;
        const bool odd_scale = s0 != 0.0f && !(s0 >= 0x1p-100f && s0 <= 0x1p100f);
        // the last candidates are up to num_bins times narrower than the first
        if (__builtin_amdgcn_ballot_w64(odd_scale) != 0 || a.num_bins_f > 0x1p20f)
            search(std::false_type{});
        else
            search(std::true_type{});

        // ---- per-row parameters: lane 0 of the row writes scale, lane 1 bias, lanes 2, 3 min, max
        const float scale = (hi - lo) / QMAXF;
        {
            float *dst = j == 0 ? a.scale : j == 1 ? a.bias : j == 2 ? a.row_min : a.row_max;
            const float v = j == 0 ? scale : j == 1 ? lo : j == 2 ? X_min : X_max;
            if (j < 4 && dst && live) dst[k] = v;
        }

        // ---- final codes by F_Q as written; h[i] = the four codes of x[i], first element lowest
        uint32_t h[4], h8[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t q0 = (uint32_t)fq_code_f(x[i].x, lo, hi, scale, QMAXF);
            const uint32_t q1 = (uint32_t)fq_code_f(x[i].y, lo, hi, scale, QMAXF);
            const uint32_t q2 = (uint32_t)fq_code_f(x[i].z, lo, hi, scale, QMAXF);
            const uint32_t q3 = (uint32_t)fq_code_f(x[i].w, lo, hi, scale, QMAXF);
            h[i] = q0 | (q1 << BITS) | (q2 << (2 * BITS)) | (q3 << (3 * BITS));
            h8[i] = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
        }
        if (a.codes && live)
            *reinterpret_cast<uint4 *>(a.codes + k * (uint64_t)DIM + 16 * j) = make_uint4(h8[0], h8[1], h8[2], h8[3]);

        // ---- packed codes: this lane's bits are bytes [2 * BITS * j, 2 * BITS * (j + 1)) of the row
        if (a.packed) {
            uint8_t *dst = a.packed + k * P + 2 * BITS * j;
            if constexpr (BITS == 8) {
                if (live) *reinterpret_cast<uint4 *>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
            } else if constexpr (BITS == 4) {
                if (live) *reinterpret_cast<uint2 *>(dst) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            } else if constexpr (BITS == 2) {
                if (live) *reinterpret_cast<uint32_t *>(dst) = h[0] | (h[1] << 8) | (h[2] << 16) | (h[3] << 24);
            } else {  // 3 bits: 48 bits per lane; even lanes append their right neighbour's 48 bits
                const uint32_t w0 = h[0] | (h[1] << 12) | (h[2] << 24);  // stream bits 0..31
                const uint32_t w1 = (h[2] >> 8) | (h[3] << 4);           // stream bits 32..47
                const uint32_t n0 = (uint32_t)dpp_i<0xB1>((int)w0);      // lane ^ 1
                const uint32_t n1 = (uint32_t)dpp_i<0xB1>((int)w1);
                if (live && !(j & 1)) {
                    uint32_t *d3 = reinterpret_cast<uint32_t *>(dst);
                    d3[0] = w0;
                    d3[1] = w1 | (n0 << 16);
                    d3[2] = (n0 >> 16) | (n1 << 16);
                }
            }
        }
    }
}

template <int L, int BITS>
__global__ void __launch_bounds__(kBlock) quantize_greedy_kernel(const QuantBatch b) {
    uint32_t carry = 0;
    for (uint32_t t = 0; t < b.n_jobs; ++t) greedy_table<L, BITS>(b.job[t], b.n_waves, carry);
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
    const int lane = tid_x() & (kWave - 1);
    const uint64_t n_waves = (uint64_t)grid_x() * kWavesPerBlock;
    const uint64_t P = (uint64_t)dim * BITS / 8;
    for (uint64_t k = (uint64_t)wg_x() * kWavesPerBlock + tid_x() / kWave; k < n; k += n_waves) {
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
    const uint64_t stride = (uint64_t)grid_x() * kBlock;
    for (uint64_t o = (uint64_t)wg_x() * kBlock + tid_x(); o < total; o += stride) {
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

uint64_t most_rows(const QuantBatch &b) {
    uint64_t m = 0;
    for (uint32_t t = 0; t < b.n_jobs; ++t)
        if (b.job[t].n_max > m) m = b.job[t].n_max;
    return m;
}

template <int M, int BITS>
void launch_rows16(cnr_ctx *ctx, QuantBatch &b, hipStream_t s) {
    const unsigned grid = cnr_grid(ctx, most_rows(b), 16u * kWavesPerBlock,
                                   cnr_resident_blocks_per_cu<quantize_rows16_kernel<M, BITS>>());
    b.n_waves = grid * kWavesPerBlock;
    hipLaunchKernelGGL((quantize_rows16_kernel<M, BITS>), dim3(grid), dim3(kBlock), 0, s, b);
}

template <int L, int BITS>
void launch_greedy(cnr_ctx *ctx, QuantBatch &b, hipStream_t s) {
    const unsigned grid = cnr_grid(ctx, most_rows(b), (uint64_t)(kWave / L) * kWavesPerBlock,
                                   cnr_resident_blocks_per_cu<quantize_greedy_kernel<L, BITS>>());
    b.n_waves = grid * kWavesPerBlock;
    hipLaunchKernelGGL((quantize_greedy_kernel<L, BITS>), dim3(grid), dim3(kBlock), 0, s, b);
}

template <int BITS>
void launch_bits(cnr_ctx *ctx, QuantBatch &b, hipStream_t s) {
    const QuantArgs &c = b.job[0];                              // dim, mode, n_iter are common to the batch
    const bool greedy = c.mode == kModeGreedy && c.n_iter > 0;  // zero iterations: plain min/max
    if (c.dim == 64) return greedy ? launch_greedy<4, BITS>(ctx, b, s) : launch_rows16<1, BITS>(ctx, b, s);
    if (c.dim == 128) return greedy ? launch_greedy<8, BITS>(ctx, b, s) : launch_rows16<2, BITS>(ctx, b, s);
    if (c.dim == 256) return greedy ? launch_greedy<16, BITS>(ctx, b, s) : launch_rows16<4, BITS>(ctx, b, s);
    for (uint32_t t = 0; t < b.n_jobs; ++t) {  // other row lengths: one launch per table
        const QuantArgs &a = b.job[t];
        const unsigned grid = cnr_grid(ctx, a.n_max, kWavesPerBlock, 8);
        hipLaunchKernelGGL((quantize_rows_generic_kernel<BITS>), dim3(grid), dim3(kBlock), 0, s, a.table,
                           a.n_rows, a.dim, a.row_ids, a.n_dev, a.n_max, a.mode, a.n_iter, a.num_bins_f,
                           a.scale, a.bias, a.row_min, a.row_max, a.codes, a.packed, a.err);
    }
}

}  // namespace

extern "C" {

cnr_status cnr_quantize_rows_batch(cnr_ctx *ctx, const cnr_table_job *jobs, uint32_t n_jobs, uint32_t dim,
                                   int bits, cnr_range_mode mode, const cnr_greedy_params *greedy,
                                   void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!cnr_valid_bits(bits)) return CNR_E_BITS;
    if (dim == 0 || dim % 4 || dim > CNR_MAX_DIM || ((uint64_t)dim * (uint64_t)bits) % 8) return CNR_E_DIM;
    if (mode != CNR_RANGE_MINMAX && mode != CNR_RANGE_GREEDY && mode != CNR_RANGE_SYMMETRIC) return CNR_E_INVALID;
    if (mode == CNR_RANGE_GREEDY && !greedy) return CNR_E_INVALID;
    if (n_jobs && !jobs) return CNR_E_INVALID;
    for (uint32_t i = 0; i < n_jobs; ++i) {
        const cnr_table_job &j = jobs[i];
        if (j.capacity == 0) continue;
        if (!j.table || !j.scale || !j.bias || j.n_rows == 0 || j.n_rows >= (1ull << 32)) return CNR_E_INVALID;
        if (((uintptr_t)j.table % 16) || ((uintptr_t)j.packed % 16) || ((uintptr_t)j.codes_u8 % 4) ||
            ((uintptr_t)j.scale % 4) || ((uintptr_t)j.bias % 4) || ((uintptr_t)j.row_min % 4) ||
            ((uintptr_t)j.row_max % 4) || ((uintptr_t)j.row_ids % 16) || ((uintptr_t)j.n_dirty_dev % 8))
            return CNR_E_ALIGN;
    }
    hipStream_t s = as_stream(stream);
    for (uint32_t first = 0; first < n_jobs; first += CNR_MAX_BATCH) {
        QuantBatch b = {};
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i) {
            const cnr_table_job &j = jobs[i];
            if (j.capacity == 0) continue;
            QuantArgs &a = b.job[b.n_jobs++];
            a.table = j.table; a.n_rows = j.n_rows; a.dim = dim; a.row_ids = j.row_ids;
            a.n_dev = j.n_dirty_dev; a.n_max = j.capacity;
            a.mode = (int)mode;
            a.n_iter = mode == CNR_RANGE_GREEDY ? cnr_greedy_iterations(greedy->num_bins, greedy->ratio) : 0;
            a.num_bins_f = mode == CNR_RANGE_GREEDY ? (float)greedy->num_bins : 1.0f;
            a.scale = j.scale; a.bias = j.bias; a.row_min = j.row_min; a.row_max = j.row_max;
            a.codes = j.codes_u8; a.packed = j.packed; a.err = ctx->dev_err;
        }
        if (b.n_jobs == 0) continue;
        switch (bits) {
            case 2: launch_bits<2>(ctx, b, s); break;
            case 3: launch_bits<3>(ctx, b, s); break;
            case 4: launch_bits<4>(ctx, b, s); break;
            default: launch_bits<8>(ctx, b, s); break;
        }
        if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
    }
    return CNR_OK;
}

cnr_status cnr_quantize_rows(cnr_ctx *ctx, const float *table, uint64_t n_rows, uint32_t dim,
                             const uint32_t *row_ids, const uint64_t *n_dev, uint64_t n_max,
                             int bits, cnr_range_mode mode, const cnr_greedy_params *greedy,
                             float *scale, float *bias, float *row_min, float *row_max,
                             uint8_t *codes_u8, uint8_t *packed, void *stream) {
    cnr_table_job j = {};
    j.table = const_cast<float *>(table);
    j.n_rows = n_rows;
    j.row_ids = const_cast<uint32_t *>(row_ids);
    j.n_dirty_dev = const_cast<uint64_t *>(n_dev);
    j.capacity = n_max;
    j.scale = scale; j.bias = bias; j.row_min = row_min; j.row_max = row_max;
    j.codes_u8 = codes_u8; j.packed = packed;
    return cnr_quantize_rows_batch(ctx, &j, 1, dim, bits, mode, greedy, stream);
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
