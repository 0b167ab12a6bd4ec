// Gather + per-row uniform quantization F_Q + dense packing (Section 5.2, Approaches 1 and 3).
//
// Arithmetic contract (what makes the output comparable with a plain CPU statement of the
// formulas): fp32 throughout, one rounding per operation (the build disables contraction into fused
// multiply-adds), round-half-even, fp32 denormals kept; row minimum, maximum, scale and bias are
// bit-exact; codes may differ from the divide-and-round definition by one step where the quotient
// lies within rounding distance of a half-integer (see the tile kernel).  Error sums that only rank
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
    uint32_t n_waves;  // waves of the grid = the stride of a wave through the list, in passes
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

// ---------------------------------------------------------------------------------------------
// Tile kernel (min/max and symmetric range), dim = 64 * M.  Bound by HBM.
//
// A wave works on sixteen consecutive dirty rows per pass, in two lane layouts with a transpose
// through LDS between them:
//   load layout     sixteen lanes share a row: lane l of group g holds elements 64c + 4l .. + 3 of
//                   rows 4g .. 4g + 3 of the pass, so every 16-byte load instruction reads 256
//                   contiguous bytes per row;
//   compute layout  four lanes share a row: lane j of row rho holds the sixteen consecutive elements
//                   64c + 16j .. + 15 of every 64-element chunk c.  The row minimum and maximum then
//                   need only two cross-lane steps, the row's parameters are computed where they are
//                   used, and a lane's sixteen codes are 2 * BITS contiguous bytes of the packed row,
//                   so a wave's packed output is one contiguous run.
// The transpose is private to the wave (LDS operations of one wave complete in order, so no
// barrier is needed); a row's four quarters sit 80 bytes apart and rows 320 bytes apart, which
// spreads the lanes that the LDS serves together over its banks in both directions (what conflicts
// remain cost a few LDS cycles per instruction, far from limiting).
//
// The kernel has to stay clear of the vector-ALU issue limit (a wave64 instruction occupies a SIMD
// for four cycles) to run at the speed of its memory traffic, so the per-element work is pared down:
//   - an element's code is round((x - lo) * (1/scale)); adding 1.5 * 2^23 does the rounding
//     (half-to-even) and leaves the integer in the low mantissa bits, so four codes are merged by
//     three shift-adds and one subtraction of the merged constant.  The product differs from the
//     correctly rounded quotient by at most 1.5 ulp, which can move a code only when the quotient
//     sits within that distance of a half-integer (a few elements in a million at 4 bits); at 8
//     bits, where quotients are larger, one FMA residual step on the quotient removes that too;
//   - the reciprocal must be a normal number: rows with a scale outside [2^-100, 2^100] (denormal
//     or near-overflow ranges) are brought there by an exact power-of-two factor applied to both
//     x - lo and the scale, and a wave takes that variant only if one of its sixteen rows needs it;
//   - rows past the end of the list and row ids outside the table are handled by clamping the
//     addresses that are read and masking what is stored, not by branches.
// ---------------------------------------------------------------------------------------------
// Shapes.  Q = dim / 16.  Rows of 64 elements and more (Q = 4 * M) go through the tile in M chunks of
// 64 elements, with 16 rows per pass, 16 lanes per row in the load layout and 4 in the compute
// layout, as described above.  Rows of 32 and 16 elements (Q = 2, 1) keep 4 KB per pass by taking
// 32 and 64 rows per pass: 8 and 4 lanes per row in the load layout, 2 and 1 in the compute layout
// (a lane still holds 16 consecutive elements).
template <int Q>
struct TileShape {
    static_assert(Q == 1 || Q == 2 || (Q >= 4 && Q % 4 == 0), "row length");
    static constexpr int DIM = 16 * Q;
    static constexpr int LC = Q >= 4 ? 4 : Q;        // lanes per row, compute layout
    static constexpr int M = Q >= 4 ? Q / 4 : 1;     // chunks per row
    static constexpr int CHUNK = DIM / M;            // elements per chunk: 64, 32 or 16
    static constexpr int LR = CHUNK / 4;             // lanes per row, load layout
    static constexpr int ROWS = kWave / LC;          // rows per pass: 16, 32 or 64
    static constexpr int ROW_BYTES = 80 * (CHUNK / 16);  // tile: 16 elements + 16 bytes per segment
};
constexpr int kTileBytes = 5120;  // one wave: ROWS * ROW_BYTES for every shape

template <int LC>
__device__ __forceinline__ float row_lanes_min(float v) {  // over the LC lanes of a row
    if constexpr (LC >= 2) v = fminf(v, dpp_f<0xB1>(v));
    if constexpr (LC >= 4) v = fminf(v, dpp_f<0x4E>(v));
    return v;
}
template <int LC>
__device__ __forceinline__ float row_lanes_max(float v) {
    if constexpr (LC >= 2) v = fmaxf(v, dpp_f<0xB1>(v));
    if constexpr (LC >= 4) v = fmaxf(v, dpp_f<0x4E>(v));
    return v;
}

// Quantizes and stores this lane's 16 * M elements of row k (compute layout): x[c][i] holds elements
// CHUNK * c + 16j + 4i .. + 3.
template <int Q, int BITS>
__device__ __forceinline__ void encode_row_share(const QuantArgs &a, uint64_t k, bool live, int j,
                                                 const float4 (&x)[TileShape<Q>::M][4]) {
    using S = TileShape<Q>;
    constexpr int M = S::M, LC = S::LC, DIM = S::DIM;
    constexpr float QMAXF = (float)((1 << BITS) - 1);
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;  // packed bytes per row
    constexpr float MAGIC = 12582912.0f;              // 1.5 * 2^23: x + MAGIC rounds x to an integer
    constexpr uint32_t MAGIC_BITS = 0x4B400000u;      // bit pattern of MAGIC
    // what four magic-biased codes add up to when merged with shifts of B, 2B, 3B bits
    constexpr uint32_t MERGED_BIAS = MAGIC_BITS * (1u + (1u << BITS) + (1u << (2 * BITS)) + (1u << (3 * BITS)));
    constexpr uint32_t MERGED_BIAS8 = MAGIC_BITS * (1u + (1u << 8) + (1u << 16) + (1u << 24));

    // ---- row minimum / maximum
    float mn = x[0][0].x, mx = x[0][0].x;
#pragma unroll
    for (int c = 0; c < M; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mn = fminf(fminf(mn, x[c][i].x), fminf(x[c][i].y, fminf(x[c][i].z, x[c][i].w)));
            mx = fmaxf(fmaxf(mx, x[c][i].x), fmaxf(x[c][i].y, fmaxf(x[c][i].z, x[c][i].w)));
        }
    const float X_min = row_lanes_min<LC>(mn) + 0.0f;  // -0.0 -> +0.0
    const float X_max = row_lanes_max<LC>(mx) + 0.0f;
    float lo = X_min, hi = X_max;
    if (a.mode == kModeSymmetric) {
        const float m = fmaxf(fabsf(X_min), fabsf(X_max));
        lo = -m + 0.0f;
        hi = m;
    }

    // ---- the row's parameters: with four lanes per row, lane 0 writes scale, lane 1 bias, lanes 2, 3
    // min, max; with fewer, the lanes there are share them out
    const float scale = (hi - lo) / QMAXF;
    if constexpr (LC == 4) {
        float *dst = j == 0 ? a.scale : j == 1 ? a.bias : j == 2 ? a.row_min : a.row_max;
        const float v = j == 0 ? scale : j == 1 ? lo : j == 2 ? X_min : X_max;
        if (dst && live) store_stream<float>(dst + k, v);
    } else {
        if (live && j == 0) store_stream<float>(a.scale + k, scale);
        if (live && j == LC - 1) store_stream<float>(a.bias + k, lo);
        if (live && j == 0 && a.row_min) store_stream<float>(a.row_min + k, X_min);
        if (live && j == LC - 1 && a.row_max) store_stream<float>(a.row_max + k, X_max);
    }
    const float f = scale < 0x1p-100f ? 0x1p120f : scale > 0x1p100f ? 0x1p-120f : 1.0f;
    const float fscale = scale * f;
    const float inv = scale == 0.0f ? 0.0f : 1.0f / fscale;  // scale 0: every code 0

    // ---- quantize; h[c][i] = the four codes of x[c][i], first element lowest
    uint32_t h[M][4];
    auto quantize_by_reciprocal = [&](auto rescale) {
        constexpr bool RESCALE = decltype(rescale)::value;
        // magic-biased code of one element: MAGIC_BITS + round((x - lo) / scale)
        auto biased = [&](float xv) -> uint32_t {
            float d0 = xv - lo;
            if constexpr (RESCALE) d0 *= f;
            float t = d0 * inv;
            if constexpr (BITS == 8) t = fmaf(fmaf(-t, fscale, d0), inv, t);
            return __float_as_uint(t + MAGIC);
        };
#pragma unroll
        for (int c = 0; c < M; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 v = x[c][i];
                const uint32_t b0 = biased(v.x), b1 = biased(v.y), b2 = biased(v.z), b3 = biased(v.w);
                uint32_t m = (b3 << BITS) + b2;
                m = (m << BITS) + b1;
                h[c][i] = (m << BITS) + b0 - MERGED_BIAS;
                if (a.codes && live)  // one code per byte as well (uniform branch)
                    *reinterpret_cast<uint32_t *>(a.codes + k * (uint64_t)DIM + S::CHUNK * c + 16 * j + 4 * i) =
                        (((((b3 << 8) + b2) << 8) + b1) << 8) + b0 - MERGED_BIAS8;
            }
    };
    if (__builtin_amdgcn_ballot_w64(f != 1.0f) != 0)
        quantize_by_reciprocal(std::true_type{});
    else
        quantize_by_reciprocal(std::false_type{});

#pragma unroll
    for (int c = 0; c < M; ++c) {
        // ---- packed codes: this lane's bits are 2 * BITS contiguous bytes of the row
        if (a.packed) {
            uint8_t *dst = a.packed + k * P + (2 * BITS * LC) * c + (2 * BITS) * j;
            if constexpr (BITS == 8) {
                if (live) store_stream<u32x4>(dst, u32x4{h[c][0], h[c][1], h[c][2], h[c][3]});
            } else if constexpr (BITS == 4) {
                if (live) store_stream<u32x2>(dst, u32x2{h[c][0] | (h[c][1] << 16), h[c][2] | (h[c][3] << 16)});
            } else if constexpr (BITS == 2) {
                if (live) store_stream<uint32_t>(dst, h[c][0] | (h[c][1] << 8) | (h[c][2] << 16) | (h[c][3] << 24));
            } else {  // 3 bits: 48 bits per lane; even lanes append their right neighbour's 48 bits
                const uint32_t w0 = h[c][0] | (h[c][1] << 12) | (h[c][2] << 24);  // stream bits 0..31
                const uint32_t w1 = (h[c][2] >> 8) | (h[c][3] << 4);              // stream bits 32..47
                if constexpr (LC == 1) {  // the row is this lane's 48 bits alone
                    uint16_t *d2 = reinterpret_cast<uint16_t *>(dst);
                    if (live) {
                        d2[0] = (uint16_t)w0;
                        d2[1] = (uint16_t)(w0 >> 16);
                        d2[2] = (uint16_t)w1;
                    }
                } else {
                    const uint32_t n0 = (uint32_t)dpp_i<0xB1>((int)w0);  // lane ^ 1
                    const uint32_t n1 = (uint32_t)dpp_i<0xB1>((int)w1);
                    if (live && !(j & 1)) {
                        uint32_t *d3 = reinterpret_cast<uint32_t *>(dst);
                        store_stream<uint32_t>(d3, w0);
                        store_stream<uint32_t>(d3 + 1, w1 | (n0 << 16));
                        store_stream<uint32_t>(d3 + 2, (n0 >> 16) | (n1 << 16));
                    }
                }
            }
        }
    }
}

// Row ids a lane needs for one pass: of the four rows it helps to load, and of the row it encodes.
struct PassIds {
    uint32_t rid[4];
    uint32_t own;
};

// Ids of pass `pass` of ROWS rows (which must hold at least one row).  Rows past the end repeat the
// last row of the pass; nothing of theirs is stored.
template <int ROWS>
__device__ __forceinline__ void load_pass_ids(const QuantArgs &a, uint64_t n, uint64_t pass, int g, int rho, PassIds &o) {
    const uint64_t base = pass * (uint64_t)ROWS;
    const uint64_t left = n - base;
    const uint32_t rows = left < (uint64_t)ROWS ? (uint32_t)left : (uint32_t)ROWS;  // uniform
    const uint32_t own_i = (uint32_t)rho < rows ? (uint32_t)rho : rows - 1u;
    uint32_t idx[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) idx[u] = (uint32_t)(4 * g + u) < rows ? (uint32_t)(4 * g + u) : rows - 1u;
    if (!a.row_ids) {  // row k of the list is row k of the table; beyond 2^32 - 1: outside any table
        const uint64_t ko = base + own_i;
        o.own = ko > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)ko;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t ku = base + idx[u];
            o.rid[u] = ku > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)ku;
        }
        return;
    }
    o.own = a.row_ids[base + own_i];
    if (rows == (uint32_t)ROWS) {  // one 16-byte load
        const uint4 v = *reinterpret_cast<const uint4 *>(a.row_ids + base + 4u * (uint32_t)g);
        o.rid[0] = v.x; o.rid[1] = v.y; o.rid[2] = v.z; o.rid[3] = v.w;
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) o.rid[u] = a.row_ids[base + idx[u]];
    }
}

template <int Q, int BITS>
__device__ __forceinline__ void encode_table(const QuantArgs &a, unsigned char *tile /* this wave's kTileBytes of LDS */) {
    using S = TileShape<Q>;
    constexpr int DIM = S::DIM, M = S::M, ROWS = S::ROWS;
    const uint64_t n = row_count(a);
    const int lane = tid_x() & (kWave - 1);
    const int g = lane / S::LR, l = lane % S::LR;   // load layout: group (four rows), lane in group
    const int rho = lane / S::LC, j = lane % S::LC; // compute layout: row of the pass, share of the row
    const uint32_t last_row = (uint32_t)a.n_rows - 1u;  // the host checks 1 <= n_rows < 2^32
    unsigned char *const wr = tile + (4 * g) * S::ROW_BYTES + (l >> 2) * 80 + (l & 3) * 16;
    const unsigned char *const rd = tile + rho * S::ROW_BYTES + j * 80;

    // Requests this lane's share of the rows of a pass (ids outside the table read the last row
    // instead).
    f32x4 ld[4][M];
    auto gather = [&](const PassIds &ids) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t r = ids.rid[u] < last_row ? ids.rid[u] : last_row;
            const float *src = a.table + (uint64_t)r * DIM + 4u * (uint32_t)l;
#pragma unroll
            for (int c = 0; c < M; ++c) ld[u][c] = load_stream<f32x4>(src + S::CHUNK * c);
        }
    };

    // Software pipeline: while a pass is transposed, quantized and stored, the rows of the wave's
    // next pass and the ids of the one after that are on their way.
    const uint32_t n_waves = a.n_waves;
    uint64_t pass = wave_in_grid();
    if (pass * ROWS >= n) return;
    PassIds ids;
    load_pass_ids<ROWS>(a, n, pass, g, rho, ids);
    gather(ids);
    uint32_t own = ids.own;
    uint64_t next = pass + n_waves;
    if (next * ROWS < n) load_pass_ids<ROWS>(a, n, next, g, rho, ids);
    for (;;) {
        const uint64_t base = pass * (uint64_t)ROWS;  // first row of the pass (uniform)
        const uint64_t left = n - base;
        const uint32_t rows = left < (uint64_t)ROWS ? (uint32_t)left : (uint32_t)ROWS;
        const bool in_table = own <= last_row;
        const bool live = (uint32_t)rho < rows && in_table;
        if ((uint32_t)rho < rows && !in_table && j == 0) raise_flag(a.err, CNR_FLAG_ROW_ID);

        // ---- transpose through the wave's LDS tile, one chunk at a time
        float4 x[M][4];
#pragma unroll
        for (int c = 0; c < M; ++c) {
#pragma unroll
            for (int u = 0; u < 4; ++u) *reinterpret_cast<f32x4 *>(wr + u * S::ROW_BYTES) = ld[u][c];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 4; ++i) x[c][i] = *reinterpret_cast<const float4 *>(rd + 16 * i);
            __builtin_amdgcn_wave_barrier();
        }

        // ---- the load registers are free again: request the next pass
        const bool has_next = next * ROWS < n;  // uniform
        const uint64_t next2 = next + n_waves;
        if (has_next) {
            gather(ids);
            own = ids.own;
            if (next2 * ROWS < n) load_pass_ids<ROWS>(a, n, next2, g, rho, ids);
        }

        encode_row_share<Q, BITS>(a, base + (uint32_t)rho, live, j, x);
        if (!has_next) break;
        pass = next;
        next = next2;
    }
}

// One launch takes up to CNR_MAX_BATCH tables (grid y = table; a slice of a long list counts as a
// table).  Workgroups are handed out x first, so the tables of a launch are swept one after the
// other by all compute units, each on one moving front, with nothing idle between them; a table
// that needs fewer workgroups than the largest of the launch sends the surplus home at once.
// The register budget is pinned to 6 / 4 / 2 waves per SIMD for rows of up to 64 / 128 / 256
// elements: left alone, the compiler lands a few registers to either side of those limits from one
// small change to the next.
struct QuantBatchArgs {
    QuantArgs job[CNR_MAX_BATCH];
};
template <int Q, int BITS>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(Q <= 4 ? 6 : Q == 8 ? 4 : 2, Q <= 4 ? 6 : Q == 8 ? 4 : 2)))
quantize_tile_kernel(const QuantBatchArgs b) {
    __shared__ __align__(16) unsigned char tiles[kWavesPerBlock * kTileBytes];
    const QuantArgs &a = b.job[wg_y()];
    if (wg_x() * kWavesPerBlock >= a.n_waves) return;
    encode_table<Q, BITS>(a, tiles + (tid_x() / kWave) * kTileBytes);
}

// ---------------------------------------------------------------------------------------------
// Greedy range search (Approach 3), dim = 16 * G * L in {16, 32, 64, 128, 256}: L lanes per row, G
// groups of sixteen elements per lane.  Bound by vector-ALU issue: 1 + 2 * n_iter candidate ranges are
// tried per row.
//
// Every lane owns 16 * G consecutive elements (4 * G 16-byte loads) of one row, L neighbouring lanes
// own the row, a wave handles 64 / L consecutive dirty rows per pass.  A candidate's error is summed
// over a lane's registers and then over the L lanes with log2(L) DPP exchanges, and a group's sixteen
// codes are exactly 2 * BITS contiguous bytes of the packed row.  What a candidate costs beyond its
// elements (its scale and reciprocal, the exchange between lanes, the comparison) is paid once per
// lane, so more elements per lane mean less of it: with 64 instead of 16 (G = 4; a row of 64 floats
// is then one lane's, with no exchange at all) a long list takes 13 % less time, 0.90 instead of 0.78
// of the issue bound of the element arithmetic alone.  A lane then works four times as long on a
// row, so short lists, which cannot fill the SIMDs either way, keep G = 1.  The rows are read in this
// layout directly (each lane its own 64 * G bytes): the kernel is far from the memory system's limits,
// so the transpose through LDS that the tile kernel pays for coalesced loads would buy nothing.
// A candidate is evaluated with the cheapest sequence that still ranks candidates as F_Q would.  On
// this GPU a wave's add, subtract or multiply occupies a SIMD for two clocks, every other vector
// instruction used here (fused multiply-add, median, round, conversion, all fp64) for four (measured
// with single-instruction loops), so an element costs 26 clocks per candidate: clip (4), subtract (2),
// multiply by the reciprocal of the scale (2), round (4), de-quantize (2 + 2), residual (2), convert
// and accumulate its square in fp64 (4 + 4; d * d is exact in fp64, so fma(d, d, acc) is the
// multiply-then-add of the definition).  The candidate's scale is range / (2^b - 1) correctly rounded
// (reciprocal multiply plus one FMA residual step) and its reciprocal likewise; the quotient itself
// is the plain product, within 1.5 ulp of the correctly rounded quotient, which can move a code of a
// candidate only where the quotient lies that close to a half-integer (about 3 elements in a million
// at 4 bits) and then changes the candidate's error by about 1e-7 of itself: a search leaves the path
// of the divide-as-written sequence only if that coincides with two candidates that close, about one
// row in a few million.  (Correcting the quotient too, two more FMAs per element, took 34 clocks per
// element and candidate.)  A wave holding a row whose scale lies outside [2^-100, 2^100], or whose
// span is only a few float spacings wide, divides instead.  The final codes of the chosen range are
// produced by division, exactly as F_Q is written.
// ---------------------------------------------------------------------------------------------
template <int L>
__device__ __forceinline__ float lanes_min(float v) {
    if constexpr (L >= 2) v = fminf(v, dpp_f<0xB1>(v));
    if constexpr (L >= 4) v = fminf(v, dpp_f<0x4E>(v));
    if constexpr (L >= 8) v = fminf(v, dpp_f<0x141>(v));
    if constexpr (L >= 16) v = fminf(v, dpp_f<0x140>(v));
    return v;
}
template <int L>
__device__ __forceinline__ float lanes_max(float v) {
    if constexpr (L >= 2) v = fmaxf(v, dpp_f<0xB1>(v));
    if constexpr (L >= 4) v = fmaxf(v, dpp_f<0x4E>(v));
    if constexpr (L >= 8) v = fmaxf(v, dpp_f<0x141>(v));
    if constexpr (L >= 16) v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
template <int L>
__device__ __forceinline__ double lanes_sum(double v) {
    if constexpr (L >= 2) v += dpp_d<0xB1>(v);
    if constexpr (L >= 4) v += dpp_d<0x4E>(v);
    if constexpr (L >= 8) v += dpp_d<0x141>(v);
    if constexpr (L >= 16) v += dpp_d<0x140>(v);
    return v;
}

template <int L, int BITS, int G>
__global__ void __launch_bounds__(kBlock) quantize_greedy_kernel(const QuantArgs a, uint64_t n_from, uint64_t n_below) {
    constexpr int EPL = 16 * G;  // elements per lane
    constexpr int DIM = EPL * L;
    constexpr int kRowsPerPass = kWave / L;
    constexpr float QMAXF = (float)((1 << BITS) - 1);
    constexpr float INV_QMAX = 1.0f / QMAXF;
    constexpr uint64_t P = (uint64_t)DIM * BITS / 8;  // packed bytes per row
    const uint64_t n = row_count(a);
    if (n < n_from || n >= n_below) return;  // this list length is the other launch's (uniform over the grid)
    const int lane = tid_x() & (kWave - 1);
    const int j = lane % L;  // lane within the row
    const uint32_t n_waves = a.n_waves;
    for (uint64_t pass = wave_in_grid(); pass * kRowsPerPass < n; pass += n_waves) {
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
        float4 x[4 * G];
        {
            const float *src = a.table + rid * (uint64_t)DIM + (uint64_t)(EPL * j);
#pragma unroll
            for (int i = 0; i < 4 * G; ++i) x[i] = *reinterpret_cast<const float4 *>(src + 4 * i);
        }

        // ---- row minimum / maximum
        float mn = fminf(fminf(x[0].x, x[0].y), fminf(x[0].z, x[0].w));
        float mx = fmaxf(fmaxf(x[0].x, x[0].y), fmaxf(x[0].z, x[0].w));
#pragma unroll
        for (int i = 1; i < 4 * G; ++i) {
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
                    const float t = (c - c_lo) * inv;
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
                for (int i = 0; i < 4 * G; ++i) {
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
        // The bounds are moved by cumulative fp32 additions, each rounded to the spacing of the bounds'
        // magnitude, so after k moves a bound sits up to k/2 spacings off the exact lattice.  Where the
        // step is not many spacings wide (a row whose span is tiny against its magnitude) a candidate
        // range can close or turn inside out before the search ends, and there the median-of-three
        // clip of the fast sequence is no longer min(max(x, lo), hi): such rows take the sequence as
        // F_Q is written.  Safe when range >= num_bins^2 spacings (twice the drift num_bins moves allow).
        const float mag = fmaxf(fabsf(lo), fabsf(hi));
        const bool narrow = hi != lo && (hi - lo) < a.num_bins_f * a.num_bins_f * (mag * 0x1p-23f);
        // the last candidates are up to num_bins times narrower than the first
        if (__builtin_amdgcn_ballot_w64(odd_scale || narrow) != 0 || a.num_bins_f > 0x1p20f)
            search(std::false_type{});
        else
            search(std::true_type{});

        // ---- per-row parameters: lane 0 of the row writes scale, lane 1 bias, lanes 2, 3 min, max
        // (with fewer than four lanes per row, the lanes there are share them out)
        const float scale = (hi - lo) / QMAXF;
        if constexpr (L >= 4) {
            float *dst = j == 0 ? a.scale : j == 1 ? a.bias : j == 2 ? a.row_min : a.row_max;
            const float v = j == 0 ? scale : j == 1 ? lo : j == 2 ? X_min : X_max;
            if (j < 4 && dst && live) dst[k] = v;
        } else {
            if (live && j == 0) a.scale[k] = scale;
            if (live && j == L - 1) a.bias[k] = lo;
            if (live && j == 0 && a.row_min) a.row_min[k] = X_min;
            if (live && j == L - 1 && a.row_max) a.row_max[k] = X_max;
        }

        // ---- final codes by F_Q as written; h[i] = the four codes of x[i], first element lowest
        uint32_t h[4 * G], h8[4 * G];
#pragma unroll
        for (int i = 0; i < 4 * G; ++i) {
            const uint32_t q0 = (uint32_t)fq_code_f(x[i].x, lo, hi, scale, QMAXF);
            const uint32_t q1 = (uint32_t)fq_code_f(x[i].y, lo, hi, scale, QMAXF);
            const uint32_t q2 = (uint32_t)fq_code_f(x[i].z, lo, hi, scale, QMAXF);
            const uint32_t q3 = (uint32_t)fq_code_f(x[i].w, lo, hi, scale, QMAXF);
            h[i] = q0 | (q1 << BITS) | (q2 << (2 * BITS)) | (q3 << (3 * BITS));
            h8[i] = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
        }
        if (a.codes && live) {
#pragma unroll
            for (int g = 0; g < G; ++g)
                *reinterpret_cast<uint4 *>(a.codes + k * (uint64_t)DIM + EPL * j + 16 * g) =
                    make_uint4(h8[4 * g], h8[4 * g + 1], h8[4 * g + 2], h8[4 * g + 3]);
        }

        // ---- packed codes: this lane's bits are bytes [2 * BITS * G * j, 2 * BITS * G * (j + 1)) of the row,
        // 2 * BITS bytes per group of sixteen elements
        if (a.packed) {
            uint8_t *dst = a.packed + k * P + 2 * BITS * G * j;
            if constexpr (BITS == 8) {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (live) *reinterpret_cast<uint4 *>(dst + 16 * g) = make_uint4(h[4 * g], h[4 * g + 1], h[4 * g + 2], h[4 * g + 3]);
            } else if constexpr (BITS == 4) {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (live)
                        *reinterpret_cast<uint2 *>(dst + 8 * g) =
                            make_uint2(h[4 * g] | (h[4 * g + 1] << 16), h[4 * g + 2] | (h[4 * g + 3] << 16));
            } else if constexpr (BITS == 2) {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (live)
                        *reinterpret_cast<uint32_t *>(dst + 4 * g) =
                            h[4 * g] | (h[4 * g + 1] << 8) | (h[4 * g + 2] << 16) | (h[4 * g + 3] << 24);
            } else {  // 3 bits: 48 bits per group
                uint32_t w0[G], w1[G];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    w0[g] = h[4 * g] | (h[4 * g + 1] << 12) | (h[4 * g + 2] << 24);  // stream bits 0..31 of the group
                    w1[g] = (h[4 * g + 2] >> 8) | (h[4 * g + 3] << 4);               // stream bits 32..47
                }
                if constexpr (G >= 2) {  // two groups make three whole words
#pragma unroll
                    for (int g = 0; g < G; g += 2) {
                        uint32_t *d3 = reinterpret_cast<uint32_t *>(dst + 6 * g);
                        if (live) {
                            d3[0] = w0[g];
                            d3[1] = w1[g] | (w0[g + 1] << 16);
                            d3[2] = (w0[g + 1] >> 16) | (w1[g + 1] << 16);
                        }
                    }
                } else if constexpr (L == 1) {  // the row is this lane's 48 bits alone
                    uint16_t *d2 = reinterpret_cast<uint16_t *>(dst);
                    if (live) {
                        d2[0] = (uint16_t)w0[0];
                        d2[1] = (uint16_t)(w0[0] >> 16);
                        d2[2] = (uint16_t)w1[0];
                    }
                } else {  // even lanes append their right neighbour's 48 bits
                    const uint32_t n0 = (uint32_t)dpp_i<0xB1>((int)w0[0]);  // lane ^ 1
                    const uint32_t n1 = (uint32_t)dpp_i<0xB1>((int)w1[0]);
                    if (live && !(j & 1)) {
                        uint32_t *d3 = reinterpret_cast<uint32_t *>(dst);
                        d3[0] = w0[0];
                        d3[1] = w1[0] | (n0 << 16);
                        d3[2] = (n0 >> 16) | (n1 << 16);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Greedy search at any other dim (dim % 4 == 0, dim * bits % 8 == 0): one wavefront per row, lanes
// stride over the row, which is re-read from cache for each candidate.  Output bytes are produced
// one per lane-visit from the codes they cover, so no staging or barrier is needed.  Divides as F_Q
// is written.
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
// Other row lengths, min/max and symmetric range: LPR lanes per row (a power of two, at least the
// row's number of 16-byte units up to 64), 64 / LPR rows per wave and pass; lane j takes the
// units j, j + LPR, ... of its row.  The row is read twice, for its range and to quantize (the second
// time from cache), so nothing depends on its length; a unit's four codes are 4 * BITS bits, stored
// as one, two or four bytes, and at 3 bits even lanes store three bytes for themselves and their
// right neighbour.  Same arithmetic as the tile kernel.
// ---------------------------------------------------------------------------------------------
template <int LPR>
__device__ __forceinline__ float lpr_min(float v) {
    v = fminf(v, dpp_f<0xB1>(v));
    v = fminf(v, dpp_f<0x4E>(v));
    if constexpr (LPR >= 8) v = fminf(v, dpp_f<0x141>(v));
    if constexpr (LPR >= 16) v = fminf(v, dpp_f<0x140>(v));
    if constexpr (LPR >= 32) v = fminf(v, __shfl_xor(v, 16));
    if constexpr (LPR >= 64) v = fminf(v, __shfl_xor(v, 32));
    return v;
}
template <int LPR>
__device__ __forceinline__ float lpr_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    if constexpr (LPR >= 8) v = fmaxf(v, dpp_f<0x141>(v));
    if constexpr (LPR >= 16) v = fmaxf(v, dpp_f<0x140>(v));
    if constexpr (LPR >= 32) v = fmaxf(v, __shfl_xor(v, 16));
    if constexpr (LPR >= 64) v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

template <int LPR, int BITS>
__global__ void __launch_bounds__(kBlock) quantize_strided_kernel(const QuantArgs a) {
    constexpr int kRowsPerPass = kWave / LPR;
    constexpr float QMAXF = (float)((1 << BITS) - 1);
    constexpr float MAGIC = 12582912.0f;          // 1.5 * 2^23 (see the tile kernel)
    constexpr uint32_t MAGIC_BITS = 0x4B400000u;
    constexpr uint32_t MERGED_BIAS = MAGIC_BITS * (1u + (1u << BITS) + (1u << (2 * BITS)) + (1u << (3 * BITS)));
    constexpr uint32_t MERGED_BIAS8 = MAGIC_BITS * (1u + (1u << 8) + (1u << 16) + (1u << 24));
    const uint64_t n = row_count(a);
    const uint32_t dim = a.dim, n4 = dim / 4;      // 16-byte units per row
    const uint64_t P = (uint64_t)dim * BITS / 8;   // packed bytes per row
    const int lane = tid_x() & (kWave - 1);
    const uint32_t j = lane % LPR;
    const uint32_t last_row = (uint32_t)a.n_rows - 1u;
    const uint32_t n_waves = a.n_waves;
    for (uint64_t pass = wave_in_grid(); pass * kRowsPerPass < n; pass += n_waves) {
        const uint64_t k = pass * kRowsPerPass + lane / LPR;
        const uint64_t kc = k < n ? k : n - 1;     // rows past the end repeat the last one; nothing of theirs is stored
        uint32_t rid;
        if (a.row_ids)
            rid = a.row_ids[kc];
        else
            rid = kc > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)kc;
        const bool in_table = rid <= last_row;
        const bool live = k < n && in_table;
        if (k < n && !in_table && j == 0) raise_flag(a.err, CNR_FLAG_ROW_ID);
        const float4 *row = reinterpret_cast<const float4 *>(a.table + (uint64_t)(in_table ? rid : last_row) * dim);

        // ---- row minimum / maximum (every lane starts from the row's first unit, so idle lanes are neutral)
        const float4 first = row[0];
        float mn = fminf(fminf(first.x, first.y), fminf(first.z, first.w));
        float mx = fmaxf(fmaxf(first.x, first.y), fmaxf(first.z, first.w));
        for (uint32_t u = j; u < n4; u += LPR) {
            const float4 v = row[u];
            mn = fminf(fminf(mn, v.x), fminf(v.y, fminf(v.z, v.w)));
            mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
        }
        const float X_min = lpr_min<LPR>(mn) + 0.0f;  // -0.0 -> +0.0
        const float X_max = lpr_max<LPR>(mx) + 0.0f;
        float lo = X_min, hi = X_max;
        if (a.mode == kModeSymmetric) {
            const float m = fmaxf(fabsf(X_min), fabsf(X_max));
            lo = -m + 0.0f;
            hi = m;
        }
        const float scale = (hi - lo) / QMAXF;
        {
            float *dst = j == 0 ? a.scale : j == 1 ? a.bias : j == 2 ? a.row_min : a.row_max;
            const float v = j == 0 ? scale : j == 1 ? lo : j == 2 ? X_min : X_max;
            if (j < 4 && dst && live) dst[k] = v;
        }
        const float f = scale < 0x1p-100f ? 0x1p120f : scale > 0x1p100f ? 0x1p-120f : 1.0f;
        const float fscale = scale * f;
        const float inv = scale == 0.0f ? 0.0f : 1.0f / fscale;  // scale 0: every code 0
        auto biased = [&](float xv) -> uint32_t {  // MAGIC_BITS + round((x - lo) / scale)
            const float d0 = (xv - lo) * f;
            float t = d0 * inv;
            if constexpr (BITS == 8) t = fmaf(fmaf(-t, fscale, d0), inv, t);
            return __float_as_uint(t + MAGIC);
        };

        // ---- quantize unit by unit; all lanes take every trip so that the 3-bit exchange has partners
        const uint32_t trips = (n4 + LPR - 1) / LPR;
        for (uint32_t trip = 0; trip < trips; ++trip) {
            const uint32_t u = j + trip * LPR;
            const bool mine = u < n4;
            const float4 v = row[mine ? u : 0];
            const uint32_t b0 = biased(v.x), b1 = biased(v.y), b2 = biased(v.z), b3 = biased(v.w);
            uint32_t m = (b3 << BITS) + b2;
            m = (m << BITS) + b1;
            const uint32_t h = (m << BITS) + b0 - MERGED_BIAS;  // 4 * BITS bits
            const bool store = mine && live;
            if (a.codes && store)
                *reinterpret_cast<uint32_t *>(a.codes + k * (uint64_t)dim + 4 * u) =
                    (((((b3 << 8) + b2) << 8) + b1) << 8) + b0 - MERGED_BIAS8;
            if (a.packed) {
                uint8_t *out = a.packed + k * P;
                if constexpr (BITS == 8) {
                    if (store) *reinterpret_cast<uint32_t *>(out + 4 * u) = h;
                } else if constexpr (BITS == 4) {
                    if (store) *reinterpret_cast<uint16_t *>(out + 2 * u) = (uint16_t)h;
                } else if constexpr (BITS == 2) {
                    if (store) out[u] = (uint8_t)h;
                } else {  // 3 bits: units come in pairs (dim % 8 == 0); the even one stores both
                    const uint32_t nb = (uint32_t)dpp_i<0xB1>((int)h);  // lane ^ 1: unit u + 1
                    if (store && !(u & 1)) {
                        const uint32_t w = h | (nb << 12);
                        uint8_t *o3 = out + 3 * (u >> 1);
                        o3[0] = (uint8_t)w;
                        o3[1] = (uint8_t)(w >> 8);
                        o3[2] = (uint8_t)(w >> 16);
                    }
                }
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

// n tables (or slices) in one launch: every one with the grid its own list calls for (cnr_row_grid).
template <int Q, int BITS>
void launch_tile(QuantBatchArgs &b, uint32_t n, hipStream_t s) {
    unsigned grid = 1;
    for (uint32_t i = 0; i < n; ++i) {
        const unsigned g = cnr_row_grid(b.job[i].n_max, (uint64_t)TileShape<Q>::ROWS * kWavesPerBlock);
        b.job[i].n_waves = g * kWavesPerBlock;
        if (g > grid) grid = g;
    }
    hipLaunchKernelGGL((quantize_tile_kernel<Q, BITS>), dim3(grid, n), dim3(kBlock), 0, s, b);
}
template <int BITS>
void launch_tile_bits(QuantBatchArgs &b, uint32_t n, uint32_t dim, hipStream_t s) {
    switch (dim) {
        case 16: return launch_tile<1, BITS>(b, n, s);
        case 32: return launch_tile<2, BITS>(b, n, s);
        case 64: return launch_tile<4, BITS>(b, n, s);
        case 128: return launch_tile<8, BITS>(b, n, s);
        default: return launch_tile<16, BITS>(b, n, s);
    }
}
inline void launch_tile_any(QuantBatchArgs &b, uint32_t n, uint32_t dim, int bits, hipStream_t s) {
    switch (bits) {
        case 2: return launch_tile_bits<2>(b, n, dim, s);
        case 3: return launch_tile_bits<3>(b, n, dim, s);
        case 4: return launch_tile_bits<4>(b, n, dim, s);
        default: return launch_tile_bits<8>(b, n, dim, s);
    }
}

// Runs for lists of n_from <= n < n_below rows (n is the count on the device where there is one).
template <int L, int BITS, int G>
void launch_greedy(cnr_ctx *ctx, QuantArgs &a, hipStream_t s, uint64_t n_from, uint64_t n_below) {
    // the large grid here too: the search is bound by arithmetic, but workgroups handed out as others
    // finish even out the end of the launch (4 % on a 1.5 M-row list)
    const uint64_t most = a.n_max < n_below ? a.n_max : n_below;
    const unsigned grid = cnr_row_grid(most, (uint64_t)(kWave / L) * kWavesPerBlock);
    a.n_waves = grid * kWavesPerBlock;
    hipLaunchKernelGGL((quantize_greedy_kernel<L, BITS, G>), dim3(grid), dim3(kBlock), 0, s, a, n_from, n_below);
}
// Long lists give every lane 64 elements (32 at dim 32); short ones keep 16 per lane, four times the
// lanes per row and a quarter of the time per row, which is what counts while the list cannot fill
// the SIMDs anyway.  The break-even was measured at about 8 M elements (128 K rows of 64).  Where the
// length is a count on the device and the capacity allows a long list, both kernels are launched
// and the one whose range the count is not in returns at once.
template <int L_NARROW, int L_WIDE, int G_WIDE, int BITS>
void launch_greedy_by_length(cnr_ctx *ctx, QuantArgs &a, hipStream_t s) {
    const uint64_t wide_rows = (1ull << 23) / a.dim;
    const bool may_be_wide = a.n_max >= wide_rows;
    const bool may_be_narrow = !may_be_wide || a.n_dev != nullptr;
    if (may_be_narrow) launch_greedy<L_NARROW, BITS, 1>(ctx, a, s, 0, may_be_wide ? wide_rows : ~0ull);
    if (may_be_wide) launch_greedy<L_WIDE, BITS, G_WIDE>(ctx, a, s, may_be_narrow ? wide_rows : 0, ~0ull);
}

template <int LPR, int BITS>
void launch_strided(cnr_ctx *ctx, QuantArgs &a, hipStream_t s) {
    const unsigned grid = cnr_grid(ctx, a.n_max, (uint64_t)(kWave / LPR) * kWavesPerBlock,
                                   cnr_resident_blocks_per_cu<quantize_strided_kernel<LPR, BITS>>());
    a.n_waves = grid * kWavesPerBlock;
    hipLaunchKernelGGL((quantize_strided_kernel<LPR, BITS>), dim3(grid), dim3(kBlock), 0, s, a);
}

// The kernels that take one table per launch: the greedy search at any row length, and min/max or
// symmetric ranges at row lengths the tile kernel does not take.
template <int BITS>
void launch_bits(cnr_ctx *ctx, QuantArgs &a, hipStream_t s) {
    const bool greedy = a.mode == kModeGreedy && a.n_iter > 0;  // zero iterations: plain min/max
    if (greedy && a.dim == 16) return launch_greedy<1, BITS, 1>(ctx, a, s, 0, ~0ull);
    if (greedy && a.dim == 32) return launch_greedy_by_length<2, 1, 2, BITS>(ctx, a, s);
    if (greedy && a.dim == 64) return launch_greedy_by_length<4, 1, 4, BITS>(ctx, a, s);
    if (greedy && a.dim == 128) return launch_greedy_by_length<8, 2, 4, BITS>(ctx, a, s);
    if (greedy && a.dim == 256) return launch_greedy_by_length<16, 4, 4, BITS>(ctx, a, s);
    if (greedy) {  // other row lengths, greedy: one wave per row
        const unsigned grid = cnr_grid(ctx, a.n_max, kWavesPerBlock, 8);
        hipLaunchKernelGGL((quantize_rows_generic_kernel<BITS>), dim3(grid), dim3(kBlock), 0, s, a.table,
                           a.n_rows, a.dim, a.row_ids, a.n_dev, a.n_max, a.mode, a.n_iter, a.num_bins_f,
                           a.scale, a.bias, a.row_min, a.row_max, a.codes, a.packed, a.err);
        return;
    }
    const uint32_t n4 = a.dim / 4;
    if (n4 <= 4) return launch_strided<4, BITS>(ctx, a, s);
    if (n4 <= 8) return launch_strided<8, BITS>(ctx, a, s);
    if (n4 <= 16) return launch_strided<16, BITS>(ctx, a, s);
    if (n4 <= 32) return launch_strided<32, BITS>(ctx, a, s);
    return launch_strided<64, BITS>(ctx, a, s);
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
        if (((uintptr_t)j.table % 16) || ((uintptr_t)j.packed % 16) || ((uintptr_t)j.codes_u8 % 16) ||
            ((uintptr_t)j.scale % 4) || ((uintptr_t)j.bias % 4) || ((uintptr_t)j.row_min % 4) ||
            ((uintptr_t)j.row_max % 4) || ((uintptr_t)j.row_ids % 16) || ((uintptr_t)j.n_dirty_dev % 8))
            return CNR_E_ALIGN;
    }
    hipStream_t s = as_stream(stream);
    const uint32_t n_iter = mode == CNR_RANGE_GREEDY ? cnr_greedy_iterations(greedy->num_bins, greedy->ratio) : 0;
    const uint64_t prb = (uint64_t)dim * (uint64_t)bits / 8u;
    // rows k0 .. k0 + m - 1 of job j's list as arguments of its own
    auto part = [&](const cnr_table_job &j, uint64_t k0, uint64_t m) {
        QuantArgs a = {};
        a.dim = dim;
        if (j.row_ids) {
            a.table = j.table; a.n_rows = j.n_rows; a.row_ids = j.row_ids + k0;
        } else {  // no id list: the table from row k0 on
            a.table = j.table + k0 * dim; a.n_rows = j.n_rows - k0; a.row_ids = nullptr;
        }
        a.n_dev = j.n_dirty_dev; a.n_max = m;
        a.mode = (int)mode; a.n_iter = n_iter;
        a.num_bins_f = mode == CNR_RANGE_GREEDY ? (float)greedy->num_bins : 1.0f;
        a.scale = j.scale + k0; a.bias = j.bias + k0;
        a.row_min = j.row_min ? j.row_min + k0 : nullptr;
        a.row_max = j.row_max ? j.row_max + k0 : nullptr;
        a.codes = j.codes_u8 ? j.codes_u8 + k0 * dim : nullptr;
        a.packed = j.packed ? j.packed + k0 * prb : nullptr;
        a.err = ctx->dev_err;
        return a;
    };
    // The tile kernel takes up to CNR_MAX_BATCH tables per launch.  Small tables (rows of at most
    // kSideBySideBytes at capacity) and large ones go into launches of their own kind, so that a
    // small table is not given a large one's grid; a list whose length the host knows is cut into
    // slices (cnr_slice_rows), each a table of the launch.
    const bool tile_dim = dim == 16 || dim == 32 || dim == 64 || dim == 128 || dim == 256;
    if (tile_dim && n_iter == 0) {
        for (int large = 0; large < 2; ++large) {
            QuantBatchArgs b = {};
            uint32_t n = 0;
            auto flush = [&]() -> cnr_status {
                if (n == 0) return CNR_OK;
                launch_tile_any(b, n, dim, bits, s);
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
    // greedy search, other row lengths: one launch per table
    for (uint32_t i = 0; i < n_jobs; ++i) {
        const cnr_table_job &j = jobs[i];
        if (j.capacity == 0) continue;
        QuantArgs a = part(j, 0, j.capacity);
        switch (bits) {
            case 2: launch_bits<2>(ctx, a, s); break;
            case 3: launch_bits<3>(ctx, a, s); break;
            case 4: launch_bits<4>(ctx, a, s); break;
            default: launch_bits<8>(ctx, a, s); break;
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
