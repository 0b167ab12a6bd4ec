// Tracking bit-vector (Section 5.1.1) and its compaction into the incremental view (Section 5.1).
#include "cnr_common.h"

// ---------------------------------------------------------------------------------------------
// mark: one bit per looked-up row.
//
// The index stream is read once, coalesced (each lane one index per pass, four passes in flight).
// Hot rows repeat many times under a skewed lookup distribution, so the word is tested with a
// plain load first and the atomic OR is issued only for bits not yet seen as set: a stale zero
// merely costs a redundant OR, and bits never go back to zero while marking.
// ---------------------------------------------------------------------------------------------
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
mark_kernel(uint32_t *__restrict__ bitmap, uint64_t n_rows, const IdxT *__restrict__ idx,
            uint64_t n, cnr_dev_errors *err) {
    constexpr int kUnroll = 4;
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    unsigned bad = 0;
    for (; i < n; i += stride * kUnroll) {
        IdxT v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t p = i + (uint64_t)u * stride;
            v[u] = p < n ? idx[p] : (IdxT)0;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t p = i + (uint64_t)u * stride;
            if (p >= n) continue;
            const int64_t r = (int64_t)v[u];
            if (r < 0 || (uint64_t)r >= n_rows) {
                ++bad;
                continue;
            }
            uint32_t *w = bitmap + ((uint64_t)r >> 5);
            const uint32_t bit = 1u << ((uint32_t)r & 31u);
            if (!(*w & bit)) atomicOr(w, bit);
        }
    }
    // one atomic per wave that saw out-of-range indices
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off);
    if (bad && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(&err->n_bad_indices, (unsigned long long)bad);
}

// ---------------------------------------------------------------------------------------------
// mark, bulk variant: no atomics.
//
// On this GPU the L2 caches of the eight XCDs are not coherent with each other, so a device-scope
// atomic OR is carried out at the memory side: each one costs a 64-byte read and a 32-byte write
// there, and a few million of them dominate a checkpoint.  Plain byte stores do not have that
// problem: different threads may write different bytes of one cache line from anywhere, and
// writing the same value twice is harmless.  So a long index stream is first scattered into one
// flag byte per row (scratch, all zero on entry), and a second kernel folds the flag bytes into
// the bitmap 32 rows per thread, with plain read-modify-write because every bitmap word has exactly
// one owner there, and zeroes the bytes it found set so that the scratch is clean again.
// ---------------------------------------------------------------------------------------------
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
mark_flags_kernel(uint8_t *__restrict__ flags, uint64_t n_rows, const IdxT *__restrict__ idx, uint64_t n,
                  cnr_dev_errors *err) {
    constexpr int kUnroll = 4;
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    unsigned bad = 0;
    for (; i < n; i += stride * kUnroll) {
        IdxT v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t p = i + (uint64_t)u * stride;
            v[u] = p < n ? idx[p] : (IdxT)-1;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t p = i + (uint64_t)u * stride;
            const int64_t r = (int64_t)v[u];
            if (r >= 0 && (uint64_t)r < n_rows)
                flags[r] = 1;
            else if (p < n)
                ++bad;
        }
    }
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off);
    if (bad && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(&err->n_bad_indices, (unsigned long long)bad);
}

// Eight flag bytes (each 0 or 1) to eight bits, first byte in bit 0.
__device__ __forceinline__ uint32_t flags_to_bits(uint64_t eight) {
    return (uint32_t)((eight * 0x0102040810204080ull) >> 56);
}

__global__ void __launch_bounds__(kBlock)
fold_flags_kernel(uint8_t *__restrict__ flags, uint32_t *__restrict__ bitmap, uint64_t n_words) {
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    for (uint64_t w = (uint64_t)blockIdx.x * kBlock + threadIdx.x; w < n_words; w += stride) {
        ulonglong2 *src = reinterpret_cast<ulonglong2 *>(flags + 32u * w);
        const ulonglong2 a = src[0], b = src[1];
        if ((a.x | a.y | b.x | b.y) == 0) continue;
        const uint32_t bits = flags_to_bits(a.x) | (flags_to_bits(a.y) << 8) | (flags_to_bits(b.x) << 16) |
                              (flags_to_bits(b.y) << 24);
        bitmap[w] |= bits;
        src[0] = make_ulonglong2(0, 0);
        src[1] = make_ulonglong2(0, 0);
    }
}

// ---------------------------------------------------------------------------------------------
// compact: set-bit positions in ascending order.
//
// Two kernels, no inter-workgroup waiting.  Each workgroup owns kBlock consecutive 64-bit bitmap
// words (one per thread = 16384 rows).
//   count:   population count of the tile -> block_count[b]
//   scatter: base = sum of block_count[0..b) (read back by every workgroup; at most a few thousand
//            values), exclusive scan of the per-thread counts inside the workgroup (wave shuffles +
//            one LDS step across the four waves), then every wave walks its 64 words: the word
//            itself is the ballot of "row is dirty" for 64 consecutive rows, a lane's rank is the
//            population count of the word below its own bit, so the 64 lanes write a contiguous,
//            ascending run of ids.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t load_tile_word(const uint32_t *__restrict__ bitmap,
                                                   uint64_t n_rows, uint64_t n_words32, uint64_t w64) {
    const uint64_t i0 = 2 * w64, i1 = 2 * w64 + 1;
    uint64_t lo = i0 < n_words32 ? bitmap[i0] : 0u;
    uint64_t hi = i1 < n_words32 ? bitmap[i1] : 0u;
    uint64_t w = lo | (hi << 32);
    // ignore bits at positions >= n_rows
    const uint64_t first_row = w64 * 64u;
    if (first_row >= n_rows) return 0;
    const uint64_t live = n_rows - first_row;
    if (live < 64u) w &= (~0ull) >> (64u - live);
    return w;
}

__device__ __forceinline__ unsigned block_sum_u32(unsigned v, unsigned *lds /* kWavesPerBlock */) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    const int wave = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) lds[wave] = v;
    __syncthreads();
    unsigned t = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
    return t;
}

__global__ void __launch_bounds__(kBlock)
compact_count_kernel(const uint32_t *__restrict__ bitmap, uint64_t n_rows, uint64_t n_words32,
                     uint32_t *__restrict__ block_count) {
    __shared__ unsigned lds[kWavesPerBlock];
    const uint64_t w64 = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const unsigned c = __popcll(load_tile_word(bitmap, n_rows, n_words32, w64));
    const unsigned total = block_sum_u32(c, lds);
    if (threadIdx.x == 0) block_count[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kBlock)
compact_scatter_kernel(const uint32_t *__restrict__ bitmap, uint64_t n_rows, uint64_t n_words32,
                       const uint32_t *__restrict__ block_count, uint32_t *__restrict__ row_ids,
                       uint64_t capacity, uint64_t *__restrict__ n_dirty, cnr_dev_errors *err) {
    __shared__ unsigned lds[kWavesPerBlock];
    __shared__ unsigned wave_total[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;

    // dirty rows in all earlier tiles
    unsigned part = 0;
    for (unsigned b = threadIdx.x; b < blockIdx.x; b += kBlock) part += block_count[b];
    const uint64_t base = block_sum_u32(part, lds);

    const uint64_t w64 = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t word = load_tile_word(bitmap, n_rows, n_words32, w64);
    const unsigned c = __popcll(word);

    // inclusive scan of c over the wave
    unsigned incl = c;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const unsigned up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) wave_total[wave] = incl;
    __syncthreads();
    unsigned before_wave = 0, block_total = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) {
        const unsigned t = wave_total[k];
        if (k < wave) before_wave += t;
        block_total += t;
    }
    const unsigned excl = before_wave + incl - c;  // dirty rows of this tile before my word

    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const uint64_t total = base + block_total;
        *n_dirty = total;
        if (total > capacity) raise_flag(err, CNR_FLAG_CAPACITY);
    }

    const uint32_t lo32 = (uint32_t)word, hi32 = (uint32_t)(word >> 32);
    const uint64_t wave_row0 = ((uint64_t)blockIdx.x * kBlock + (uint64_t)wave * kWave) * 64u;
    const uint64_t below_me = lane ? ((~0ull) >> (64 - lane)) : 0ull;
    for (int i = 0; i < kWave; ++i) {
        const uint64_t wi = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)lo32, i) |
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi32, i) << 32);
        if (wi == 0) continue;  // uniform over the wave
        const unsigned off_i = (unsigned)__builtin_amdgcn_readlane((int)excl, i);
        if ((wi >> lane) & 1ull) {
            const uint64_t pos = base + off_i + (unsigned)__popcll(wi & below_me);
            if (pos < capacity) row_ids[pos] = (uint32_t)(wave_row0 + (uint64_t)i * 64u + (uint64_t)lane);
        }
    }
}

extern "C" {

size_t cnr_mark_scratch_bytes(uint64_t n_rows) { return (size_t)(cnr_bitmap_words(n_rows) * 32u); }

cnr_status cnr_mark_touched(cnr_ctx *ctx, uint32_t *bitmap, uint64_t n_rows, const void *indices,
                            uint64_t n_indices, cnr_index_type type, void *scratch, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (type != CNR_IDX_I32 && type != CNR_IDX_I64) return CNR_E_INVALID;
    if (n_rows >= (1ull << 32)) return CNR_E_INVALID;
    if (n_indices == 0) return CNR_OK;
    if (!indices || (!bitmap && n_rows)) return CNR_E_INVALID;
    const uintptr_t align = type == CNR_IDX_I64 ? 8 : 4;
    if (((uintptr_t)indices % align) || ((uintptr_t)bitmap % 4) || ((uintptr_t)scratch % 16)) return CNR_E_ALIGN;
    hipStream_t s = as_stream(stream);
    // The flag-byte route pays a pass over n_rows bytes; below this stream length the atomics are
    // cheaper (about 16 G atomics/s against about 5 TB/s for the fold, plus one more launch).
    const bool bulk = scratch && n_rows && n_indices > n_rows / 256 + 65536;
    const unsigned grid = cnr_grid(ctx, n_indices, (uint64_t)kBlock * 4, 8);
    if (bulk) {
        uint8_t *flags = (uint8_t *)scratch;
        if (type == CNR_IDX_I64)
            hipLaunchKernelGGL(mark_flags_kernel<int64_t>, dim3(grid), dim3(kBlock), 0, s, flags, n_rows,
                               (const int64_t *)indices, n_indices, ctx->dev_err);
        else
            hipLaunchKernelGGL(mark_flags_kernel<int32_t>, dim3(grid), dim3(kBlock), 0, s, flags, n_rows,
                               (const int32_t *)indices, n_indices, ctx->dev_err);
        st = cnr_launch_status(ctx);
        if (st != CNR_OK) return st;
        const uint64_t words = cnr_bitmap_words(n_rows);
        hipLaunchKernelGGL(fold_flags_kernel, dim3(cnr_grid(ctx, words, kBlock, 8)), dim3(kBlock), 0, s, flags,
                           bitmap, words);
        return cnr_launch_status(ctx);
    }
    if (type == CNR_IDX_I64)
        hipLaunchKernelGGL(mark_kernel<int64_t>, dim3(grid), dim3(kBlock), 0, s, bitmap, n_rows,
                           (const int64_t *)indices, n_indices, ctx->dev_err);
    else
        hipLaunchKernelGGL(mark_kernel<int32_t>, dim3(grid), dim3(kBlock), 0, s, bitmap, n_rows,
                           (const int32_t *)indices, n_indices, ctx->dev_err);
    return cnr_launch_status(ctx);
}

cnr_status cnr_compact_dirty(cnr_ctx *ctx, const uint32_t *bitmap, uint64_t n_rows,
                             uint32_t *row_ids, uint64_t capacity, uint64_t *n_dirty_dev,
                             void *scratch, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (!n_dirty_dev || !scratch || n_rows >= (1ull << 32)) return CNR_E_INVALID;
    if ((!bitmap && n_rows) || (!row_ids && capacity)) return CNR_E_INVALID;
    if (((uintptr_t)bitmap % 4) || ((uintptr_t)row_ids % 4) || ((uintptr_t)n_dirty_dev % 8) ||
        ((uintptr_t)scratch % 8))
        return CNR_E_ALIGN;
    uint64_t blocks = (n_rows + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    if (blocks < 1) blocks = 1;  // an empty table still has to produce a zero count
    const uint64_t n_words32 = cnr_bitmap_words(n_rows);
    uint32_t *block_count = (uint32_t *)scratch;
    hipLaunchKernelGGL(compact_count_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, as_stream(stream),
                       bitmap, n_rows, n_words32, block_count);
    st = cnr_launch_status(ctx);
    if (st != CNR_OK) return st;
    hipLaunchKernelGGL(compact_scatter_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, as_stream(stream),
                       bitmap, n_rows, n_words32, block_count, row_ids, capacity, n_dirty_dev,
                       ctx->dev_err);
    return cnr_launch_status(ctx);
}

}  // extern "C"
