// Tracking bit-vector (Section 5.1.1) and its compaction into the incremental view (Section 5.1).
//
// Every kernel here takes a batch of tables (a GPU holds several embedding tables, Section 2.1, and
// a checkpoint covers all of them): a workgroup's y index selects the table, its x index the share
// of that table's work, so the tables of a batch run side by side in one launch.  The single-table
// entry points are batches of one.
#include "cnr_common.h"

#include <type_traits>

// Per-tile counts of cnr_compact_dirty_noalloc: a fixed array in the library's device image instead
// of a buffer from the caller.  Every GPU that loads the library holds its own copy at its own
// address.  In host code this name is only a handle for hipGetSymbolAddress, never a device address:
// kernels get the looked-up pointer (cnr_ctx::static_scratch) as an argument like any other scratch.
static __device__ __align__(256) uint32_t scratch[CNR_NOALLOC_SCRATCH_BYTES / sizeof(uint32_t)];

namespace {

struct TrackJob {
    uint32_t *bitmap;
    uint64_t n_rows;
    const void *idx;      // mark: look-up indices
    uint64_t n_idx;
    uint8_t *flags;       // mark, bulk route: the scratch (flag bytes or slabs), zero on entry and on exit
    uint32_t parts;       // mark, LDS slices: workgroups that share this table's stream = slabs to fold
    uint32_t *row_ids;    // compact
    uint64_t capacity;
    uint64_t *n_dirty;
    uint32_t *block_count;
};
struct TrackBatch {
    TrackJob job[CNR_MAX_BATCH];
    uint32_t grid_x;  // workgroups per table
};

__global__ void __launch_bounds__(kBlock) clear_kernel(const TrackBatch b) {
    const TrackJob &t = b.job[wg_y()];
    const uint64_t n = (t.n_rows + 31u) / 32u;
    const uint64_t stride = (uint64_t)b.grid_x * kBlock;
    for (uint64_t i = (uint64_t)wg_x() * kBlock + tid_x(); i < n; i += stride) t.bitmap[i] = 0u;
}

// ---------------------------------------------------------------------------------------------
// mark: one bit per looked-up row.
//
// The index stream is read once, coalesced (each lane one index per pass, four passes in flight).
// Hot rows repeat many times under a skewed lookup distribution, so the word is tested with a
// plain load first and the atomic OR is issued only for bits not yet seen as set: a stale zero
// merely costs a redundant OR, and bits never go back to zero while marking.
// ---------------------------------------------------------------------------------------------
template <typename IdxT>
__global__ void __launch_bounds__(kBlock) mark_kernel(const TrackBatch b, cnr_dev_errors *err) {
    const TrackJob &t = b.job[wg_y()];
    uint32_t *__restrict__ bitmap = t.bitmap;
    const IdxT *__restrict__ idx = static_cast<const IdxT *>(t.idx);
    const uint64_t n_rows = t.n_rows, n = t.n_idx;
    constexpr int kUnroll = 4;
    const uint64_t stride = (uint64_t)b.grid_x * kBlock;
    uint64_t i = (uint64_t)wg_x() * kBlock + tid_x();
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
    if (bad && (tid_x() & (kWave - 1)) == 0) atomicAdd(&err->n_bad_indices, (unsigned long long)bad);
}

// ---------------------------------------------------------------------------------------------
// mark, bulk variants: no device-scope atomics.  The first, for tables too large for the second.
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
// Most look-ups of a skewed stream repeat a row that the same compute unit has flagged already, and a
// scattered byte store is the expensive part (each one is a request of its own to the L2, about 17 ps
// of the whole chip's time).  So a workgroup keeps, in 128 KB of LDS, a direct-mapped table of the
// rows it has flagged lately: h = row * odd constant (a bijection on 32 bits), slot = high 16 bits of
// h, and the slot holds the low 16 bits, so slot and content together name exactly one row.  A
// look-up that finds its own row there is dropped, any other one takes the slot over and stores its
// flag byte.  A row found in the table has had its store issued (or about to be issued, in program
// order) by the lane that put it there, so nothing is ever lost; collisions only cost a repeated
// store.  The content 0xFFFF marks an empty slot; the one row in 65,536 whose own low bits are
// 0xFFFF bypasses the table.  One workgroup of kSeenThreads threads per compute unit (the table
// fills the LDS; two smaller tables per unit do worse, each sees half the repeats); the stream is
// read as 16-byte vectors.
constexpr int kSeenThreads = 1024;
constexpr uint32_t kSeenSlots = 65536;

template <typename IdxT>
__global__ void __launch_bounds__(kSeenThreads) mark_flags_kernel(const TrackBatch b, cnr_dev_errors *err) {
    constexpr int kVec = 16 / (int)sizeof(IdxT);
    typedef IdxT vec_t __attribute__((ext_vector_type(kVec)));
    constexpr int kUnroll = 4;
    __shared__ uint16_t seen[kSeenSlots];
    const TrackJob &t = b.job[wg_y()];
    uint8_t *__restrict__ flags = t.flags;
    const uint32_t n_rows = (uint32_t)t.n_rows;  // the host checks n_rows < 2^32
    const uint32_t tid = tid_x();
    for (uint32_t i = tid; i < kSeenSlots / 2; i += kSeenThreads) reinterpret_cast<uint32_t *>(seen)[i] = 0xFFFFFFFFu;
    __syncthreads();

    // the stream as [head][16-byte vectors][tail]: head and tail are fewer than kVec elements each
    const IdxT *idx = static_cast<const IdxT *>(t.idx);
    const uint64_t n = t.n_idx;
    uint64_t head = ((16u - (uint32_t)((uintptr_t)idx & 15u)) & 15u) / sizeof(IdxT);
    if (head > n) head = n;
    const vec_t *vecs = reinterpret_cast<const vec_t *>(idx + head);
    const uint64_t n_vec = (n - head) / kVec;
    const uint64_t tail = head + n_vec * kVec;

    unsigned bad = 0;
    auto look_up = [&](IdxT v) {
        bool valid = (uint32_t)v < n_rows;
        if constexpr (sizeof(IdxT) == 8) valid = valid && ((uint64_t)v >> 32) == 0;
        else valid = valid && v >= 0;
        if (!valid) {
            ++bad;
            return;
        }
        const uint32_t r = (uint32_t)v;
        const uint32_t h = r * 0x9E3779B1u;
        const uint32_t slot = h >> 16, low = h & 0xFFFFu;
        if (seen[slot] != low || low == 0xFFFFu) {
            seen[slot] = (uint16_t)low;
            flags[r] = 1;
        }
    };
    const uint64_t stride = (uint64_t)b.grid_x * kSeenThreads;
    for (uint64_t p = (uint64_t)wg_x() * kSeenThreads + tid; p < n_vec; p += stride * kUnroll) {
        vec_t v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t q = p + (uint64_t)u * stride;
            if (q < n_vec) v[u] = load_stream<vec_t>(vecs + q);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t q = p + (uint64_t)u * stride;
            if (q < n_vec) {
#pragma unroll
                for (int e = 0; e < kVec; ++e) look_up(v[u][e]);
            }
        }
    }
    if (wg_x() == 0) {
        if (tid < head) look_up(idx[tid]);
        else if (tid - head < n - tail) look_up(idx[tail + (tid - head)]);
    }
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off);
    if (bad && (tid & (kWave - 1)) == 0) atomicAdd(&err->n_bad_indices, (unsigned long long)bad);
}

// ---------------------------------------------------------------------------------------------
// mark, second bulk variant, for tables of up to a few tens of millions of rows: bitmap slices in LDS.
//
// A workgroup owns kSliceRows consecutive rows of one table as a bitmap in LDS (all 160 KB of a
// compute unit) and one part of the table's index stream (an eighth; down to a thirty-second for
// small tables, see slice_parts_max): it reads its share of the stream, sets the bits of the
// look-ups that fall into its rows with LDS atomics, and stores the slice to slab s (= its part of
// the stream) of the scratch buffer, partial bitmaps that fold_slabs_kernel ORs into the bitmap and
// zeroes again.  Nothing is scattered to memory; the price is that the W = ceil(n_rows / kSliceRows)
// workgroups of a team read the same part of the stream.  Workgroups are dealt to the eight XCDs in
// turn along x and the number of parts is a multiple of eight, so x & 7 names both the part (mod 8)
// and the XCD: a team shares its part of the stream through one L2 and memory is read once.
// ---------------------------------------------------------------------------------------------
constexpr int kSliceThreads = 1024;
constexpr uint32_t kSliceWords = 40960;
constexpr uint64_t kSliceRows = 32ull * kSliceWords;
constexpr uint32_t kStreamParts = 8;      // parts of a stream, at least
constexpr uint32_t kStreamPartsMax = 32;  // and at most, where the scratch has room for that many slabs
// The scratch of a table: one byte per row (eight slabs, or the flag bytes), and never less than 32
// slabs of one whole slice, so that a table of one or two slices, whose 8 or 16 workgroups would
// leave most of the chip idle, can be shared out over 32 or 16 parts of its stream instead.
constexpr uint64_t kScratchFloorBytes = (uint64_t)kStreamPartsMax * kSliceWords * 4u;
inline uint64_t mark_scratch_bytes(uint64_t n_rows) {
    const uint64_t words = cnr_bitmap_words(n_rows);
    const uint64_t per_row = words * 32u, slabs32 = words * 4u * kStreamPartsMax;
    const uint64_t floor = slabs32 < kScratchFloorBytes ? slabs32 : kScratchFloorBytes;
    return per_row > floor ? per_row : floor;
}
// The most parts (a multiple of eight) a table's scratch has slabs for.
inline uint32_t slice_parts_max(uint64_t n_rows) {
    const uint64_t words = cnr_bitmap_words(n_rows);
    if (words == 0) return kStreamParts;
    const uint64_t fit = (mark_scratch_bytes(n_rows) / (words * 4u)) & ~7ull;
    return (uint32_t)(fit > kStreamPartsMax ? kStreamPartsMax : fit < kStreamParts ? kStreamParts : fit);
}

template <typename IdxT>
__global__ void __launch_bounds__(kSliceThreads) mark_slices_kernel(const TrackBatch b, cnr_dev_errors *err) {
    constexpr int kVec = 16 / (int)sizeof(IdxT);
    typedef IdxT vec_t __attribute__((ext_vector_type(kVec)));
    constexpr int kUnroll = 4;
    __shared__ uint32_t bits[kSliceWords];
    const TrackJob &t = b.job[wg_y()];
    const uint32_t part = wg_x() % t.parts, w = wg_x() / t.parts;
    const uint32_t n_rows = (uint32_t)t.n_rows;
    const uint64_t first = (uint64_t)w * kSliceRows;
    if (first >= t.n_rows) return;  // the whole workgroup: tables of a batch differ in size
    const uint32_t lo = (uint32_t)first;
    const uint32_t span = n_rows - lo < kSliceRows ? n_rows - lo : (uint32_t)kSliceRows;
    const uint32_t tid = tid_x();
    for (uint32_t i = tid; i < kSliceWords; i += kSliceThreads) bits[i] = 0u;
    __syncthreads();

    // the stream as [head][16-byte vectors][tail]: head and tail are fewer than kVec elements each
    const IdxT *idx = static_cast<const IdxT *>(t.idx);
    const uint64_t n = t.n_idx;
    uint64_t head = ((16u - (uint32_t)((uintptr_t)idx & 15u)) & 15u) / sizeof(IdxT);
    if (head > n) head = n;
    const vec_t *vecs = reinterpret_cast<const vec_t *>(idx + head);
    const uint64_t n_vec = (n - head) / kVec;
    const uint64_t tail = head + n_vec * kVec;
    const uint64_t per_part = (n_vec + t.parts - 1u) / t.parts;
    const uint64_t v0 = part * per_part;
    const uint64_t v1 = v0 + per_part < n_vec ? v0 + per_part : n_vec;

    unsigned bad = 0;
    // COUNT: also count the indices outside the table (the team's first workgroup does, for its part
    // of the stream).  A look-up inside this slice is inside the table, so the bit needs no more
    // than the slice test.
    auto run = [&](auto count_tag) {
        constexpr bool COUNT = decltype(count_tag)::value;
        auto look_up = [&](IdxT v) {
            const uint32_t d = (uint32_t)v - lo;
            bool mine = d < span;
            if constexpr (sizeof(IdxT) == 8) mine = mine && ((uint64_t)v >> 32) == 0;
            if (mine)
                __hip_atomic_fetch_or(&bits[d >> 5], 1u << (d & 31u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if constexpr (COUNT) {
                bool valid = (uint32_t)v < n_rows;
                if constexpr (sizeof(IdxT) == 8) valid = valid && ((uint64_t)v >> 32) == 0;
                bad += valid ? 0u : 1u;
            }
        };
        for (uint64_t p = v0 + tid; p < v1; p += (uint64_t)kSliceThreads * kUnroll) {
            vec_t v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint64_t q = p + (uint64_t)u * kSliceThreads;
                if (q < v1) v[u] = vecs[q];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint64_t q = p + (uint64_t)u * kSliceThreads;
                if (q < v1) {
#pragma unroll
                    for (int e = 0; e < kVec; ++e) look_up(v[u][e]);
                }
            }
        }
        if (part == 0) {
            if (tid < head) look_up(idx[tid]);
            else if (tid - head < n - tail) look_up(idx[tail + (tid - head)]);
        }
    };
    if (w == 0) run(std::true_type{});
    else run(std::false_type{});
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off);
    if (bad && (tid & (kWave - 1)) == 0) atomicAdd(&err->n_bad_indices, (unsigned long long)bad);
    __syncthreads();

    const uint64_t n_words = (t.n_rows + 31u) / 32u;
    uint32_t *slab = reinterpret_cast<uint32_t *>(t.flags) + part * n_words + (uint64_t)w * kSliceWords;
    const uint32_t words = (span + 31u) / 32u;
    for (uint32_t i = tid; i < words; i += kSliceThreads) slab[i] = bits[i];
}

// bitmap |= OR of the table's slabs; the slabs are left all zero.
__global__ void __launch_bounds__(kBlock) fold_slabs_kernel(const TrackBatch b) {
    const TrackJob &t = b.job[wg_y()];
    uint32_t *__restrict__ slabs = reinterpret_cast<uint32_t *>(t.flags);
    uint32_t *__restrict__ bitmap = t.bitmap;
    const uint64_t n_words = (t.n_rows + 31u) / 32u;
    const uint64_t stride = (uint64_t)b.grid_x * kBlock;
    for (uint64_t i = (uint64_t)wg_x() * kBlock + tid_x(); i < n_words; i += stride) {
        uint32_t acc = 0;
        for (uint32_t s = 0; s < t.parts; ++s) {
            acc |= slabs[s * n_words + i];
            slabs[s * n_words + i] = 0u;
        }
        if (acc) bitmap[i] |= acc;
    }
}

// Eight flag bytes (each 0 or 1) to eight bits, first byte in bit 0.
__device__ __forceinline__ uint32_t flags_to_bits(uint64_t eight) {
    return (uint32_t)((eight * 0x0102040810204080ull) >> 56);
}

__global__ void __launch_bounds__(kBlock) fold_flags_kernel(const TrackBatch b) {
    const TrackJob &t = b.job[wg_y()];
    uint8_t *__restrict__ flags = t.flags;
    uint32_t *__restrict__ bitmap = t.bitmap;
    const uint64_t n_words = (t.n_rows + 31u) / 32u;
    const uint64_t stride = (uint64_t)b.grid_x * kBlock;
    for (uint64_t w = (uint64_t)wg_x() * kBlock + tid_x(); w < n_words; w += stride) {
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
//            one LDS step across the four waves), then every lane walks the set bits of its own
//            word and writes their row numbers, as 16-bit offsets from the tile's first row, to its
//            place in an LDS copy of the tile's part of the list, which the workgroup then stores
//            to the list with every lane writing consecutive ids.
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
    const int wave = tid_x() / kWave;
    __syncthreads();
    if ((tid_x() & (kWave - 1)) == 0) lds[wave] = v;
    __syncthreads();
    unsigned t = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
    return t;
}

// Tiles of one table; an empty table still has one, so that its count is written.
__device__ __forceinline__ uint64_t compact_tiles(uint64_t n_rows) {
    const uint64_t tiles = (n_rows + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    return tiles ? tiles : 1;
}

__global__ void __launch_bounds__(kBlock) compact_count_kernel(const TrackBatch b) {
    __shared__ unsigned lds[kWavesPerBlock];
    const TrackJob &t = b.job[wg_y()];
    const uint64_t n_rows = t.n_rows, n_words32 = (n_rows + 31u) / 32u;
    if (wg_x() >= compact_tiles(n_rows)) return;  // uniform over the workgroup
    const uint32_t *__restrict__ bitmap = t.bitmap;
    uint32_t *__restrict__ block_count = t.block_count;
    const uint64_t w64 = (uint64_t)wg_x() * kBlock + tid_x();
    const unsigned c = __popcll(load_tile_word(bitmap, n_rows, n_words32, w64));
    const unsigned total = block_sum_u32(c, lds);
    if (tid_x() == 0) block_count[wg_x()] = total;
}

__global__ void __launch_bounds__(kBlock) compact_scatter_kernel(const TrackBatch b, cnr_dev_errors *err) {
    __shared__ unsigned lds[kWavesPerBlock];
    __shared__ unsigned wave_total[kWavesPerBlock];
    __shared__ uint16_t tile_ids[kCompactRowsPerBlock];
    const TrackJob &t = b.job[wg_y()];
    const uint64_t n_rows = t.n_rows, n_words32 = (n_rows + 31u) / 32u, capacity = t.capacity;
    const uint64_t tiles = compact_tiles(n_rows);
    if (wg_x() >= tiles) return;  // uniform over the workgroup
    const uint32_t *__restrict__ bitmap = t.bitmap;
    const uint32_t *__restrict__ block_count = t.block_count;
    uint32_t *__restrict__ row_ids = t.row_ids;
    uint64_t *__restrict__ n_dirty = t.n_dirty;
    const int lane = tid_x() & (kWave - 1);
    const int wave = tid_x() / kWave;

    // dirty rows in all earlier tiles
    unsigned part = 0;
    for (unsigned b = tid_x(); b < wg_x(); b += kBlock) part += block_count[b];
    const uint64_t base = block_sum_u32(part, lds);

    const uint64_t w64 = (uint64_t)wg_x() * kBlock + tid_x();
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

    if (wg_x() == tiles - 1 && tid_x() == 0) {
        const uint64_t total = base + block_total;
        *n_dirty = total;
        if (total > capacity) raise_flag(err, CNR_FLAG_CAPACITY);
    }

    // ids of the tile in ascending order, as 16-bit offsets from its first row, into LDS: every lane
    // walks the set bits of its own word ...
    {
        uint64_t rest = word;
        unsigned k = excl;
        const uint32_t off0 = tid_x() * 64u;
        while (rest) {
            tile_ids[k++] = (uint16_t)(off0 + (uint32_t)__builtin_ctzll(rest));
            rest &= rest - 1;
        }
    }
    __syncthreads();
    // ... and from there to the list, every lane storing
    const uint64_t tile_row0 = (uint64_t)wg_x() * kCompactRowsPerBlock;
    for (unsigned p = tid_x(); p < block_total; p += kBlock) {
        const uint64_t pos = base + p;
        if (pos < capacity) row_ids[pos] = (uint32_t)(tile_row0 + tile_ids[p]);
    }
}

// Workgroups per table for a grid-stride kernel over a batch: enough for the largest share of work,
// at most an equal part of `blocks_per_cu` workgroups per compute unit.
unsigned batch_grid_x(const cnr_ctx *ctx, uint64_t max_items, uint64_t per_block, unsigned blocks_per_cu,
                      uint32_t n_jobs) {
    uint64_t need = (max_items + per_block - 1) / per_block;
    uint64_t cap = (uint64_t)ctx->n_cu * blocks_per_cu / n_jobs;
    if (cap < 1) cap = 1;
    if (need < 1) need = 1;
    return (unsigned)(need < cap ? need : cap);
}

cnr_status check_tracked_table(const cnr_table_job &j) {
    if (j.n_rows >= (1ull << 32)) return CNR_E_INVALID;
    if (!j.bitmap && j.n_rows) return CNR_E_INVALID;
    if ((uintptr_t)j.bitmap % 4) return CNR_E_ALIGN;
    return CNR_OK;
}

}  // namespace

extern "C" {

size_t cnr_mark_scratch_bytes(uint64_t n_rows) { return (size_t)mark_scratch_bytes(n_rows); }

cnr_status cnr_clear_bitmap_batch(cnr_ctx *ctx, const cnr_table_job *jobs, uint32_t n_jobs, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (n_jobs && !jobs) return CNR_E_INVALID;
    for (uint32_t i = 0; i < n_jobs; ++i)
        if ((st = check_tracked_table(jobs[i])) != CNR_OK) return st;
    for (uint32_t first = 0; first < n_jobs; first += CNR_MAX_BATCH) {
        TrackBatch b = {};
        uint32_t n = 0;
        uint64_t max_words = 0;
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i) {
            if (jobs[i].n_rows == 0) continue;
            b.job[n].bitmap = jobs[i].bitmap;
            b.job[n].n_rows = jobs[i].n_rows;
            const uint64_t words = cnr_bitmap_words(jobs[i].n_rows);
            if (words > max_words) max_words = words;
            ++n;
        }
        if (n == 0) continue;
        b.grid_x = batch_grid_x(ctx, max_words, kBlock * 4, 4, n);
        hipLaunchKernelGGL(clear_kernel, dim3(b.grid_x, n), dim3(kBlock), 0, as_stream(stream), b);
        if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
    }
    return CNR_OK;
}

cnr_status cnr_clear_bitmap(cnr_ctx *ctx, uint32_t *bitmap, uint64_t n_rows, void *stream) {
    cnr_table_job j = {};
    j.bitmap = bitmap;
    j.n_rows = n_rows;
    return cnr_clear_bitmap_batch(ctx, &j, 1, stream);
}

cnr_status cnr_mark_touched_batch(cnr_ctx *ctx, const cnr_table_job *jobs, uint32_t n_jobs,
                                  cnr_index_type type, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (type != CNR_IDX_I32 && type != CNR_IDX_I64) return CNR_E_INVALID;
    if (n_jobs && !jobs) return CNR_E_INVALID;
    const uintptr_t align = type == CNR_IDX_I64 ? 8 : 4;
    for (uint32_t i = 0; i < n_jobs; ++i) {
        const cnr_table_job &j = jobs[i];
        if (j.n_rows >= (1ull << 32)) return CNR_E_INVALID;
        if (j.n_indices == 0) continue;
        if (!j.indices || (!j.bitmap && j.n_rows)) return CNR_E_INVALID;
        if (((uintptr_t)j.indices % align) || ((uintptr_t)j.bitmap % 4) || ((uintptr_t)j.mark_scratch % 16))
            return CNR_E_ALIGN;
    }
    hipStream_t s = as_stream(stream);
    for (uint32_t first = 0; first < n_jobs; first += CNR_MAX_BATCH) {
        // Three routes.  Short streams: atomic ORs on the bitmap (about 16 G atomics/s; the other two
        // pay a pass over n_rows bytes).  Long streams: bitmap slices in LDS, or one flag byte per row
        // and a fold.  The slices cost every workgroup of a table its part of the stream (an eighth or
        // less, at the 60 GB/s a workgroup of that kernel gets through it), whatever the stream holds, and
        // all tables of a call run side by side as long as their workgroups fit the chip; the flag bytes cost
        // one scattered store per look-up that gets past the table of lately flagged rows (about 17 ps
        // of the whole chip's time each, a third of the look-ups on the skewed streams that embedding
        // look-ups are), one table after the other.  So one or two tables marked alone are faster
        // through flag bytes (a 5 M-row table, 20 M Zipf look-ups: 67-121 against 250-445 us) and a
        // batch of many tables through slices (8 x 5 M rows, 3 M look-ups each: 89 against 385 us); the
        // call takes, for all its tables of up to kSliceTeamMax slices together, the route this
        // estimate makes the cheaper one.  Larger tables always take the flag bytes.
        constexpr uint64_t kSliceTeamMax = 16;
        constexpr double kSlicePsPerByte = 1e12 / 60e9;                  // a workgroup gets through its part of the stream at 60 GB/s
        constexpr double kFlagPsPerLookup = 6.0;                         // 17 ps x about a third that become stores
        uint64_t elig_teams = 0, elig_sum_idx = 0;
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i) {
            const cnr_table_job &j = jobs[i];
            const uint64_t team = (j.n_rows + kSliceRows - 1) / kSliceRows;
            if (j.n_indices == 0 || !(j.mark_scratch && j.n_rows && j.n_indices > j.n_rows / 256 + 65536) || team > kSliceTeamMax)
                continue;
            elig_teams += team;
            elig_sum_idx += j.n_indices;
        }
        // Parts per stream: eight, or as many more (in eights, as far as a table's scratch has slabs) as
        // it takes for the workgroups of the call to fill the chip.
        uint32_t want_parts = kStreamParts;
        if (elig_teams) {
            const uint64_t fill = (((uint64_t)ctx->n_cu + elig_teams - 1) / elig_teams + 7u) & ~7ull;
            want_parts = (uint32_t)(fill < kStreamParts ? kStreamParts : fill > kStreamPartsMax ? kStreamPartsMax : fill);
        }
        uint64_t elig_wgs = 0;
        double elig_longest = 0;  // the longest part of a stream a workgroup reads, in look-ups
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i) {
            const cnr_table_job &j = jobs[i];
            const uint64_t team = (j.n_rows + kSliceRows - 1) / kSliceRows;
            if (j.n_indices == 0 || !(j.mark_scratch && j.n_rows && j.n_indices > j.n_rows / 256 + 65536) || team > kSliceTeamMax)
                continue;
            const uint32_t most = slice_parts_max(j.n_rows);
            const uint32_t parts = want_parts < most ? want_parts : most;
            elig_wgs += team * parts;
            if ((double)j.n_indices / parts > elig_longest) elig_longest = (double)j.n_indices / parts;
        }
        const uint64_t rounds = (elig_wgs + (uint64_t)ctx->n_cu - 1) / (uint64_t)ctx->n_cu;
        const bool slices_pay = elig_longest * (type == CNR_IDX_I64 ? 8.0 : 4.0) * kSlicePsPerByte * (double)rounds <
                                (double)elig_sum_idx * kFlagPsPerLookup;
        TrackBatch slices = {}, bulk = {}, direct = {};
        uint32_t n_slices = 0, n_bulk = 0, n_direct = 0;
        uint64_t slices_words = 0, slices_team = 0, bulk_idx = 0, bulk_words = 0, direct_idx = 0;
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i) {
            const cnr_table_job &j = jobs[i];
            if (j.n_indices == 0) continue;
            const bool long_stream = j.mark_scratch && j.n_rows && j.n_indices > j.n_rows / 256 + 65536;
            const uint64_t team = (j.n_rows + kSliceRows - 1) / kSliceRows;
            const bool use_slices = long_stream && team <= kSliceTeamMax && slices_pay;
            TrackJob &t = use_slices ? slices.job[n_slices++] : long_stream ? bulk.job[n_bulk++] : direct.job[n_direct++];
            t.bitmap = j.bitmap;
            t.n_rows = j.n_rows;
            t.idx = j.indices;
            t.n_idx = j.n_indices;
            t.flags = (uint8_t *)j.mark_scratch;
            const uint64_t words = cnr_bitmap_words(j.n_rows);
            if (use_slices) {
                const uint32_t most = slice_parts_max(j.n_rows);
                t.parts = want_parts < most ? want_parts : most;
                if (team * t.parts > slices_team) slices_team = team * t.parts;
                if (words > slices_words) slices_words = words;
            } else if (long_stream) {
                if (j.n_indices > bulk_idx) bulk_idx = j.n_indices;
                if (words > bulk_words) bulk_words = words;
            } else if (j.n_indices > direct_idx) {
                direct_idx = j.n_indices;
            }
        }
        if (n_slices) {
            const dim3 grid((unsigned)slices_team, n_slices);  // the most workgroups any table of the launch has
            if (type == CNR_IDX_I64)
                hipLaunchKernelGGL(mark_slices_kernel<int64_t>, grid, dim3(kSliceThreads), 0, s, slices, ctx->dev_err);
            else
                hipLaunchKernelGGL(mark_slices_kernel<int32_t>, grid, dim3(kSliceThreads), 0, s, slices, ctx->dev_err);
            if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
            slices.grid_x = batch_grid_x(ctx, slices_words, kBlock, 8, n_slices);
            hipLaunchKernelGGL(fold_slabs_kernel, dim3(slices.grid_x, n_slices), dim3(kBlock), 0, s, slices);
            if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
        }
        if (n_bulk) {
            // one workgroup per compute unit in all (each fills a unit's LDS), shared out over the tables
            bulk.grid_x = batch_grid_x(ctx, bulk_idx, (uint64_t)kSeenThreads * 8, 1, n_bulk);
            const dim3 grid(bulk.grid_x, n_bulk);
            if (type == CNR_IDX_I64)
                hipLaunchKernelGGL(mark_flags_kernel<int64_t>, grid, dim3(kSeenThreads), 0, s, bulk, ctx->dev_err);
            else
                hipLaunchKernelGGL(mark_flags_kernel<int32_t>, grid, dim3(kSeenThreads), 0, s, bulk, ctx->dev_err);
            if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
            bulk.grid_x = batch_grid_x(ctx, bulk_words, kBlock, 8, n_bulk);
            hipLaunchKernelGGL(fold_flags_kernel, dim3(bulk.grid_x, n_bulk), dim3(kBlock), 0, s, bulk);
            if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
        }
        if (n_direct) {
            direct.grid_x = batch_grid_x(ctx, direct_idx, (uint64_t)kBlock * 4, 8, n_direct);
            const dim3 grid(direct.grid_x, n_direct);
            if (type == CNR_IDX_I64)
                hipLaunchKernelGGL(mark_kernel<int64_t>, grid, dim3(kBlock), 0, s, direct, ctx->dev_err);
            else
                hipLaunchKernelGGL(mark_kernel<int32_t>, grid, dim3(kBlock), 0, s, direct, ctx->dev_err);
            if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
        }
    }
    return CNR_OK;
}

cnr_status cnr_mark_touched(cnr_ctx *ctx, uint32_t *bitmap, uint64_t n_rows, const void *indices,
                            uint64_t n_indices, cnr_index_type type, void *scratch, void *stream) {
    cnr_table_job j = {};
    j.bitmap = bitmap;
    j.n_rows = n_rows;
    j.indices = indices;
    j.n_indices = n_indices;
    j.mark_scratch = scratch;
    return cnr_mark_touched_batch(ctx, &j, 1, type, stream);
}

cnr_status cnr_compact_dirty_batch(cnr_ctx *ctx, const cnr_table_job *jobs, uint32_t n_jobs, void *stream) {
    cnr_status st = cnr_enter(ctx);
    if (st != CNR_OK) return st;
    if (n_jobs && !jobs) return CNR_E_INVALID;
    for (uint32_t i = 0; i < n_jobs; ++i) {
        const cnr_table_job &j = jobs[i];
        if (!j.n_dirty_dev || !j.compact_scratch || j.n_rows >= (1ull << 32)) return CNR_E_INVALID;
        if ((!j.bitmap && j.n_rows) || (!j.row_ids && j.capacity)) return CNR_E_INVALID;
        if (((uintptr_t)j.bitmap % 4) || ((uintptr_t)j.row_ids % 4) || ((uintptr_t)j.n_dirty_dev % 8) ||
            ((uintptr_t)j.compact_scratch % 8))
            return CNR_E_ALIGN;
    }
    for (uint32_t first = 0; first < n_jobs; first += CNR_MAX_BATCH) {
        TrackBatch b = {};
        uint32_t n = 0;
        uint64_t max_tiles = 1;
        for (uint32_t i = first; i < n_jobs && i < first + CNR_MAX_BATCH; ++i, ++n) {
            const cnr_table_job &j = jobs[i];
            b.job[n].bitmap = j.bitmap;
            b.job[n].n_rows = j.n_rows;
            b.job[n].row_ids = j.row_ids;
            b.job[n].capacity = j.capacity;
            b.job[n].n_dirty = j.n_dirty_dev;
            b.job[n].block_count = (uint32_t *)j.compact_scratch;
            const uint64_t tiles = (j.n_rows + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
            if (tiles > max_tiles) max_tiles = tiles;
        }
        b.grid_x = (uint32_t)max_tiles;
        const dim3 grid(b.grid_x, n);
        hipLaunchKernelGGL(compact_count_kernel, grid, dim3(kBlock), 0, as_stream(stream), b);
        if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
        hipLaunchKernelGGL(compact_scatter_kernel, grid, dim3(kBlock), 0, as_stream(stream), b, ctx->dev_err);
        if ((st = cnr_launch_status(ctx)) != CNR_OK) return st;
    }
    return CNR_OK;
}

cnr_status cnr_compact_dirty(cnr_ctx *ctx, const uint32_t *bitmap, uint64_t n_rows,
                             uint32_t *row_ids, uint64_t capacity, uint64_t *n_dirty_dev,
                             void *scratch, void *stream) {
    cnr_table_job j = {};
    j.bitmap = const_cast<uint32_t *>(bitmap);
    j.n_rows = n_rows;
    j.row_ids = row_ids;
    j.capacity = capacity;
    j.n_dirty_dev = n_dirty_dev;
    j.compact_scratch = scratch;
    return cnr_compact_dirty_batch(ctx, &j, 1, stream);
}

cnr_status cnr_compact_dirty_noalloc(cnr_ctx *ctx, const uint32_t *bitmap, uint64_t n_rows,
                                     uint32_t *row_ids, uint64_t capacity, uint64_t *n_dirty_dev,
                                     void *stream) {
    if (!ctx) return CNR_E_INVALID;
    if (n_rows > CNR_NOALLOC_MAX_ROWS) return CNR_E_TOO_LARGE;
    static_assert(CNR_NOALLOC_SCRATCH_BYTES >= (CNR_NOALLOC_MAX_ROWS / kCompactRowsPerBlock) * sizeof(uint32_t) + 8u,
                  "the fixed scratch holds one count per tile of the largest table");
    if (!ctx->static_scratch || cnr_scratch_bytes(n_rows) > CNR_NOALLOC_SCRATCH_BYTES) return CNR_E_INVALID;
    // from here on the plain call with this device's array as its scratch: argument checks and two
    // kernel launches, no allocation
    return cnr_compact_dirty(ctx, bitmap, n_rows, row_ids, capacity, n_dirty_dev, ctx->static_scratch, stream);
}

}  // extern "C"

cnr_status cnr_bind_static_scratch(cnr_ctx *ctx) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return cnr_hip_status(ctx, e);
    if (!p) return cnr_hip_status(ctx, hipErrorInvalidSymbol);
    ctx->static_scratch = p;
    return CNR_OK;
}
