// Internal declarations shared by the translation units of libcnr (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cnr.h"

// Counters the kernels update when they meet a condition they must not fault on.
struct cnr_dev_errors {
    unsigned long long n_bad_indices;  // look-up indices outside the table (mark)
    unsigned int flags;                // CNR_FLAG_*
    unsigned int pad;
};

struct cnr_ctx {
    int device;
    int n_cu;                  // compute units of the device
    cnr_dev_errors *dev_err;   // device
    cnr_dev_errors *host_err;  // pinned host mirror used by cnr_poll_errors
    double *host_scalar;       // pinned host double (behind host_err) for results read back one at a time
    void *static_scratch;      // this device's copy of the library's fixed compaction scratch
    int last_hip_error;
};

constexpr int kWave = 64;
constexpr int kBlock = 256;                    // threads per workgroup everywhere
constexpr int kWavesPerBlock = kBlock / kWave;

// Rows of the bitmap one compact workgroup covers: one 64-bit bitmap word per thread.
constexpr uint64_t kCompactRowsPerBlock = (uint64_t)kBlock * 64u;

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Makes ctx's device current; returns CNR_OK or CNR_E_HIP.
cnr_status cnr_enter(cnr_ctx *ctx);
// Records a HIP failure in the context and maps it to a status.
cnr_status cnr_hip_status(cnr_ctx *ctx, hipError_t e);
// Looks up, on ctx's device (which must be current), the address of the fixed scratch array that
// cnr_compact_dirty_noalloc uses, and keeps it in the context.
cnr_status cnr_bind_static_scratch(cnr_ctx *ctx);
// Status of the launch that was just enqueued.
static inline cnr_status cnr_launch_status(cnr_ctx *ctx) { return cnr_hip_status(ctx, hipGetLastError()); }

static inline bool cnr_valid_bits(int bits) { return bits == 2 || bits == 3 || bits == 4 || bits == 8; }

// Number of workgroups for `work_items` items at `per_block` items per workgroup pass, capped so
// that a grid-stride loop keeps every compute unit busy without oversubscribing the dispatcher.
static inline unsigned cnr_grid(const cnr_ctx *ctx, uint64_t work_items, uint64_t per_block,
                                unsigned blocks_per_cu) {
    uint64_t need = (work_items + per_block - 1) / per_block;
    uint64_t cap = (uint64_t)ctx->n_cu * blocks_per_cu;
    if (need < 1) need = 1;
    return (unsigned)(need < cap ? need : cap);
}

// A table whose rows (at capacity) come to no more than this many bytes counts as small: in a batch
// it shares a launch with the other small tables instead of taking one of its own.
constexpr uint64_t kSideBySideBytes = 64ull << 20;

// Rows per launch for a list whose length the host knows (no count on the device).  The waves of a
// long encode or restore launch drift apart and stop sweeping one region of the table together;
// slices of about 512 MB of table rows keep them together (3 to 5 % faster on lists of several
// million rows).  A multiple of 1024 rows, so that every slice starts as aligned as the buffers do.
static inline uint64_t cnr_slice_rows(uint64_t n, uint32_t dim) {
    uint64_t target = ((512ull << 20) / (4ull * dim)) & ~1023ull;
    if (target < 1024) target = 1024;
    if (n <= target + target / 2) return n ? n : 1;
    const uint64_t n_slices = (n + target - 1) / target;
    const uint64_t per = (n + n_slices - 1) / n_slices;
    return (per + 1023u) & ~1023ull;
}

// Workgroups for the bandwidth-bound row kernels (tile encode, restore): many more than are resident
// at once.  The hardware hands workgroups out in order as others finish, which keeps all waves on
// one front that moves through the table however unevenly they progress; a grid of exactly the
// resident workgroups, each striding through the whole list, lets them drift apart (measured on
// 1.5 M rows of 64 floats: encode 80 -> 76 us, restore 98 -> 83 us; more on longer lists).  The row
// count is only known on the device, so the grid follows n_max and is capped: workgroups beyond
// the count leave at once, and 24 K of them cost about 4 us.  (Caps from 16 K to 32 K are within a
// few per cent of each other from 5 % to 100 % of a 5 M-row table; 64 K and more lose on short lists.)
constexpr uint64_t kRowKernelMaxBlocks = 24576;
static inline unsigned cnr_row_grid(uint64_t n_max, uint64_t rows_per_block) {
    uint64_t need = (n_max + rows_per_block - 1) / rows_per_block;
    if (need < 1) need = 1;
    return (unsigned)(need < kRowKernelMaxBlocks ? need : kRowKernelMaxBlocks);
}

#ifdef __HIPCC__
// Workgroups of `Kernel` (kBlock threads, no dynamic LDS) that fit on one compute unit at once, at
// most 8.  A persistent (grid-stride) kernel launched with more workgroups than are resident runs
// them in rounds and leaves the last round under-filled, so grids are sized to exactly one round.
// (A second, partial round is what hurts; the row kernels go far beyond it, see cnr_row_grid.)
template <auto Kernel>
static inline unsigned cnr_resident_blocks_per_cu() {
    static int cached = 0;
    if (cached == 0) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, Kernel, kBlock, 0) != hipSuccess || nb < 1) nb = 4;
        cached = nb > 8 ? 8 : nb;
    }
    return (unsigned)cached;
}

// Streaming accesses: data that is touched once (gathered rows, encoded output, restored rows)
// carries the non-temporal hint so that it does not linger in L2 until the end of the kernel.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename T>
__device__ __forceinline__ void store_stream(void *p, T v) {
    __builtin_nontemporal_store(v, reinterpret_cast<T *>(p));
}
// A 16-byte streaming store that is also written through to memory at once (system scope) instead
// of waiting in the L2 as a dirty line until it is evicted: memory then sees the rows in the order
// the kernel sweeps the table.  Pays only where one instruction writes a whole row (measured, restore
// of rows of up to 64 floats at up to 4 bits: 1.5 to 2 % faster; rows written in several pieces are
// better left to the L2, which gathers the pieces: rows of 256 floats lose 19 % with it).  No builtin
// gives this combination of cache bits, hence the assembly; the two idle states behind it are what
// the hardware asks for before the store's data registers may be overwritten.
__device__ __forceinline__ void store_stream_through(void *p, f32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
template <typename T>
__device__ __forceinline__ T load_stream(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const T *>(p));
}

// ---- cross-lane helpers (wave64) -------------------------------------------------------------
// DPP controls: quad_perm [1,0,3,2] = 0xB1 (lane ^ 1), quad_perm [2,3,0,1] = 0x4E (lane ^ 2),
// row_half_mirror = 0x141 (lane i <-> 7 - i within 8), row_mirror = 0x140 (i <-> 15 - i within 16).
// After those four exchanges, applied in that order with a commutative and associative combine,
// all 16 lanes of a DPP row hold the combination of the row's 16 values.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(dpp_i<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    int lo = dpp_i<CTRL>(__double2loint(v));
    int hi = dpp_i<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float row16_min(float v) {
    v = fminf(v, dpp_f<0xB1>(v));
    v = fminf(v, dpp_f<0x4E>(v));
    v = fminf(v, dpp_f<0x141>(v));
    v = fminf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ double row16_sum(double v) {
    v += dpp_d<0xB1>(v);
    v += dpp_d<0x4E>(v);
    v += dpp_d<0x141>(v);
    v += dpp_d<0x140>(v);
    return v;
}

// Launch coordinates read from the hardware registers: the workgroup id arrives in a scalar
// register, so everything derived from it stays out of the vector registers.
__device__ __forceinline__ uint32_t wg_x() { return __builtin_amdgcn_workgroup_id_x(); }
__device__ __forceinline__ uint32_t wg_y() { return __builtin_amdgcn_workgroup_id_y(); }
__device__ __forceinline__ uint32_t tid_x() { return __builtin_amdgcn_workitem_id_x(); }
// Workgroups along x of a grid of kBlock-thread workgroups.
__device__ __forceinline__ uint32_t grid_x() { return __builtin_amdgcn_grid_size_x() / (uint32_t)kBlock; }
// Index of this wave in a one-dimensional grid of kBlock-thread workgroups, in a scalar register.
__device__ __forceinline__ uint32_t wave_in_grid() {
    return wg_x() * kWavesPerBlock + (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid_x() / kWave));
}

// min(*n_dev, n_max) (n_max when n_dev is NULL), in scalar registers: the number of rows a kernel
// works on when the count is only known on the device.
__device__ __forceinline__ uint64_t live_rows(const uint64_t *n_dev, uint64_t n_max) {
    uint64_t n = n_max;
    if (n_dev) {
        const uint64_t nd = *n_dev;
        n = nd < n_max ? nd : n_max;
    }
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)n);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(n >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ void raise_flag(cnr_dev_errors *err, unsigned flag) {
    atomicOr(&err->flags, flag);
}
#endif
