// Ceilings of the machine that the rooflines of bench.py are read against, measured with plain kernels:
//
//   1. how long a wave's vector instruction occupies a SIMD on gfx950, per kind of instruction: the
//      figures behind the instruction-issue bound quoted for the greedy range search (Section 5.2,
//      Approach 3), whose inner loop is pure vector arithmetic.  Every kernel runs one kind of
//      instruction over 32 independent registers per lane (16 for fp64), so that nothing waits for an
//      earlier result, with 8 waves per SIMD on all 256 compute units.  Inline assembly pins the
//      instruction; every operand is a register the kernel owns.
//   2. what the memory system sustains for the access patterns of the encode and the restore
//      (Sections 5.1, 5.2): rows of 256 bytes, 30 % of a 20 M-row table in ascending order, gathered
//      (read only) and scattered (written only) with the kernels' lane mapping (16 lanes per row, 16
//      bytes per lane), and rows of 512 bytes, 25 % of 10 M, next to a sequential read, write and
//      copy of the same table.
//   4. what one compute unit streams from the L2 of its XCD (the bound of the bulk mark through bitmap
//      slices, Section 5.1.1).
//   3. what the host link sustains for 64 MiB of pinned host memory (the size of one table's
//      incremental checkpoint, Sections 4.4 and 5.1): read and written by a kernel directly, and
//      moved by the runtime's asynchronous copies.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 bench_ceilings.hip -o bench_ceilings && ./bench_ceilings
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <vector>

#define OP1(op, d, s) asm volatile(op " %0, %1" : "=v"(d) : "v"(s))
#define OP2(op, d, s, t) asm volatile(op " %0, %1, %2" : "=v"(d) : "v"(s), "v"(t))
#define OP3(op, d, s, t, u) asm volatile(op " %0, %1, %2, %3" : "=v"(d) : "v"(s), "v"(t), "v"(u))

enum Kind { ADD, SUB, MUL, FMA, MED3, RNDNE, CVT_F64_F32, FMA_F64, ADD_F64, GREEDY_MIX };

template <int KIND>
__global__ void __launch_bounds__(256) rate_kernel(float x, double xd, int iters, float *out) {
    float a[32];
    double b[16];
    for (int i = 0; i < 32; ++i) a[i] = threadIdx.x * 1e-3f + i;
    for (int i = 0; i < 16; ++i) b[i] = threadIdx.x * 1e-3 + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if (KIND == ADD) OP2("v_add_f32_e32", a[i], a[i], x);
            if (KIND == SUB) OP2("v_sub_f32_e32", a[i], a[i], x);
            if (KIND == MUL) OP2("v_mul_f32_e32", a[i], a[i], x);
            if (KIND == FMA) OP3("v_fma_f32", a[i], a[i], x, x);
            if (KIND == MED3) OP3("v_med3_f32", a[i], a[i], x, x);
            if (KIND == RNDNE) OP1("v_rndne_f32_e32", a[i], a[i]);
            if (KIND == CVT_F64_F32) OP1("v_cvt_f64_f32_e32", b[i % 16], a[i]);
            if (KIND == FMA_F64) OP3("v_fma_f64", b[i % 16], b[i % 16], xd, xd);
            if (KIND == ADD_F64) OP2("v_add_f64", b[i % 16], b[i % 16], xd);
            if (KIND == GREEDY_MIX && i < 8) {
                // one element of the greedy loop: clip, subtract, multiply, round, multiply, add, subtract,
                // convert, accumulate the square (9 instructions)
                float c, d;
                double dd;
                OP3("v_med3_f32", c, a[i], x, a[i + 8]);
                OP2("v_sub_f32_e32", c, c, x);
                OP2("v_mul_f32_e32", c, c, a[i + 16]);
                OP1("v_rndne_f32_e32", c, c);
                OP2("v_mul_f32_e32", c, c, a[i + 24]);
                OP2("v_add_f32_e32", c, c, x);
                OP2("v_sub_f32_e32", d, a[i], c);
                OP1("v_cvt_f64_f32_e32", dd, d);
                OP3("v_fma_f64", b[i], dd, dd, b[i]);
            }
        }
    }
    float s = 0;
    for (int i = 0; i < 32; ++i) s += a[i];
    for (int i = 0; i < 16; ++i) s += (float)b[i];
    if (s == 123.456f) out[0] = s;  // keeps the registers alive; never true in practice
}

template <int KIND>
static int run(const char *name, int per_trip, float *out) {
    const int iters = 4000, waves_per_simd = 8;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
    const int grid = 256 * waves_per_simd;  // workgroups of 4 waves: waves_per_simd waves on every SIMD
    rate_kernel<KIND><<<grid, 256>>>(1.0001f, 1.0001, 16, out);
    if (hipEventRecord(e0) != hipSuccess) return 1;
    rate_kernel<KIND><<<grid, 256>>>(1.0001f, 1.0001, iters, out);
    if (hipEventRecord(e1) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return 1;
    float ms = 0;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return 1;
    const double ns = ms * 1e6 / ((double)waves_per_simd * iters * per_trip);
    printf("%-34s %7.3f ms  %5.2f ns per wave instruction per SIMD = %4.1f clocks at 2.4 GHz\n", name, ms, ns, ns * 2.4);
    return 0;
}

// ---- memory ceilings ------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr uint64_t kRows = 20000000;  // rows of 64 floats: 5.12 GB
constexpr int kRowFloats = 64;

// rows ids[k], k < n, of 64 * PIECES floats, each by 16 lanes (a lane takes 16 bytes of every 256-byte
// piece); four rows per 16-lane group and pass, as in the library's kernels
// With SIDE > 0 every pass of 16 rows also moves 64 * SIDE consecutive bytes of `side` the other way
// (what the packed codes are to the restore, which reads them, and to the encode, which writes them:
// SIDE = 8 for 32 bytes per row, 32 for 128).
// THROUGH: the scatter's stores carry the write-through bits the restore kernel uses for rows that one
// instruction writes whole (system-scope, streaming), instead of the plain non-temporal hint.
template <bool WRITE, int PIECES, int SIDE = 0, bool THROUGH = false>
__global__ void __launch_bounds__(256) sparse_rows_kernel(float *__restrict__ table, const uint32_t *__restrict__ ids, uint64_t n,
                                                          uint32_t n_waves, float *out, float *__restrict__ side = nullptr) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const int lane = threadIdx.x & 63, g = lane >> 4, l = lane & 15;
    float acc = 0;
    for (uint64_t pass = (uint64_t)blockIdx.x * 4 + threadIdx.x / 64; pass * 16 < n; pass += n_waves) {
        const uint64_t k0 = pass * 16 + 4 * g;
        if constexpr (WRITE && SIDE == 8) {
            const f32x2 v = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(side) + pass * 64 + lane);
            acc += v.x + v.y;
        } else if constexpr (WRITE && SIDE >= 16) {
#pragma unroll
            for (int i = 0; i < SIDE / 16; ++i) {
                const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(side) + (pass * (SIDE / 16) + i) * 64 + lane);
                acc += v.x + v.w;
            }
        }
        uint32_t rid[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) rid[u] = k0 + u < n ? ids[k0 + u] : 0xFFFFFFFFu;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (rid[u] == 0xFFFFFFFFu) continue;  // ids are below kRows by construction
            f32x4 *p = reinterpret_cast<f32x4 *>(table + (uint64_t)rid[u] * (kRowFloats * PIECES) + 4 * l);
#pragma unroll
            for (int c = 0; c < PIECES; ++c) {
                if (WRITE && THROUGH) {
                    const f32x4 v = {1.f, 2.f, (float)l, (float)u};
                    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(p + 16 * c), "v"(v) : "memory");
                } else if (WRITE) {
                    __builtin_nontemporal_store(f32x4{1.f, 2.f, (float)l, (float)u}, p + 16 * c);
                } else {
                    const f32x4 v = __builtin_nontemporal_load(p + 16 * c);
                    acc += v.x + v.y + v.z + v.w;
                }
            }
        }
        if constexpr (!WRITE && SIDE == 8) {
            __builtin_nontemporal_store(f32x2{acc, acc}, reinterpret_cast<f32x2 *>(side) + pass * 64 + lane);
        } else if constexpr (!WRITE && SIDE >= 16) {
#pragma unroll
            for (int i = 0; i < SIDE / 16; ++i)
                __builtin_nontemporal_store(f32x4{acc, acc, acc, acc}, reinterpret_cast<f32x4 *>(side) + (pass * (SIDE / 16) + i) * 64 + lane);
        }
    }
    if (acc == 123.456f) out[0] = acc;
}
// MODE 0: read, 1: write, 2: copy a -> b, n16 units of 16 bytes
template <int MODE>
__global__ void __launch_bounds__(256) stream_kernel(const f32x4 *__restrict__ a, f32x4 *__restrict__ b, uint64_t n16, float *out) {
    float acc = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * 256) {
        if (MODE == 0) { const f32x4 v = __builtin_nontemporal_load(a + i); acc += v.x + v.w; }
        if (MODE == 1) __builtin_nontemporal_store(f32x4{1.f, 2.f, 3.f, 4.f}, b + i);
        if (MODE == 2) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
    }
    if (acc == 123.456f) out[0] = acc;
}
template <typename F>
static float time_us(F launch, int reps, hipStream_t stream = 0) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1;
    launch();
    launch();
    if (hipDeviceSynchronize() != hipSuccess || hipEventRecord(e0, stream) != hipSuccess) return -1;
    for (int i = 0; i < reps; ++i) launch();
    if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1;
    float ms = 0;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1;
    return ms / reps * 1e3f;
}
// a fraction of the rows of 64 * PIECES floats of the same 5.12 GB, ascending: gathered, then scattered
template <int PIECES>
static int sparse_rows(float *t[2], double fraction, int *flip, float *out) {
    const uint64_t rows = kRows / PIECES;
    std::vector<uint32_t> h;
    uint64_t s = 88172645463325252ull;  // xorshift
    for (uint64_t r = 0; r < rows; ++r) {
        s ^= s << 13; s ^= s >> 7; s ^= s << 17;
        if ((s >> 11) * (1.0 / 9007199254740992.0) < fraction) h.push_back((uint32_t)r);
    }
    const uint64_t n = h.size();
    uint32_t *ids;
    if (hipMalloc(&ids, n * 4) != hipSuccess || hipMemcpy(ids, h.data(), n * 4, hipMemcpyHostToDevice) != hipSuccess) return 1;
    const double row_bytes = (double)n * kRowFloats * PIECES * 4;
    const unsigned grid = (unsigned)((n + 63) / 64) < 24576u ? (unsigned)((n + 63) / 64) : 24576u;
    const float gr = time_us([&] { sparse_rows_kernel<false, PIECES><<<grid, 256>>>(t[*flip ^= 1], ids, n, grid * 4, out); }, 10);
    const float sw = time_us([&] { sparse_rows_kernel<true, PIECES><<<grid, 256>>>(t[*flip ^= 1], ids, n, grid * 4, out); }, 10);
    if (gr < 0 || sw < 0) return 1;
    printf("%llu of %llu rows of %d bytes, ascending, %u workgroups: gather-read %6.2f TB/s   scatter-write %6.2f TB/s (row bytes alone)\n",
           (unsigned long long)n, (unsigned long long)rows, kRowFloats * PIECES * 4, grid, row_bytes / gr / 1e6, row_bytes / sw / 1e6);
    // the restore's mix: the same scatter while 64 * SIDE bytes per 16 rows are read from the other table (n * SIDE * 4 bytes
    // in all, far less than the table holds)
    constexpr int kSide = PIECES == 1 ? 8 : 32;
    const float mix = time_us([&] {
        *flip ^= 1;
        sparse_rows_kernel<true, PIECES, kSide><<<grid, 256>>>(t[*flip], ids, n, grid * 4, out, t[*flip ^ 1]);
    }, 10);
    if (mix < 0) return 1;
    printf("  the same scatter with %d bytes per row read from a sequential buffer meanwhile: %6.2f TB/s (rows + that buffer)\n", kSide * 4,
           (row_bytes + (double)n * kSide * 4) / mix / 1e6);
    const float swt = time_us([&] { sparse_rows_kernel<true, PIECES, 0, true><<<grid, 256>>>(t[*flip ^= 1], ids, n, grid * 4, out); }, 10);
    const float mixt = time_us([&] {
        *flip ^= 1;
        sparse_rows_kernel<true, PIECES, kSide, true><<<grid, 256>>>(t[*flip], ids, n, grid * 4, out, t[*flip ^ 1]);
    }, 10);
    if (swt < 0 || mixt < 0) return 1;
    printf("  with write-through stores: scatter alone %6.2f TB/s, with the %d bytes per row read meanwhile %6.2f TB/s\n", row_bytes / swt / 1e6,
           kSide * 4, (row_bytes + (double)n * kSide * 4) / mixt / 1e6);
    // the encode's mix: the gather while that many bytes per row are written to the other table
    const float xim = time_us([&] {
        *flip ^= 1;
        sparse_rows_kernel<false, PIECES, kSide><<<grid, 256>>>(t[*flip], ids, n, grid * 4, out, t[*flip ^ 1]);
    }, 10);
    if (xim < 0) return 1;
    printf("  the same gather with %d bytes per row written to a sequential buffer meanwhile: %6.2f TB/s (rows + that buffer)\n", kSide * 4,
           (row_bytes + (double)n * kSide * 4) / xim / 1e6);
    (void)hipFree(ids);
    return 0;
}

static int memory_ceilings(float *out) {
    float *t[2];
    for (int i = 0; i < 2; ++i)
        if (hipMalloc(&t[i], kRows * kRowFloats * 4) != hipSuccess || hipMemset(t[i], 0, kRows * kRowFloats * 4) != hipSuccess) return 1;
    const uint64_t n16 = kRows * kRowFloats / 4;
    const double table_bytes = (double)kRows * kRowFloats * 4;
    int flip = 0;
    for (unsigned grid : {2048u, 8192u, 24576u}) {
        const float r = time_us([&] { stream_kernel<0><<<grid, 256>>>((const f32x4 *)t[0], (f32x4 *)t[1], n16, out); }, 5);
        const float w = time_us([&] { stream_kernel<1><<<grid, 256>>>((const f32x4 *)t[0], (f32x4 *)t[flip ^= 1], n16, out); }, 5);
        const float c = time_us([&] { stream_kernel<2><<<grid, 256>>>((const f32x4 *)t[0], (f32x4 *)t[1], n16, out); }, 5);
        if (r < 0 || w < 0 || c < 0) return 1;
        printf("whole table, %5u workgroups: read %6.2f TB/s   write %6.2f TB/s   copy %6.2f TB/s (read + write)\n", grid,
               table_bytes / r / 1e6, table_bytes / w / 1e6, 2 * table_bytes / c / 1e6);
    }
    if (sparse_rows<1>(t, 0.30, &flip, out) || sparse_rows<2>(t, 0.25, &flip, out)) return 1;
    (void)hipFree(t[0]); (void)hipFree(t[1]);
    return 0;
}

static int host_link_ceilings(float *out) {
    const uint64_t bytes = 64ull << 20, n16 = bytes / 16;
    void *host = nullptr, *host_dev = nullptr;
    float *dev = nullptr;
    if (hipHostMalloc(&host, bytes, hipHostMallocDefault) != hipSuccess || hipHostGetDevicePointer(&host_dev, host, 0) != hipSuccess ||
        hipMalloc(&dev, bytes) != hipSuccess || hipMemset(dev, 0, bytes) != hipSuccess)
        return 1;
    for (uint64_t i = 0; i < bytes / 4; ++i) ((float *)host)[i] = 1.0f;
    for (unsigned grid : {256u, 1024u, 4096u}) {
        const float r = time_us([&] { stream_kernel<2><<<grid, 256>>>((const f32x4 *)host_dev, (f32x4 *)dev, n16, out); }, 5);
        const float w = time_us([&] { stream_kernel<2><<<grid, 256>>>((const f32x4 *)dev, (f32x4 *)host_dev, n16, out); }, 5);
        if (r < 0 || w < 0) return 1;
        printf("64 MiB of pinned host memory, %4u workgroups: a kernel reads it at %5.1f GB/s, writes it at %5.1f GB/s\n", grid,
               bytes / r / 1e3, bytes / w / 1e3);
    }
    hipStream_t s;
    if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) return 1;
    for (int round = 0; round < 2; ++round) {
        const float cr = time_us([&] { (void)hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, s); }, 10, s);
        const float cw = time_us([&] { (void)hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, s); }, 10, s);
        if (cr < 0 || cw < 0) return 1;
        printf("the runtime's asynchronous copy of the same 64 MiB on a stream: host to device %5.1f GB/s, device to host %5.1f GB/s\n",
               bytes / cr / 1e3, bytes / cw / 1e3);
    }
    (void)hipStreamDestroy(s);
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    (void)hipFree(dev);
    (void)hipHostFree(host);
    return 0;
}

// ---- what one compute unit streams ----------------------------------------------------------------
// The bulk mark through bitmap slices (Section 5.1.1) has every workgroup (1,024 threads, one per
// compute unit) read one eighth of a table's index stream, the same eighth as the other workgroups
// of its team, so that the bytes come from the L2 of the workgroup's XCD.  This is that read alone:
// 256 workgroups, workgroup x reads eighth x & 7 of a 24 MB buffer with 16-byte loads, UNROLL loads
// per lane in flight.
template <int UNROLL>
__global__ void __launch_bounds__(1024) shared_stream_kernel(const f32x4 *__restrict__ a, uint64_t n16, float *out) {
    const uint64_t per_part = n16 / 8;
    const f32x4 *p = a + (blockIdx.x & 7) * per_part;
    float acc = 0;
    for (uint64_t i = threadIdx.x; i < per_part; i += 1024 * UNROLL) {
        f32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (i + 1024 * u < per_part) v[u] = p[i + 1024 * u];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (i + 1024 * u < per_part) acc += v[u].x + v[u].w;
    }
    if (acc == 123.456f) out[0] = acc;
}
static int compute_unit_stream(float *out) {
    const uint64_t bytes = 24ull << 20, n16 = bytes / 16;
    float *buf = nullptr;
    if (hipMalloc(&buf, bytes) != hipSuccess || hipMemset(buf, 0, bytes) != hipSuccess) return 1;
    const float t4 = time_us([&] { shared_stream_kernel<4><<<256, 1024>>>((const f32x4 *)buf, n16, out); }, 10);
    const float t16 = time_us([&] { shared_stream_kernel<16><<<256, 1024>>>((const f32x4 *)buf, n16, out); }, 10);
    if (t4 < 0 || t16 < 0) return 1;
    const double per_wg = (double)bytes / 8;
    printf("256 workgroups of 1024 threads, each streaming an eighth (3 MB) of a 24 MB buffer shared by 32 of them: %5.1f GB/s per compute unit with 4 loads "
           "per lane in flight, %5.1f with 16 (%4.1f and %4.1f TB/s over the chip)\n",
           per_wg / t4 / 1e3, per_wg / t16 / 1e3, 256 * per_wg / t4 / 1e6, 256 * per_wg / t16 / 1e6);
    (void)hipFree(buf);
    return 0;
}

int main() {
    float *out;
    if (hipMalloc(&out, 4) != hipSuccess) return 1;
    int rc = 0;
    rc |= run<ADD>("v_add_f32", 32, out);
    rc |= run<SUB>("v_sub_f32", 32, out);
    rc |= run<MUL>("v_mul_f32", 32, out);
    rc |= run<FMA>("v_fma_f32", 32, out);
    rc |= run<MED3>("v_med3_f32", 32, out);
    rc |= run<RNDNE>("v_rndne_f32", 32, out);
    rc |= run<CVT_F64_F32>("v_cvt_f64_f32", 32, out);
    rc |= run<FMA_F64>("v_fma_f64", 32, out);
    rc |= run<ADD_F64>("v_add_f64", 32, out);
    rc |= run<GREEDY_MIX>("greedy element (9 instructions)", 72, out);
    rc |= memory_ceilings(out);
    rc |= host_link_ceilings(out);
    rc |= compute_unit_stream(out);
    if (hipDeviceSynchronize() != hipSuccess) rc = 1;
    (void)hipFree(out);
    return rc;
}
