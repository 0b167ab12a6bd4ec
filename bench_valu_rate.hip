// How long a wave's vector instruction occupies a SIMD on gfx950, per kind of instruction: the figures
// behind the instruction-issue bound that bench.py quotes for the greedy range search (Section 5.2,
// Approach 3), whose inner loop is pure vector arithmetic.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 bench_valu_rate.hip -o bench_valu_rate && ./bench_valu_rate
//
// Every kernel runs one kind of instruction over 32 independent registers per lane (16 for fp64), so
// that nothing waits for an earlier result, with 8 waves per SIMD on all 256 compute units, and prints
// the time per wave instruction per SIMD.  Inline assembly pins the instruction; every operand is a
// register the kernel owns, nothing is loaded or stored inside the loops.
#include <hip/hip_runtime.h>
#include <stdio.h>

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
    if (hipDeviceSynchronize() != hipSuccess) rc = 1;
    (void)hipFree(out);
    return rc;
}
