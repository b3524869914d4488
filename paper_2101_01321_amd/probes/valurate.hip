// Probe (not part of the library): issue cost, in cycles per wavefront instruction on one SIMD, of the multiply and conversion instructions an exact requantization can be built from.
// Build and run:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops valurate.hip -o /tmp/valurate && /tmp/valurate
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define CK(x) do { if ((x) != hipSuccess) { std::fprintf(stderr, "%s failed\n", #x); return 1; } } while (0)

// One wavefront per SIMD (256 threads on one CU), 8 independent chains per lane so that result latency is hidden:
// the time per instruction is then its issue cost.
#define CHAINS 8
#define BODY(ASM, ...)                                                                   \
    for (int r = 0; r < reps; ++r) {                                                     \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                  \
            _Pragma("unroll") for (int c = 0; c < CHAINS; ++c) asm volatile(ASM : __VA_ARGS__); \
        }                                                                                \
    }

__global__ __launch_bounds__(256) void k(int which, int reps, int seed, int* out, long long* cyc)
{
    int32_t a[CHAINS], b = seed | 0x40000001, lo = 0;
    long long w[CHAINS];
    double d[CHAINS];
    for (int c = 0; c < CHAINS; ++c) { a[c] = seed + c * 77 + threadIdx.x; w[c] = a[c]; d[c] = (double)a[c]; }
    const double md = 1.0000001, rd = 0.5;
    const long long t0 = __builtin_readcyclecounter();
    switch (which) {
        case 0: BODY("v_mad_i64_i32 %0, vcc, %1, %2, %0", "+v"(w[c]) : "v"(a[c]), "v"(b) : "vcc") break;
        case 1: BODY("v_mul_hi_i32 %0, %0, %1", "+v"(a[c]) : "v"(b)) break;
        case 2: BODY("v_mul_lo_u32 %0, %0, %1", "+v"(a[c]) : "v"(b)) break;
        case 3: BODY("v_mul_i32_i24 %0, %0, %1", "+v"(a[c]) : "v"(b)) break;
        case 4: BODY("v_mul_hi_i32_i24 %0, %0, %1", "+v"(a[c]) : "v"(b)) break;
        case 5: BODY("v_fma_f64 %0, %0, %1, %2", "+v"(d[c]) : "v"(md), "v"(rd)) break;
        case 6: BODY("v_cvt_f64_i32 %0, %1", "=v"(d[c]) : "v"(a[c])) break;
        case 7: BODY("v_floor_f64 %0, %0", "+v"(d[c]) : ) break;
        case 8: BODY("v_cvt_i32_f64 %0, %1", "=v"(a[c]) : "v"(d[c])) break;
        case 9: BODY("v_add_u32 %0, %0, %1", "+v"(a[c]) : "v"(b)) break;
        case 10: BODY("v_ashrrev_i64 %0, %1, %0", "+v"(w[c]) : "v"(lo)) break;
        case 11: BODY("v_mad_u64_u32 %0, vcc, %1, %2, %0", "+v"(w[c]) : "v"(a[c]), "v"(b) : "vcc") break;
        case 12: BODY("v_mul_f64 %0, %0, %1", "+v"(d[c]) : "v"(md)) break;
        case 13: BODY("v_mad_i32_i24 %0, %0, %1, %1", "+v"(a[c]) : "v"(b)) break;
        default: break;
    }
    const long long t1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) cyc[0] = t1 - t0;
    long long s = 0;
    for (int c = 0; c < CHAINS; ++c) s += a[c] + w[c] + (long long)d[c];
    if (s == 0x123456789LL) out[0] = 1;
}

int main()
{
    int* out; long long* cyc; CK(hipMalloc(&out, 4)); CK(hipMalloc(&cyc, 8));
    const char* names[] = {"v_mad_i64_i32", "v_mul_hi_i32", "v_mul_lo_u32", "v_mul_i32_i24", "v_mul_hi_i32_i24", "v_fma_f64",
                           "v_cvt_f64_i32", "v_floor_f64", "v_cvt_i32_f64", "v_add_u32", "v_ashrrev_i64", "v_mad_u64_u32",
                           "v_mul_f64", "v_mad_i32_i24"};
    const int reps = 4000;
    for (int which = 0; which < 14; ++which) {
        long long best = 1LL << 60;
        for (int t = 0; t < 3; ++t) {
            hipLaunchKernelGGL(k, dim3(1), dim3(256), 0, 0, which, reps, 12345, out, cyc);
            CK(hipDeviceSynchronize());
            long long h; CK(hipMemcpy(&h, cyc, 8, hipMemcpyDeviceToHost));
            if (h < best) best = h;
        }
        std::printf("%-18s %6.2f cycles per wavefront instruction\n", names[which], (double)best / (reps * 4.0 * CHAINS));
    }
    return 0;
}
