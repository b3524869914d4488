// Probe (not part of the library): global loads in MFMA-operand order (lane = row, the four lanes 16 apart share a row) against the same bytes in lane-contiguous order, L2-resident source.
// Build and run:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops fragload.hip -o /tmp/fragload && /tmp/fragload
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { if ((x) != hipSuccess) { std::fprintf(stderr, "%s failed\n", #x); return 1; } } while (0)
#include <cstdlib>
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
template <int MODE>
__global__ __launch_bounds__(256) void k(const int8_t* __restrict__ A, int lda, int K, int reps, int* __restrict__ out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mblk = blockIdx.x >> 4;              // 16 replicas (stand-ins for N tiles) share the same rows
    const int row0 = mblk * 256 + wave * 64;
    int r, c;
    if (MODE == 0) { r = lane >> 2; c = lane & 3; } else { r = lane & 15; c = lane >> 4; }
    const int8_t* p = A + (long)(row0 + r) * lda + c * 16;
    v4i acc = {0, 0, 0, 0};
    for (int rep = 0; rep < reps; ++rep) {
        for (int k0 = 0; k0 < K; k0 += 128) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                v4i a = *(const v4i*)(p + (long)t * 16 * lda + k0);
                v4i b = *(const v4i*)(p + (long)t * 16 * lda + k0 + 64);
                acc ^= a; acc ^= b;
            }
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1;
}
int main()
{
    const int M = 4096, K = 768, reps = 20;
    int8_t* A; int* out;
    CK(hipMalloc(&A, (size_t)M * K)); CK(hipMemset(A, 1, (size_t)M * K)); CK(hipMalloc(&out, 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int mode = 0; mode < 2; ++mode) {
        for (int it = 0; it < 3; ++it) {
            CK(hipEventRecord(e0));
            if (mode == 0) hipLaunchKernelGGL(k<0>, dim3(M / 256 * 16), dim3(256), 0, 0, A, K, K, reps, out);
            else hipLaunchKernelGGL(k<1>, dim3(M / 256 * 16), dim3(256), 0, 0, A, K, K, reps, out);
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            double bytes = (double)M * K * 16 * reps;
            printf("mode %d: %.1f us, %.2f TB/s, %.1f B/clk/CU @2.4GHz\n", mode, ms * 1e3, bytes / ms / 1e9, bytes / (ms * 1e-3) / 256 / 2.4e9);
        }
    }
    if (hipDeviceSynchronize() != hipSuccess) { printf("error\n"); return 1; }
    return 0;
}
