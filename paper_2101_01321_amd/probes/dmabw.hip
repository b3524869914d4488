// Probe (not part of the library): global_load_lds_dwordx4 (straight into LDS) against plain 16-byte loads, L2-resident source, one to six batches of eight requests in flight.
// Build and run:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops dmabw.hip -o /tmp/dmabw && /tmp/dmabw
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { if ((x) != hipSuccess) { std::fprintf(stderr, "%s failed\n", #x); return 1; } } while (0)
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
template <int MODE, int INFLIGHT>
__global__ __launch_bounds__(256) void k(const int8_t* __restrict__ A, int lda, int K, int reps, int* __restrict__ out)
{
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int mblk = blockIdx.x >> 4;                      // 16 replicas share the same rows
    const int row0 = mblk * 256 + wave * 64;
    // lane -> (row l/8, 16-byte chunk l%8) of a 128-byte row: 8 rows x 128 B per instruction
    const uint32_t voff = (uint32_t)(lane >> 3) * lda + ((lane & 7) << 4);
    const int8_t* base = A + (long)row0 * lda;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds + wave * 8192;
    v4i acc = {0, 0, 0, 0};
    for (int rep = 0; rep < reps; ++rep) {
        for (int k0 = 0; k0 < K; k0 += 128) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {                  // 8 instructions: 64 rows x 128 B = 8 KB per wave
                const int8_t* sb = base + (long)t * 8 * lda + k0;
                if (MODE == 0) {
                    acc ^= *(const v4i*)(sb + voff);
                } else {
                    const uint32_t la = lds0 + t * 1024;
                    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(la), "v"(voff), "s"(sb) : "memory", "m0");
                }
            }
            if (MODE == 1 && (k0 / 128) % INFLIGHT == INFLIGHT - 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1;
}
int main()
{
    const int M = 4096, K = 768, reps = 20;
    int8_t* A; int* out;
    CK(hipMalloc(&A, (size_t)M * K)); CK(hipMemset(A, 1, (size_t)M * K)); CK(hipMalloc(&out, 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int mode = 0; mode < 4; ++mode) {
        for (int it = 0; it < 2; ++it) {
            CK(hipEventRecord(e0));
            const dim3 grid(M / 256 * 16), block(256);
            if (mode == 0) hipLaunchKernelGGL((k<0, 1>), grid, block, 32768, 0, A, K, K, reps, out);
            else if (mode == 1) hipLaunchKernelGGL((k<1, 1>), grid, block, 32768, 0, A, K, K, reps, out);
            else if (mode == 2) hipLaunchKernelGGL((k<1, 2>), grid, block, 32768, 0, A, K, K, reps, out);
            else hipLaunchKernelGGL((k<1, 6>), grid, block, 32768, 0, A, K, K, reps, out);
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            double bytes = (double)M * K * 16 * reps;
            printf("mode %d: %.1f us, %.2f TB/s, %.1f B/clk/CU @2.4GHz\n", mode, ms * 1e3, bytes / ms / 1e9, bytes / (ms * 1e-3) / 256 / 2.4e9);
        }
    }
    if (hipDeviceSynchronize() != hipSuccess) { printf("error\n"); return 1; }
    return 0;
}
