// Probe (not part of the library): ds_read_b128 / ds_write_b128 throughput of one CU for the lane-to-address patterns an MFMA operand read produces, with and without row swizzles.
// Build and run:  hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops ldsbw.hip -o /tmp/ldsbw && /tmp/ldsbw
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { if ((x) != hipSuccess) { std::fprintf(stderr, "%s failed\n", #x); return 1; } } while (0)
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int pattern_addr(int pat, int l)
{
    const int r16 = l & 15, kc = l >> 4;
    switch (pat) {
        case 0: return l * 16;                                                   // linear
        case 1: return r16 * 128 + ((kc ^ (r16 & 7)) << 4);                      // frag, 128 B rows, xor row&7
        case 2: return r16 * 64 + ((kc ^ ((r16 >> 1) & 3)) << 4);                // frag, 64 B rows, xor (row>>1)&3
        case 3: return r16 * 128 + (kc << 4);                                    // frag, 128 B rows, no swizzle
        case 4: { const int g = 4;  return (((l % 4) + 4 * ((l / g) % 2)) << 4) + ((l / 4 % (g / 4)) + (g / 4) * (l / (2 * g))) * 128; }
        case 5: { const int g = 8;  return (((l % 4) + 4 * ((l / g) % 2)) << 4) + ((l / 4 % (g / 4)) + (g / 4) * (l / (2 * g))) * 128; }
        case 6: { const int g = 16; return (((l % 4) + 4 * ((l / g) % 2)) << 4) + ((l / 4 % (g / 4)) + (g / 4) * (l / (2 * g))) * 128; }
        case 7: { const int g = 32; return (((l % 4) + 4 * ((l / g) % 2)) << 4) + ((l / 4 % (g / 4)) + (g / 4) * (l / (2 * g))) * 128; }
        case 8: return r16 * 128 + ((kc ^ ((r16 >> 1) & 7)) << 4);               // frag 128 B rows, xor (row>>1)
        case 9: return r16 * 144 + (kc << 4);                                    // frag, padded rows (128+16)
        case 10: return r16 * 80 + (kc << 4);                                    // frag, padded rows (64+16)
        case 11: return r16 * 128 + ((kc ^ ((r16 & 7) ^ ((r16 >> 3) & 1))) << 4);  // current swz<8>
        case 12: return r16 * 64 + ((kc ^ (((r16 >> 1) & 3) ^ ((r16 >> 3) & 1))) << 4);   // current swz<4>
        default: return 0;
    }
}
template <bool WRITE>
__global__ __launch_bounds__(256) void k(int pat, int reps, int* __restrict__ out, long long* __restrict__ cyc)
{
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 16384 / 4; i += 256) ((int*)lds)[i] = i;
    __syncthreads();
    const uint32_t addr = (uint32_t)(wave * 4096 + pattern_addr(pat, lane));
    v4i acc = {0, 0, 0, 0};
    const long long t0 = __builtin_readcyclecounter();
    for (int r = 0; r < reps; ++r) {
        if (WRITE) {
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_write_b128 %0, %1" :: "v"(addr), "v"(acc) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        } else {
            v4i t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) asm volatile("ds_read_b128 %0, %1" : "=v"(t[u]) : "v"(addr) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= t[u];
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    if (threadIdx.x == 0) cyc[blockIdx.x] = t1 - t0;
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) out[0] = 1;
}
int main()
{
    int* out; long long* cyc; CK(hipMalloc(&out, 4)); CK(hipMalloc(&cyc, 256 * 8));
    const int reps = 2000;
    long long h[256];
    for (int w = 0; w < 2; ++w)
        for (int pat = 0; pat <= 12; ++pat) {
            for (int it = 0; it < 2; ++it) {
                if (w) hipLaunchKernelGGL(k<true>, dim3(256), dim3(256), 16384, 0, pat, reps, out, cyc);
                else hipLaunchKernelGGL(k<false>, dim3(256), dim3(256), 16384, 0, pat, reps, out, cyc);
                CK(hipDeviceSynchronize());
            }
            CK(hipMemcpy(h, cyc, sizeof(h), hipMemcpyDeviceToHost));
            double c = 0; for (int i = 0; i < 256; ++i) c += h[i]; c /= 256;
            // cycle counter here runs at 100 MHz on some parts: report raw and bytes per counter tick
            printf("%s pat %2d: %.0f ticks, %.1f B/tick/CU\n", w ? "write" : "read ", pat, c, 4.0 * 8 * reps * 1024 / c);
        }
    return 0;
}
