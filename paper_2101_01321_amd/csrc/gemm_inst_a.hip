// Instantiations of the MFMA MatMul kernel (gemm_kernel.h) for the tile configurations of gemm_instances_a.inc.
#include "gemm_kernel.h"

namespace ibert {

#define IBERT_GEMM_INSTANCE(...) template int launch_mfma<__VA_ARGS__>(GemmArgs&, bool, hipStream_t);
#include "gemm_instances_a.inc"
#undef IBERT_GEMM_INSTANCE

// K not a multiple of 16 (rows still 16-byte aligned): one configuration with the bytewise tail loader.
int launch_tail(GemmArgs& g, bool i8, hipStream_t stream)
{
    constexpr int BM = 128, BN = 128, BK = 128, RING = 2;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n * g.nbatch;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    g.xcd_chunk = 0;
    constexpr size_t lds_bytes = EpiLayout<BM, BN, BK>::LDS_BYTES;
    static bool attr_done[2] = {false, false};
    const void* kern = i8 ? reinterpret_cast<const void*>(gemm_nt_mfma_kernel<BM, BN, BK, RING, true, 2>)
                          : reinterpret_cast<const void*>(gemm_nt_mfma_kernel<BM, BN, BK, RING, false, 2>);
    if (!attr_done[i8]) {
        IBERT_HIP_CHECK(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        attr_done[i8] = true;
    }
    if (i8) hipLaunchKernelGGL((gemm_nt_mfma_kernel<BM, BN, BK, RING, true, 2>), dim3((unsigned)blocks), dim3(GEMM_THREADS), lds_bytes, stream, g);
    else hipLaunchKernelGGL((gemm_nt_mfma_kernel<BM, BN, BK, RING, false, 2>), dim3((unsigned)blocks), dim3(GEMM_THREADS), lds_bytes, stream, g);
    IBERT_LAUNCH_CHECK("gemm_nt_mfma_kernel");
    g_last_kernel = i8 ? "gemm_nt_mfma_kernel<128, 128, 128, 2, true, 2, false>" : "gemm_nt_mfma_kernel<128, 128, 128, 2, false, 2, false>";
    return IBERT_OK;
}


}  // namespace ibert
