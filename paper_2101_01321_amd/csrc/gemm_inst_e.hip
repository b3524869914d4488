// Instantiations of the MFMA MatMul kernel (gemm_kernel.h) for the tile configurations of gemm_instances_e.inc.
#include "gemm_kernel.h"

namespace ibert {

#define IBERT_GEMM_INSTANCE(...) template int launch_mfma<__VA_ARGS__>(GemmArgs&, bool, hipStream_t);
#include "gemm_instances_e.inc"
#undef IBERT_GEMM_INSTANCE

}  // namespace ibert
