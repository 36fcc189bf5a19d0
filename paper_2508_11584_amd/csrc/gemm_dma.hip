// Instantiations of the large-tile direct-to-LDS GEMM.
#include "gemm_dma.h"
#include "kernels.h"
namespace vpe {
// 256 x 128 tiles, 32-deep k-tiles, 8 waves, two workgroups per CU (the fastest shape measured:
// 970 TFLOP/s on the 3x3 conv 256->256 at 272x360, 920 on M=10992 N=8192 K=1536);
// 256 x 256 tiles with 16 waves, one workgroup per CU, as the alternative.
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s) {
    return bn == 256 ? launch_gemm_dma<256, 64, 2, 4, 4, 1>(a, amode, s) : launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, amode, s);
}
// LDS opt-in (more than 64 KB) where needed; called once at engine creation.
hipError_t configure_gemm() {
    GemmArgs a{};
    hipError_t rc = launch_gemm_dma<256, 64, 2, 4, 4, 1>(a, A_PLAIN, nullptr, true);
    return rc != hipSuccess ? rc : launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
