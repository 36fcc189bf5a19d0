// Instantiations of the large-tile direct-to-LDS GEMM.
#include "gemm_dma.h"
#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s) {
    return bn == 256 ? launch_gemm_dma<256, 32, 4>(a, amode, s) : launch_gemm_dma<128, 32, 4>(a, amode, s);
}
// LDS opt-in (more than 64 KB) for both tile widths; called once at engine creation.
hipError_t configure_gemm() {
    GemmArgs a{};
    hipError_t rc = launch_gemm_dma<256, 32, 4>(a, A_PLAIN, nullptr, true);
    return rc != hipSuccess ? rc : launch_gemm_dma<128, 32, 4>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
