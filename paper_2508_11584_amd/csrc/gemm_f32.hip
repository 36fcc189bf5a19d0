// fp32-operand instantiations of the MFMA GEMM, plus the dtype dispatch.
#include <cstdlib>

#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s);
namespace { bool g_no_splitk_f32 = false; }
hipError_t launch_gemm(int dtype, const GemmArgs& a, int amode, hipStream_t s) {
    if (dtype) return launch_gemm_bf16(a, amode, s);
    // as in the bf16 dispatch: 64 x 64 tiles with at most one tile per CU and at least 4 k-tiles (32 deep here) go
    // to the split-k kernel; VPE_NO_SPLITK (read when an engine is created) switches it off
    const bool no_splitk = g_no_splitk_f32;
    const int nz = a.nz > 1 ? a.nz : 1;
    const int64_t t64 = (int64_t)cdiv(a.M, 64) * cdiv(a.N, 64) * nz, t64x128 = (int64_t)cdiv(a.M, 64) * cdiv(a.N, 128) * nz;
    if (!no_splitk && a.epi != EPI_SWIGLU && t64x128 < 384 && t64 <= 256 && a.K >= 128)
        return launch_tile_splitk<float, 64, 64, 2, 2, 2>(a, amode, s);
    return launch_gemm_t<float>(a, amode, s);
}

// LDS opt-in of the fp32 split-k kernel; called once at engine creation, outside any stream capture.
hipError_t configure_gemm_f32() {
    g_no_splitk_f32 = getenv("VPE_NO_SPLITK") != nullptr;
    GemmArgs a{};
    return launch_tile_splitk<float, 64, 64, 2, 2, 2>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
