// bf16-operand instantiations of the register-staged MFMA GEMM, and the choice between it and
// the large-tile direct-to-LDS kernel.
#include <cstdlib>

#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s);

hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s) {
    // Large problems go to the 256-row tiles (one workgroup per CU): they need enough tiles to
    // occupy most of the 256 CUs, and byte offsets that fit 31 bits (the loader keeps them in ints).
    const char* env = getenv("VPE_GEMM_TILE");
    const int forced = env ? atoi(env) : 0;
    const int64_t a_rows = amode == A_PLAIN ? (int64_t)(a.M / a.a_rpi + 1) * (a.a_istride > a.a_rpi ? a.a_istride : a.a_rpi)
                                            : (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride;
    const bool fits = a_rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
    const int64_t t256 = (int64_t)cdiv(a.M, 256) * cdiv(a.N, 256), t128 = (int64_t)cdiv(a.M, 256) * cdiv(a.N, 128);
    // Problems with enough 256 x 128 tiles to keep two workgroups on every CU busy go to the
    // direct-to-LDS kernel; everything else stays on the register-staged tiles.
    (void)t256;
    int bn = fits && t128 >= 448 ? 128 : 0;
    if (forced == 256 || forced == 128) bn = fits ? forced : 0;
    if (forced == 1) bn = 0;
    if (bn) return launch_gemm_dma_bf16(bn, a, amode, s);
    return launch_gemm_t<bf16>(a, amode, s);
}
}  // namespace vpe
