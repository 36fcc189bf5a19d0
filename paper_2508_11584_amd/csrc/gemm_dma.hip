// Instantiations of the large-tile direct-to-LDS GEMM.
#include "conv_strip.h"
#include "gemm_dma.h"
#include "kernels.h"
namespace vpe {
// Measured on MI355X, 3x3 conv 256->256 (K = 2304) with real data, TFLOP/s at whole rounds of workgroups:
//   128: 256 x 128 tile, 32-deep k-tiles, 8 waves (64 x 64 wave tiles), two workgroups per CU      820-850
//   256: 256 x 256 tile, 64-deep k-tiles, 8 waves (64 x 128 wave tiles), one workgroup per CU       975
//   384: 384 x 256 tile, 32-deep k-tiles, 8 waves (96 x 128 wave tiles), one workgroup per CU       995
// and two small shapes for small problems (4 waves, 64-deep k-tiles), faster than their register-staged
// counterparts by 8-14 % on the ViT-S / ViT-B GEMMs and the small convolutions:
//    64: 64 x 64 tile (32 x 32 wave tiles, block-level epilogue), 65: 64 x 128 tile (32 x 64 wave tiles)
// The one-per-CU shapes run in lockstep rounds, so they pay for a partly filled last round in full; which
// shape wins depends on how the tile count divides by the 256 CUs (see launch_gemm_bf16).
hipError_t launch_gemm_dma_bf16(int kind, const GemmArgs& a, int amode, hipStream_t s) {
    if (kind == 64) return launch_gemm_dma<64, 64, 2, 2, 2, 2, 64>(a, amode, s);
    if (kind == 65) return launch_gemm_dma<128, 64, 2, 2, 2, 2, 64>(a, amode, s);
    const bool rd = amode == A_CONV3 && a.epi == EPI_ROWDOT && !a.ln_stats;   // projection epilogue from transposed accumulators
    if (kind == 384) return rd ? launch_gemm_dma<256, 32, 2, 4, 2, 1, 384, true>(a, amode, s) : launch_gemm_dma<256, 32, 2, 4, 2, 1, 384>(a, amode, s);
    if (kind == 256) return rd ? launch_gemm_dma<256, 64, 2, 4, 2, 1, 256, true>(a, amode, s) : launch_gemm_dma<256, 64, 2, 4, 2, 1>(a, amode, s);
    return launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, amode, s);
}
// 3x3 convolution from an input strip in LDS (conv_strip.h): 384 x 256 tiles, 96 x 128 wave tiles.
bool conv_strip_applies(const GemmArgs& a) { return conv_strip_fits<384, 256>(a); }
int64_t conv_strip_tiles(const GemmArgs& a) {
    return (strip_positions(a.M / (a.cH * a.cW), a.cH, a.cW) + 383) / 384 * cdiv(a.N, 256) * (a.nz > 1 ? a.nz : 1);
}
hipError_t launch_conv_strip_bf16(const GemmArgs& a, hipStream_t s) {
    return a.epi == EPI_ROWDOT ? launch_conv_strip<384, 256, 4, 2, 1, true>(a, s) : launch_conv_strip<384, 256, 4, 2, 1, false>(a, s);
}

// LDS opt-in (more than 64 KB) where needed; called once at engine creation.
hipError_t configure_gemm() {
    GemmArgs a{};
    hipError_t rc = launch_conv_strip<384, 256, 4, 2, 1, true>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_conv_strip<384, 256, 4, 2, 1, false>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 32, 2, 4, 2, 1, 384>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 32, 2, 4, 2, 1, 384, true>(a, A_CONV3, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 64, 2, 4, 2, 1, 256, true>(a, A_CONV3, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<64, 64, 2, 2, 2, 2, 64>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<128, 64, 2, 2, 2, 2, 64>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 64, 2, 4, 2, 1>(a, A_PLAIN, nullptr, true);
    return rc != hipSuccess ? rc : launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
