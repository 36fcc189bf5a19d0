// Instantiations of the large-tile direct-to-LDS GEMM.
#include <cstdlib>

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
// 3x3 convolution from an input strip in LDS (conv_strip.h), 96 x 128 wave tiles: 768 x 128 tiles (eight waves on top
// of each other; per 16-channel chunk a tile loads a strip of 768 + 2 (W + 1) + 2 positions and 128 x 9 weight rows: at
// W = 360, 22 % fewer bytes through the direct-to-LDS path than the 384 x 256 shape) or 384 x 256 tiles (4 x 2 waves).
// Returns the shape to use (0: none, 1: 384 x 256, 2: 768 x 128) and its tile count.  VPE_STRIP_SHAPE = 1 / 2 in the
// environment (read at engine creation) keeps to one of them.
static int g_strip_shape = 0;
static int64_t strip_tiles(const GemmArgs& a, int bm, int bn) {
    return (strip_positions(a.M / (a.cH * a.cW), a.cH, a.cW) + bm - 1) / bm * cdiv(a.N, bn) * (a.nz > 1 ? a.nz : 1);
}
int conv_strip_shape(const GemmArgs& a, bool any_size, int64_t* tiles) {
    const bool one_round_only = !any_size;
    for (int shape = 2; shape >= 1; --shape) {
        if (g_strip_shape && g_strip_shape != shape) continue;
        const bool fits = shape == 2 ? conv_strip_fits<768, 128>(a) : conv_strip_fits<384, 256>(a);
        if (!fits) continue;
        const int64_t t = shape == 2 ? strip_tiles(a, 768, 128) : strip_tiles(a, 384, 256);
        if (one_round_only && !(t > 192 && t <= 256)) continue;    // one well-filled round of the 256 CUs
        if (tiles) *tiles = t;
        return shape;
    }
    return 0;
}
hipError_t launch_conv_strip_bf16(int shape, const GemmArgs& a, hipStream_t s) {
    const bool rd = a.epi == EPI_ROWDOT;
    if (shape == 2) return rd ? launch_conv_strip<768, 128, 8, 1, 1, true>(a, s) : launch_conv_strip<768, 128, 8, 1, 1, false>(a, s);
    return rd ? launch_conv_strip<384, 256, 4, 2, 1, true>(a, s) : launch_conv_strip<384, 256, 4, 2, 1, false>(a, s);
}

// LDS opt-in (more than 64 KB) where needed; called once at engine creation.
hipError_t configure_gemm() {
    GemmArgs a{};
    const char* env = getenv("VPE_STRIP_SHAPE");
    g_strip_shape = env ? atoi(env) : 0;
    hipError_t rc = launch_conv_strip<384, 256, 4, 2, 1, true>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_conv_strip<384, 256, 4, 2, 1, false>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_conv_strip<768, 128, 8, 1, 1, true>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_conv_strip<768, 128, 8, 1, 1, false>(a, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 32, 2, 4, 2, 1, 384>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 32, 2, 4, 2, 1, 384, true>(a, A_CONV3, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 64, 2, 4, 2, 1, 256, true>(a, A_CONV3, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<64, 64, 2, 2, 2, 2, 64>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<128, 64, 2, 2, 2, 2, 64>(a, A_PLAIN, nullptr, true);
    if (rc == hipSuccess) rc = launch_gemm_dma<256, 64, 2, 4, 2, 1>(a, A_PLAIN, nullptr, true);
    return rc != hipSuccess ? rc : launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
