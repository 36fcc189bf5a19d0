// bf16-operand instantiations of the register-staged MFMA GEMM, and the choice between them and
// the large-tile direct-to-LDS kernel.
#include <cstdlib>

#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s);

namespace {
// Candidate tilings: tile, workgroups a CU holds at once, and the two coefficients of the time model
//     t [us] = alpha * max(r, 1) + beta * r * (bm * bn * K / 1e6),     r = ceil(tiles / 256) / held,
// r being the number of "rounds" on the busiest of the 256 CUs (it gets ceil(tiles / 256) tiles and works on
// `held` of them at a time); alpha is the cost a workgroup pays whatever its size (first loads, epilogue), not
// discounted on a partly filled chip.  Fitted (relative least squares) to 28 measured shapes x 6 tilings on
// MI355X with random bf16 data: the QKV / proj / fc1 / fc2 GEMMs of ViT-S, -B, -L (batch 4) and -g (batch 8),
// the heads' 1x1 projections, and the 3x3 convolutions at 34x45 ... 296x296 grids (batch 1 and 4).  The
// model's pick is the measured best or within 4 % of it on every one of them (0.2 % in total time).
struct Cand { int kind, bm, bn, held; float alpha, beta; };
constexpr Cand kCands[] = {
    {128, 256, 128, 2, 5.35f, 1.057f},    // direct-to-LDS, 64 x 64 wave tiles
    {256, 256, 256, 1, 12.15f, 0.333f},   // direct-to-LDS, 64 x 128 wave tiles
    {384, 384, 256, 1, 16.00f, 0.359f},   // direct-to-LDS, 96 x 128 wave tiles
    {1, 128, 128, 2, 7.85f, 1.116f},      // register-staged
    {2, 64, 128, 3, 6.08f, 1.980f},
    {3, 64, 64, 4, 4.90f, 3.201f},
};
}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s) {
    const char* env = getenv("VPE_GEMM_TILE");
    const int forced = env ? atoi(env) : 0;
    // the direct-to-LDS loader keeps byte offsets in 32-bit ints
    const int64_t a_rows = amode == A_PLAIN ? (int64_t)(a.M / a.a_rpi + 1) * (a.a_istride > a.a_rpi ? a.a_istride : a.a_rpi)
                                            : (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride;
    const bool fits = a_rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
    int best = 3;
    float best_cost = 0.0f;
    for (const Cand& c : kCands) {
        if (c.kind >= 128 && !fits) continue;
        if (c.kind == 3 && a.epi == EPI_SWIGLU) continue;       // needs 64-column wave tiles
        const int64_t tiles = (int64_t)cdiv(a.M, c.bm) * cdiv(a.N, c.bn) * (a.nz > 1 ? a.nz : 1);
        const float r = (float)cdiv(tiles, 256) / c.held;
        const float cost = c.alpha * (r > 1.0f ? r : 1.0f) + c.beta * r * (1e-6f * c.bm * c.bn * a.K);
        if (best_cost == 0.0f || cost < best_cost) { best_cost = cost; best = c.kind; }
    }
    if ((forced == 384 || forced == 256 || forced == 128) && fits) best = forced;
    if (forced == 1) best = a.epi == EPI_SWIGLU ? 2 : 3;
    switch (best) {
        case 128: case 256: case 384: return launch_gemm_dma_bf16(best, a, amode, s);
        case 1: return launch_tile<bf16, 128, 128, 2, 2>(a, amode, s);
        case 2: return launch_tile<bf16, 64, 128, 2, 2>(a, amode, s);
        default: return launch_tile<bf16, 64, 64, 2, 2>(a, amode, s);
    }
}
}  // namespace vpe
