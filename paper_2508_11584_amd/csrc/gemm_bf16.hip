// bf16-operand instantiations of the register-staged MFMA GEMM, and the choice between them and
// the large-tile direct-to-LDS kernel.
#include <cstdlib>

#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s);

namespace {
// Candidate tilings with the number of workgroups a 256-CU chip holds at once and a relative
// efficiency per unit of tile area, from measurements on MI355X (3x3 conv 256->256 on 272x360 and on
// grids that give whole rounds; M=10992 N=8192 K=1536).  `q` is per unit of area at equal slot counts, so
// the one-workgroup-per-CU shapes (256 slots) carry twice the per-CU figure: 2 x 1.18.  The small register-
// staged tiles are latency-bound, their factors only rank them.
struct Cand { int kind, bm, bn, slots; float q; };
constexpr Cand kCands[] = {
    {128, 256, 128, 512, 1.00f},   // direct-to-LDS, two workgroups per CU
    {256, 256, 256, 256, 2.36f},   // direct-to-LDS, 64 x 128 wave tiles, one workgroup per CU
    {384, 384, 256, 256, 2.36f},   // direct-to-LDS, 96 x 128 wave tiles, one workgroup per CU
    {1, 128, 128, 512, 0.82f},     // register-staged
    {2, 64, 128, 768, 0.40f},
    {3, 64, 64, 1024, 0.30f},
};
}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s) {
    const char* env = getenv("VPE_GEMM_TILE");
    const int forced = env ? atoi(env) : 0;
    // the direct-to-LDS loader keeps byte offsets in 32-bit ints
    const int64_t a_rows = amode == A_PLAIN ? (int64_t)(a.M / a.a_rpi + 1) * (a.a_istride > a.a_rpi ? a.a_istride : a.a_rpi)
                                            : (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride;
    const bool fits = a_rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
    // estimated time = rounds of resident workgroups (at least 1) x tile area / efficiency
    int best = 3;
    float best_cost = 0.0f;
    for (const Cand& c : kCands) {
        if (c.kind >= 128 && !fits) continue;
        if (c.kind == 3 && a.epi == EPI_SWIGLU) continue;       // needs 64-column wave tiles
        const int64_t tiles = (int64_t)cdiv(a.M, c.bm) * cdiv(a.N, c.bn) * (a.nz > 1 ? a.nz : 1);
        // several workgroups per CU do not run in lockstep (measured times grow linearly with tiles / slots);
        // one workgroup per CU does: a partly filled round costs a whole one
        float rounds = tiles > c.slots ? (float)tiles / c.slots : 1.0f;
        if (c.slots == 256) rounds = (float)cdiv(tiles, c.slots);
        const float cost = rounds * c.bm * c.bn / c.q;
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
