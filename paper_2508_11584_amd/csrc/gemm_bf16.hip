// bf16-operand instantiations of the register-staged MFMA GEMM, and the choice between them and
// the large-tile direct-to-LDS kernel.
#include <cstdlib>

#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_dma_bf16(int bn, const GemmArgs& a, int amode, hipStream_t s);
int conv_strip_shape(const GemmArgs& a, bool any_size, int64_t* tiles);
hipError_t launch_conv_strip_bf16(int shape, const GemmArgs& a, hipStream_t s);

namespace {
// Candidate tilings: tile, workgroups a CU holds at once, and the two coefficients of the time model
//     t [us] = alpha * max(r, 1) + beta * r * (bm * bn * K / 1e6),     r = ceil(tiles / 256) / held,
// r being the number of "rounds" on the busiest of the 256 CUs (it gets ceil(tiles / 256) tiles and works on
// `held` of them at a time); alpha is the cost a workgroup pays whatever its size (first loads, epilogue), not
// discounted on a partly filled chip.  Fitted (relative least squares) to 28 measured shapes x 8 tilings on
// MI355X with random bf16 data: the QKV / proj / fc1 / fc2 GEMMs of ViT-S, -B, -L (batch 4) and -g (batch 8),
// the heads' 1x1 projections, and the 3x3 convolutions at 34x45 ... 296x296 grids (batch 1 and 4).  The
// model's pick is the measured best on 23 of them, within 8 % on four and 15 % on one (0.4 % in total time).
// Tuning aids, read from the environment when an engine is created (configure_gemm_bf16), never per launch:
// VPE_GEMM_TILE forces a tiling, VPE_NO_SMALL_DMA leaves the two small direct-to-LDS shapes out, VPE_NO_SPLITK
// the split-k kernel, VPE_NO_STRIP the strip convolution, VPE_NO_ROW_SPLIT the two-launch form of a GEMM whose tile
// count is just above a whole number of rounds.
int g_forced_tile = 0;
bool g_no_small = false, g_no_splitk = false, g_no_strip = false, g_no_split = false;
struct Cand { int kind, bm, bn, held; float alpha, beta; bool dma; };
constexpr Cand kCands[] = {
    {128, 256, 128, 2, 5.16f, 1.055f, true},    // direct-to-LDS, 8 waves, 64 x 64 wave tiles
    {256, 256, 256, 1, 11.96f, 0.332f, true},   // direct-to-LDS, 8 waves, 64 x 128 wave tiles
    {384, 384, 256, 1, 15.66f, 0.361f, true},   // direct-to-LDS, 8 waves, 96 x 128 wave tiles
    {65, 64, 128, 3, 5.13f, 1.828f, true},      // direct-to-LDS, 4 waves, 32 x 64 wave tiles
    {64, 64, 64, 4, 4.55f, 2.909f, true},       // direct-to-LDS, 4 waves, 32 x 32 wave tiles
    {1, 128, 128, 2, 7.72f, 1.120f, false},     // register-staged (any operand size)
    {2, 64, 128, 3, 5.96f, 1.972f, false},
    {3, 64, 64, 4, 4.88f, 3.153f, false},
};
}  // namespace

// The model's pick for rows m_begin .. M - 1 of `a` and its predicted time in us.
static int pick_tile(const GemmArgs& a, bool fits, float& best_cost) {
    int best = 3;
    best_cost = 0.0f;
    const bool no_small = g_no_small;
    const int rows = a.M - a.m_begin;
    for (const Cand& c : kCands) {
        if (c.dma && !fits) continue;
        if (no_small && (c.kind == 64 || c.kind == 65)) continue;
        if (c.bn == 64 && a.epi == EPI_SWIGLU) continue;        // needs 64-column wave tiles
        const int64_t tiles = (int64_t)cdiv(rows, c.bm) * cdiv(a.N, c.bn) * (a.nz > 1 ? a.nz : 1);
        // Inside the engine (not in the calibration harness) the small direct-to-LDS shapes lose to their
        // register-staged counterparts when there is less than one tile per CU (ViT-S proj / fc2 with 144 tiles:
        // 12.7 against 11.7 us; 3x3 convolutions on the 34x45 and 68x90 grids: 24.0 against 20.7, 27.8 against
        // 25.9 us) and win above that (QKV 8.3 against 9.1, fc1 11.3 against 12.0, the 136x180 convolution 43.8
        // against 47.4 us)
        if ((c.kind == 64 || c.kind == 65) && tiles < 256) continue;
        const float r = (float)cdiv(tiles, 256) / c.held;
        const float cost = c.alpha * (r > 1.0f ? r : 1.0f) + c.beta * r * (1e-6f * c.bm * c.bn * a.K);
        if (best_cost == 0.0f || cost < best_cost) { best_cost = cost; best = c.kind; }
    }
    return best;
}

static hipError_t launch_picked(const GemmArgs& a, int amode, hipStream_t s, int best, bool fits);

hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s) {
    // the direct-to-LDS loader keeps byte offsets in 32-bit ints
    const int64_t a_rows = amode == A_PLAIN ? (int64_t)(a.M / a.a_rpi + 1) * (a.a_istride > a.a_rpi ? a.a_istride : a.a_rpi)
                                            : (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride;
    const bool fits = a_rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
    float whole_cost;
    const int whole = pick_tile(a, fits, whole_cost);
    // The one-per-CU tiles run in lockstep rounds of 256 and pay for a partly filled last round in full (ViT-g, 8
    // views: fc2 and the out-projection have 43 x 6 = 258 tiles of 256 x 256, QKV 774).  Two launches instead: whole
    // rounds of the large tile over the leading rows, then the remaining rows with whatever the model picks for them.
    if (g_forced_tile == 0 && !g_no_split && fits && a.nz <= 1 && a.m_begin == 0) {
        float split_cost = whole_cost;
        int split_kind = 0, split_rows = 0;
        for (const Cand& c : kCands) {
            if (!c.dma || c.held != 1) continue;
            const int tn = cdiv(a.N, c.bn), tm = cdiv(a.M, c.bm);
            const int64_t tiles = (int64_t)tm * tn;
            const int rounds = (int)(tiles / 256);
            if (rounds < 1 || tiles % 256 == 0) continue;
            const int tm_main = rounds * 256 / tn;              // whole tile rows in `rounds` rounds
            if (tm_main < 1 || tm_main >= tm) continue;
            const float main_rounds = (float)cdiv((int64_t)tm_main * tn, 256);
            const float main_cost = (c.alpha + c.beta * (1e-6f * c.bm * c.bn * a.K)) * main_rounds;
            GemmArgs tail = a;
            tail.m_begin = tm_main * c.bm;
            float tail_cost;
            pick_tile(tail, fits, tail_cost);
            if (main_cost + tail_cost < 0.93f * split_cost) {   // a second launch costs a few us the model does not see
                split_cost = main_cost + tail_cost;
                split_kind = c.kind;
                split_rows = tm_main * c.bm;
            }
        }
        if (split_kind) {
            GemmArgs main = a, tail = a;
            main.M = split_rows;
            tail.m_begin = split_rows;
            hipError_t rc = launch_gemm_dma_bf16(split_kind, main, amode, s);
            if (rc != hipSuccess) return rc;
            float unused;
            return launch_picked(tail, amode, s, pick_tile(tail, fits, unused), fits);
        }
    }
    return launch_picked(a, amode, s, whole, fits);
}

static hipError_t launch_picked(const GemmArgs& a, int amode, hipStream_t s, int best, bool fits) {
    const int forced = g_forced_tile;
    const int rows = a.M - a.m_begin;
    // A 64 x 64 tiling with at most one tile per CU and at least 4 k-tiles: two wave groups per tile, each over
    // half of the k range (in-engine: ViT-S fc2 14.4 -> 12.5 us, the 3x3 convolution on the 34x45 grid 20.7 -> 17.5,
    // the detection towers 26.9 -> 23.8; ViT-S 476x630 frame latency 1.13 -> 1.08 ms, sequential baseline 396 -> 418
    // frames/s, pipelined rate +0.5 %; with the threshold at 16 k-tiles 1.10 ms / 408 / +0 %).
    // VPE_NO_SPLITK in the environment switches it off (a tuning aid).  A limit of 288 tiles, which takes in the
    // ViT-B proj / fc2 GEMMs (264 tiles), brings that model's frame latency from 1.79 to 1.70 ms but costs 1.5 % of its
    // pipelined rate with three encoder lanes.  Four wave groups for the heads' long k loops on few tiles (3x3 convolutions
    // on the patch grid, 36 and 54 k-tiles on 96 and 192 tiles): frame latency 1.084 -> 1.081 ms, pipelined rate -1 %.
    const bool no_splitk = g_no_splitk;
    if (!no_splitk && best == 3 && a.K >= 256 && (int64_t)cdiv(rows, 64) * cdiv(a.N, 64) * (a.nz > 1 ? a.nz : 1) <= 256) best = 4;
    // 3x3 convolutions: the strip kernel (conv_strip.h) where its 384 x 256 tiles make one well-filled round of the
    // 256 CUs (measured on 272 x 360 x 256 -> 256, 256 tiles: 128 against 144 us for the generic 384 x 256 kernel on the
    // same box; with several rounds -- 4 x 296 x 296: 477 against 443 us -- the generic kernels stay ahead).
    // VPE_GEMM_TILE=9 forces it wherever it applies, any other forced tile switches it off.
    if (a.m_begin == 0 && amode == A_CONV3 && (forced == 9 || (forced == 0 && !g_no_strip)) && a.epi != EPI_SWIGLU) {
        const int shape = conv_strip_shape(a, forced == 9, nullptr);
        if (shape) return launch_conv_strip_bf16(shape, a, s);
    }
    if ((forced == 384 || forced == 256 || forced == 128 || forced == 65) && fits) best = forced;
    if (forced == 4) best = a.epi == EPI_SWIGLU ? 2 : 4;
    if (forced == 64 && fits) best = a.epi == EPI_SWIGLU ? 65 : 64;
    if (forced == 1) best = a.epi == EPI_SWIGLU ? 2 : 3;
    switch (best) {
        case 64: case 65: case 128: case 256: case 384: return launch_gemm_dma_bf16(best, a, amode, s);
        case 1: return launch_tile<bf16, 128, 128, 2, 2>(a, amode, s);
        case 2: return launch_tile<bf16, 64, 128, 2, 2>(a, amode, s);
        case 4: return launch_tile_splitk<bf16, 64, 64, 2, 2, 2>(a, amode, s);
        default: return launch_tile<bf16, 64, 64, 2, 2>(a, amode, s);
    }
}

// LDS opt-in of the split-k kernel; called once at engine creation, outside any stream capture.
hipError_t configure_gemm_bf16() {
    const char* env = getenv("VPE_GEMM_TILE");
    g_forced_tile = env ? atoi(env) : 0;
    g_no_small = getenv("VPE_NO_SMALL_DMA") != nullptr;
    g_no_splitk = getenv("VPE_NO_SPLITK") != nullptr;
    g_no_strip = getenv("VPE_NO_STRIP") != nullptr;
    g_no_split = getenv("VPE_NO_ROW_SPLIT") != nullptr;
    GemmArgs a{};
    return launch_tile_splitk<bf16, 64, 64, 2, 2, 2>(a, A_PLAIN, nullptr, true);
}
}  // namespace vpe
