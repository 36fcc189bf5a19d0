// 3x3 / pad 1 convolution on a channels-last grid as an implicit GEMM whose A operand is formed in LDS from a
// STRIP of input pixels (gfx950, bf16).
//
// The generic implicit GEMM (gemm_dma_kernel<.., A_CONV3>) fetches, for every one of the nine taps, a fresh
// BM x k-tile slice of the input from L2 into LDS: every input element enters LDS nine times per workgroup, and
// the direct-to-LDS load path is what limits that kernel.  Here a workgroup owns BM CONSECUTIVE positions of a
// padded, flattened pixel index
//     P(image, y, x) = (image (H + 1) + y + 1) (W + 1) + x,      x = W and y = -1 (= y = H of the image before) are pads,
// in which tap (dy, dx) of position P is position P + dy (W + 1) + dx, whatever the pixel: one zero column behind
// every image row and one zero row between images are all the padding a 3x3 window can reach (left of x = 0 lies
// the pad column of the row above).  So all nine shifted operands of a tile live in one strip of
// BM + 2 (W + 1) + 2 positions, loaded ONCE per 16-channel chunk (3.1x fewer input bytes through the load path
// at BM = 384, W = 360; with the weights, which stream as before, 41 % fewer bytes in all), and the zero padding
// is made by the loader: a pad position fetches from a page of zeros.  The k loop has no masks and no special
// cases; the price is that pad positions are computed like pixels and thrown away (0.6 % at 272 x 360), and that
// tile rows are translated back to pixels in the epilogue.
//
// k order: channel chunk (16 channels = one MFMA k-step) outer, tap row dy, tap column dx inner.  LDS:
//   strip   2 stages x SP positions x 32 bytes   (SP = BM + 2 W + 4 rounded up to 32; stage c & 1 holds chunk c)
//   weights 3 stages x 3 taps x BN rows x 32 bytes (one tap row per step)
// One barrier per step (3 taps = 36 MFMAs per wave at a 96 x 128 wave tile).  Rows of both operands are 32 bytes and
// a lane's fragment is one 16-byte half of a row.  Stored plainly, the 16 lanes the LDS serves per cycle would sit
// 32 bytes apart and collide two by two on the 64 banks (measured: 2.8 conflict cycles per busy cycle), so the two
// halves of a row change places in every other group of eight rows: half g of row r sits at
//     32 r + 16 (g ^ ((r >> 3) & 1)).
// Rows r and r + 8 then fall into different 16-byte bank groups, for any run of 16 consecutive rows, i.e. for every
// tap shift; the loader makes the exchange by fetching the other half (adjacent lanes still fetch the two halves
// of one row).
//
// Same GemmArgs (M = pixels), output maps and epilogues as the generic kernels (A_CONV3 conventions of gemm.h).
#pragma once
#include "gemm_dma.h"

namespace vpe {

constexpr int STRIP_KC = 16;              // channels per chunk = one MFMA k-step
constexpr int STRIP_MAX_SLOTS = 7;        // strip load instructions per wave and chunk (8 waves x 7 x 32 positions = 1792 at most)

// Padded positions from the first pixel of the first image to the last pixel of the last one (tiles cover exactly
// this range: the leading pad row and whatever follows the last pixel are nobody's output).
static inline int64_t strip_positions(int images, int H, int W) { return ((int64_t)(images - 1) * (H + 1) + H) * (W + 1) - 1; }

// ROWDOT = true: the instantiation for EPI_ROWDOT alone.  Its MFMAs take the weights as the first operand, so a
// lane's accumulators are one pixel's channels (pixel = lane % 32, channel 8 (v / 4) + 4 (lane / 32) + v % 4 of the
// 32-channel block) and the projection over channels is a sum inside the lane plus one exchange between the lane
// halves (rowdot_epilogue_transposed).
template <int BM, int BN, int WGM, int WGN, int OCC, bool ROWDOT>
__global__ __launch_bounds__(64 * WGM * WGN, OCC * WGM * WGN / 4) void conv_strip_kernel(const GemmArgs args, int sp_rows, int tiles_m) {
    const GemmArgs p = select_problem(args);
    constexpr int NW = WGM * WGN;
    static_assert(NW == 8 && BN % 32 == 0, "loader mapping: eight waves; a weight load instruction takes 32 rows of a tap");
    constexpr int RB = BN / 32, WQ = 3 * RB, WPW = (WQ + NW - 1) / NW;   // row blocks per tap, weight instructions per step / per wave
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int WTAP = BN * 32, WSTAGE = 3 * WTAP;     // bytes of one tap's weight tile / of one step's three
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    const int Wp = p.cW + 1, Hp = p.cH + 1, C = p.cC;
    const int images = p.M / (p.cH * p.cW);

    int tm, tn;
    tile_coords(xcd_contiguous(blockIdx.x, gridDim.x), tiles_m, (p.N + BN - 1) / BN, tm, tn);
    const int m0 = Wp + tm * BM, n0 = tn * BN;            // position W + 1 is pixel (0, 0) of the first image

    const int strip_bytes = sp_rows * 32;
    char* const s_strip = smem;                         // [2][sp_rows][32]
    char* const s_w = smem + 2 * strip_bytes;           // [3][3][BN][32]

    const char* __restrict__ A = reinterpret_cast<const char*>(p.A);
    const char* __restrict__ Wt = reinterpret_cast<const char*>(p.W);
    const char* zpage = reinterpret_cast<const char*>(p.zeros);

    // --- loader.  Strip instruction `slot` (32 positions): lane l fetches one half of the 32-byte chunk of strip
    // position 32 slot + l / 2, i.e. of padded position m0 - (W + 1) - 1 + that: a pixel's channels, or zeros for a pad
    // and for positions outside the tensor.  Where a lane reads from does not depend on the chunk, so the byte offset of
    // its pixel (chunk 0) from A, or -1 for the page of zeros, is worked out once per instruction slot (two divisions by
    // reciprocal, about 45 instructions with eight slow multiplies) and kept in LDS, one word per lane and slot, read
    // back one MFMA group ahead of the load: done between the MFMAs of every chunk, that arithmetic alone cost 480 of
    // a step's 3750 clocks, and there are no seven registers to keep the offsets in.
    const int nslots = sp_rows / 32;
    int* const s_tab = reinterpret_cast<int*>(s_w + 3 * WSTAGE) + lane;        // [nslots][64]
    // weight rows: instruction q of a step (tap q / RB, row block q % RB) is issued by wave q % 8; lane l fetches row
    // n0 + 32 (q % RB) + l / 2, the same exchange of halves
    const int woff = (int)(((int64_t)(n0 + (lane >> 1)) * p.K) * 2 + (((lane & 1) ^ ((lane >> 4) & 1)) * 16));

    // the table entry of this wave's i-th strip instruction (i < STRIP_MAX_SLOTS); only the wave itself reads its entries
    auto strip_off = [&](int i) -> int {
        const int slot = wave + NW * i;
        return slot < nslots ? s_tab[slot * 64] : -1;
    };
    // this wave's i-th strip instruction of chunk c, into strip stage c & 1, from table entry `off`
    auto dma_strip1 = [&](int c, int i, int off) {
        const int slot = wave + NW * i;
        if (slot < nslots) {
            const char* src = off >= 0 ? A + off + c * (STRIP_KC * 2) : zpage;
            __builtin_amdgcn_global_load_lds(VPE_GPTR(src), VPE_LPTR(s_strip + (c & 1) * strip_bytes + slot * 1024), 16, 0, 0);
        }
    };
    // half `part` (0 / 1) of chunk c's strip: this wave's instructions with i % 2 == part
    auto dma_strip = [&](int c, int part) {
#pragma unroll
        for (int i = 0; i < STRIP_MAX_SLOTS; ++i)
            if ((i & 1) == part) dma_strip1(c, i, strip_off(i));
    };
    // this wave's j-th weight instruction (j < WPW) of tap row dy = tg - 1 for chunk c into weight stage `stage`
    auto dma_w1 = [&](int stage, int c, int tg, int j) {
        const int q = wave + NW * j;
        if (q < WQ) {
            const int tap = q / RB, rb = q % RB;
            __builtin_amdgcn_global_load_lds(VPE_GPTR(Wt + woff + (int)((int64_t)rb * 32 * p.K * 2) + (((tg * 3 + tap) * C) + c * STRIP_KC) * 2),
                                             VPE_LPTR(s_w + stage * WSTAGE + tap * WTAP + rb * 1024), 16, 0, 0);
        }
    };
    auto dma_w = [&](int stage, int c, int tg) {
#pragma unroll
        for (int j = 0; j < WPW; ++j) dma_w1(stage, c, tg, j);
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // --- operand reads.  Strip row of tile row r for tap (tg, i): r + tg (W + 1) + i (the strip starts W + 2
    // positions before the tile); weight row n of tap i: i WTAP + 32 n.
    // One step = the three taps of a tap row = 9 (tap, row block) groups of NI MFMAs.  Weight fragments of a tap stay
    // in registers for its three row blocks (16 registers) and are re-read for the next tap one by one, each right
    // behind its last MFMA; strip fragments are double-buffered one group ahead (2 x 4 registers).  The weights sit in
    // THREE stages, so the operands of step s + 1 are complete and visible a whole step early and the last group of
    // step s reads the first fragments of step s + 1: the MFMA stream runs through the step boundary and its barrier.
    const int arow = wm * WM + li, bbase = (wn * WN + li) * 32 + ((g ^ ((li >> 3) & 1)) << 4);
    static_assert(WPW <= 3, "weight loads go with the first groups of a step");
    auto aoff = [&](int row) { return (row << 5) + ((g ^ ((row >> 3) & 1)) << 4); };   // LDS offset of this lane's half of strip row `row`
    bf16x8 fb[NI], fa[2];
    // The step's loads (next-but-one step's weights: lw_* ; half of the next chunk's strip: ls_*) are issued one
    // instruction per group, between the MFMAs: eight waves issuing all of theirs at once right behind the barrier
    // queue up at the CU's one address unit, and a wave stuck at issue starts no MFMA either.
    auto compute = [&](const char* strip, const char* wts, int tg, const char* nstrip, const char* nwts, int ntg, bool more,
                       bool lw, int lw_stage, int lw_c, int lw_tg, bool ls, int ls_c, int ls_part) {
        const char* sa[3] = {strip + aoff(arow + tg * Wp), strip + aoff(arow + tg * Wp + 1), strip + aoff(arow + tg * Wp + 2)};
        const char* sb = wts + bbase;
        int soff = -1;
        const char* na = nstrip + aoff(arow + ntg * Wp);
        const char* nb = nwts + bbase;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int cur = (i * MI + mi) & 1;
                const bool last = i == 2 && mi == MI - 1;
                if (mi + 1 < MI) fa[cur ^ 1] = *reinterpret_cast<const bf16x8*>(sa[i] + (mi + 1) * 1024);
                else if (i < 2) fa[cur ^ 1] = *reinterpret_cast<const bf16x8*>(sa[i + 1]);
                else if (more) fa[cur ^ 1] = *reinterpret_cast<const bf16x8*>(na);
                const int k = i * MI + mi;                // group 0..8: weights in groups 0..2, strip instructions in 3..6
                if (k < WPW) { if (lw) dma_w1(lw_stage, lw_c, lw_tg, k); }
                else if (k >= 3 && k - 3 < (STRIP_MAX_SLOTS + 1) / 2) { if (ls) dma_strip1(ls_c, 2 * (k - 3) + ls_part, soff); }
                if (k >= 2 && k - 2 < (STRIP_MAX_SLOTS + 1) / 2) { if (ls) soff = strip_off(2 * (k - 2) + ls_part); }   // for the next group
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nj = 0; nj < NI; ++nj) {
                    acc[mi][nj] = ROWDOT ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[nj], fa[cur], acc[mi][nj], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur], fb[nj], acc[mi][nj], 0, 0, 0);
                    if (mi == MI - 1 && i < 2) fb[nj] = *reinterpret_cast<const bf16x8*>(sb + (i + 1) * WTAP + nj * 1024);
                    if (last && more) fb[nj] = *reinterpret_cast<const bf16x8*>(nb + nj * 1024);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        static_assert((3 * MI) % 2 == 1, "nine groups per step: the last one prefetches into the odd buffer");
        fa[0] = fa[1];                                   // the next step starts on the even buffer again
    };

    // --- main loop: step s = 3 c + tg.  Top of a step: this wave's loads for step s + 1 have landed, barrier (everyone's
    // have, and everyone is done with step s - 1), then the loads of step s + 2's weights (into the stage step s - 1
    // used) and, in the first two steps of a chunk, half of the next chunk's strip (into the stage chunk c - 1 used).
    const int NC = C / STRIP_KC, NS = 3 * NC;
    dma_w(0, 0, 0);                                      // (the first weights are on their way while the offsets are worked out)
    dma_w(1, 0, 1);
    {
        const int qbase = m0 - Wp - 1 + (lane >> 1);          // lane l: row l / 2 of the instruction's 32, physical half l % 2
        const int lhalf = ((lane & 1) ^ ((lane >> 4) & 1)) * 16;   // ... which holds this logical half (rows 8..15, 24..31 exchanged)
        const float inv_wp = 1.0f / (float)Wp, inv_hp = 1.0f / (float)Hp;
        for (int slot = wave; slot < nslots; slot += NW) {
            const int q = qbase + 32 * slot;
            const int qq = q < 0 ? 0 : q;
            int line = (int)((float)qq * inv_wp);            // qq / Wp, put right below (the product may be off by one)
            line += (line + 1) * Wp <= qq;
            line -= line * Wp > qq;
            const int x = qq - line * Wp;
            int img = (int)((float)line * inv_hp);
            img += (img + 1) * Hp <= line;
            img -= img * Hp > line;
            const int y = line - img * Hp - 1;
            const bool pixel = q >= 0 && x < p.cW && y >= 0 && img < images;
            const int64_t row = (int64_t)img * p.a_istride + p.a_off + y * p.cW + x;
            s_tab[slot * 64] = pixel ? (int)(row * p.lda * 2 + lhalf) : -1;
        }
    }
    dma_strip(0, 0);
    dma_strip(0, 1);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
#pragma unroll
    for (int nj = 0; nj < NI; ++nj) fb[nj] = *reinterpret_cast<const bf16x8*>(s_w + bbase + nj * 1024);
    fa[0] = *reinterpret_cast<const bf16x8*>(s_strip + aoff(arow));
    int wst = 0;                                         // weight stage of step s (s % 3)
    for (int s = 0; s < NS; ++s) {
        const int c = s / 3, tg = s - 3 * c;
        if (s > 0) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __syncthreads();
        }
        const int nst = wst == 2 ? 0 : wst + 1, nc = (s + 1) / 3, ntg = (s + 1) - 3 * nc;
        compute(s_strip + (c & 1) * strip_bytes, s_w + wst * WSTAGE, tg, s_strip + (nc & 1) * strip_bytes, s_w + nst * WSTAGE, ntg, s + 1 < NS,
                s + 2 < NS, wst == 0 ? 2 : wst - 1, (s + 2) / 3, (s + 2) % 3, c + 1 < NC && tg < 2, c + 1, tg);
        wst = nst;
    }
    __syncthreads();                                     // the staging blocks of the epilogue overlay the operand buffers

    if constexpr (ROWDOT) {
        rowdot_epilogue_transposed<MI, NI, WM, WN, BN, 64 * NW, true>(p, acc, smem, wm, wn, tid, m0, n0);
    } else {
        wave_tile_epilogue<MI, NI, WM, WN, true>(p, acc, smem, nullptr, wave, wm, wn, lane, m0, n0);
    }
}

// Strip rows (positions) a tile needs, rounded up to whole load instructions.
template <int BM>
static inline int strip_rows(int W) { return (int)rup(BM + 2 * (W + 1) + 2, 32); }

// Can this convolution run on the strip kernel?  (bf16; whole BN-column tiles; 16-channel chunks; whole images; the
// strip of a tile within the per-wave load slots and, with the weights, within the LDS; 32-bit byte offsets.)
template <int BM, int BN>
static inline bool conv_strip_fits(const GemmArgs& a) {
    if (a.cC % STRIP_KC || a.N % BN || a.K != 9 * a.cC || a.ln_stats || !a.zeros) return false;
    if (a.cH < 1 || a.cW < 1 || a.M % (a.cH * a.cW)) return false;
    const int sp = strip_rows<BM>(a.cW);
    if (sp > 8 * STRIP_MAX_SLOTS * 32 || 2 * sp * 32 + 3 * 3 * BN * 32 + sp * 8 > 160 * 1024) return false;   // strips, weights, offset table
    if (strip_positions(a.M / (a.cH * a.cW), a.cH, a.cW) + BM >= (int64_t(1) << 31)) return false;
    const int64_t rows = (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride + a.a_off;
    return rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
}

template <int BM, int BN, int WGM, int WGN, int OCC, bool ROWDOT>
static inline hipError_t launch_conv_strip(const GemmArgs& a, hipStream_t s, bool configure_only = false) {
    constexpr int epi_b = WGM * WGN * 32 * (BN / WGN) * 4;
    constexpr int max_lds = 160 * 1024 / OCC;
    static bool configured = false;
    if (!configured) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_strip_kernel<BM, BN, WGM, WGN, OCC, ROWDOT>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (rc != hipSuccess) return rc;
        configured = true;
    }
    if (configure_only) return hipSuccess;
    if (!conv_strip_fits<BM, BN>(a) || ROWDOT != (a.epi == EPI_ROWDOT)) return hipErrorInvalidValue;
    const int sp = strip_rows<BM>(a.cW);
    const int ops_b = 2 * sp * 32 + 3 * 3 * BN * 32 + sp * 8;
    const int lds = ops_b > epi_b ? ops_b : epi_b;
    if (lds > max_lds) return hipErrorInvalidValue;
    const int tiles_m = (int)((strip_positions(a.M / (a.cH * a.cW), a.cH, a.cW) + BM - 1) / BM);
    const int tiles = tiles_m * cdiv(a.N, BN), nz = a.nz > 1 ? a.nz : 1;
    hipLaunchKernelGGL((conv_strip_kernel<BM, BN, WGM, WGN, OCC, ROWDOT>), dim3(tiles, nz), dim3(64 * WGM * WGN), lds, s, a, sp, tiles_m);
    return hipGetLastError();
}

}  // namespace vpe
