// 3x3 / pad 1 convolution on a channels-last grid as an implicit GEMM whose A operand is formed in LDS from a
// STRIP of input pixels (gfx950, bf16).
//
// The generic implicit GEMM (gemm_dma_kernel<.., A_CONV3>) fetches, for every one of the nine taps, a fresh
// BM x k-tile slice of the input from L2 into LDS: every input element enters LDS nine times per workgroup, and
// the direct-to-LDS load path is what limits that kernel.  Here a workgroup owns BM CONSECUTIVE pixels of the
// flattened (image, row, column) index; tap (dy, dx) of pixel p is pixel p + dy W + dx of the same flattened
// index, so all nine shifted operands live in one strip of BM + 2 W + 2 pixels, loaded ONCE per 16-channel chunk
// (3.1x fewer input bytes through the load path at BM = 384, W = 360; with the weights, which stream as before,
// 41 % fewer bytes in all).  What a flat shift gets wrong -- taps that leave the image on the left / right /
// top / bottom edge and would read the neighbouring row or image instead of zero padding -- is put right on the
// consumer side: each lane knows, for each of its accumulator row blocks, which of the nine taps are inside
// the image, and clears the fragment it has read otherwise (four v_and per fragment, in the shadow of the
// MFMAs).  Strip positions before the first / after the last pixel of the tensor are clamped to valid memory
// and always masked.
//
// k order: channel chunk (16 channels = one MFMA k-step) outer, tap row dy, tap column dx inner.  LDS:
//   strip   2 stages x SP pixels x 32 bytes   (SP = BM + 2 W + 2 rounded up to 32; stage c & 1 holds chunk c)
//   weights 2 stages x 3 taps x BN rows x 32 bytes (one tap row per step)
// One barrier per step (3 taps = 36 MFMAs per wave at a 96 x 128 wave tile); the loads of the next step's
// weights and a third of the next chunk's strip are issued right behind it.  Rows of both operands are 32 bytes,
// a lane's fragment is 16 of them and 32 consecutive lanes read 32 consecutive rows: every ds_read_b128 covers
// one contiguous kilobyte, no swizzle needed.
//
// Same GemmArgs, output maps and epilogues as the generic kernels (A_CONV3 conventions of gemm.h).
#pragma once
#include "gemm_dma.h"

namespace vpe {

constexpr int STRIP_KC = 16;              // channels per chunk = one MFMA k-step
constexpr int STRIP_MAX_SLOTS = 7;        // strip load instructions per wave and chunk (8 waves x 7 x 32 pixels = 1792 at most)

template <int BM, int BN, int WGM, int WGN, int OCC>
__global__ __launch_bounds__(64 * WGM * WGN, OCC * WGM * WGN / 4) void conv_strip_kernel(const GemmArgs args, int sp_rows) {
    const GemmArgs p = select_problem(args);
    constexpr int NW = WGM * WGN;
    static_assert(NW == 8 && BN == 32 * NW, "loader mapping: eight waves, each loads 32 weight rows per tap");
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int WTAP = BN * 32, WSTAGE = 3 * WTAP;     // bytes of one tap's weight tile / of one step's three
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    const int Wd = p.cW, HW = p.cH * p.cW, C = p.cC;

    int tm, tn;
    tile_coords(xcd_contiguous(blockIdx.x, gridDim.x), (p.M + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    const int strip_bytes = sp_rows * 32;
    char* const s_strip = smem;                         // [2][sp_rows][32]
    char* const s_w = smem + 2 * strip_bytes;           // [2][3][BN][32]

    const char* __restrict__ A = reinterpret_cast<const char*>(p.A);
    const char* __restrict__ Wt = reinterpret_cast<const char*>(p.W);

    // --- loader state.  Strip instruction `slot` (32 pixels): lane l fetches half l & 1 of the 32-byte chunk of strip
    // pixel 32 slot + l / 2, i.e. of flattened pixel m0 - W - 1 + that, clamped into the tensor.  The address is formed
    // per instruction (a dozen integer operations, seven times per chunk) rather than kept in seven registers.
    const int nslots = sp_rows / 32;
    const int qbase = m0 - Wd - 1 + (lane >> 1);
    const float inv_hw = 1.0f / (float)HW;
    auto strip_src = [&](int slot, int c) -> const char* {
        int q = qbase + 32 * slot;
        q = q < 0 ? 0 : (q < p.M ? q : p.M - 1);
        int img = (int)((float)q * inv_hw);              // q / HW, put right below (the product may be off by one ulp)
        img += (img + 1) * HW <= q;
        img -= img * HW > q;
        const int64_t row = (int64_t)img * p.a_istride + p.a_off + (q - img * HW);
        return A + (row * p.lda + c * STRIP_KC) * 2 + (lane & 1) * 16;
    };
    // weight rows: lane l fetches half l & 1 of row n0 + 32 wave + l / 2
    const int woff = (int)(((int64_t)(n0 + 32 * wave + (lane >> 1)) * p.K) * 2 + (lane & 1) * 16);

    // third `part` (0..2) of chunk c's strip into strip stage c & 1: slots i with i % 3 == part
    auto dma_strip = [&](int c, int part) {
        char* dst = s_strip + (c & 1) * strip_bytes;
#pragma unroll
        for (int i = 0; i < STRIP_MAX_SLOTS; ++i) {
            if (i % 3 != part) continue;
            const int slot = wave + NW * i;
            if (slot < nslots)
                __builtin_amdgcn_global_load_lds(VPE_GPTR(strip_src(slot, c)), VPE_LPTR(dst + slot * 1024), 16, 0, 0);
        }
    };
    // the three taps of row dy = tg - 1 for chunk c into weight stage `stage`
    auto dma_w = [&](int stage, int c, int tg) {
        char* dst = s_w + stage * WSTAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            __builtin_amdgcn_global_load_lds(VPE_GPTR(Wt + woff + (((tg * 3 + i) * C) + c * STRIP_KC) * 2), VPE_LPTR(dst + i * WTAP), 16, 0, 0);
    };

    // --- which taps stay inside the image, per accumulator row block of this lane: bit t = 3 (dy + 1) + dx + 1
    // (row block i in bits 9 i .. 9 i + 8 of one register)
    static_assert(MI <= 3, "nine bits per row block in one 32-bit register");
    uint32_t inside = 0;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        int r = m0 + wm * WM + i * 32 + li;
        r = r < p.M ? r : p.M - 1;
        const int pix = r % HW, y = pix / Wd, x = pix % Wd;
        uint32_t bits = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
            if (yy >= 0 && yy < p.cH && xx >= 0 && xx < Wd) bits |= 1u << t;
        }
        inside |= bits << (9 * i);
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // --- operand reads.  Strip row of accumulator row r for tap (tg, i): r + tg W + i (the strip starts W + 1
    // pixels before the tile); weight row n of tap i: i WTAP + 32 n.
    const int abase = (wm * WM + li) * 32 + g * 16, bbase = (wn * WN + li) * 32 + g * 16;
    auto compute = [&](const char* strip, const char* wts, int tg) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const char* sa = strip + abase + (tg * Wd + i) * 32;
            const char* sb = wts + bbase + i * WTAP;
            u32x4 fa[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) fa[mi] = *reinterpret_cast<const u32x4*>(sa + mi * 32 * 32);
            if (!(tg == 1 && i == 1)) {           // the centre tap is always inside
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    const uint32_t keep = 0u - ((inside >> (9 * mi + tg * 3 + i)) & 1u);
#pragma unroll
                    for (int e = 0; e < 4; ++e) fa[mi][e] &= keep;
                }
            }
            // weight fragments one column block at a time (the register file has no room for all four at once)
#pragma unroll
            for (int nj = 0; nj < NI; ++nj) {
                const bf16x8 fb = *reinterpret_cast<const bf16x8*>(sb + nj * 32 * 32);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[mi]), fb, acc[mi][nj], 0, 0, 0);
            }
        }
    };

    // --- main loop: step s = 3 c + tg.  Top of a step: everything this wave has in flight has landed (the current
    // step's weights, the strip third issued a step ago), barrier (everyone's has, and everyone is done with the
    // stages about to be overwritten), then the next step's weights and a third of the next chunk's strip.
    const int NC = C / STRIP_KC, NS = 3 * NC;
    dma_strip(0, 0);
    dma_strip(0, 1);
    dma_strip(0, 2);
    dma_w(0, 0, 0);
    for (int s = 0; s < NS; ++s) {
        const int c = s / 3, tg = s - 3 * c;
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();
        if (s + 1 < NS) dma_w((s + 1) & 1, (s + 1) / 3, (s + 1) % 3);
        if (c + 1 < NC) dma_strip(c + 1, tg);
        __builtin_amdgcn_sched_barrier(0);
        compute(s_strip + (c & 1) * strip_bytes, s_w + (s & 1) * WSTAGE, tg);
    }
    __syncthreads();                                     // the staging blocks of the epilogue overlay the operand buffers

    wave_tile_epilogue<MI, NI, WM, WN>(p, acc, smem, nullptr, wave, wm, wn, lane, m0, n0);
}

// Strip rows (pixels) a tile needs, rounded up to whole load instructions.
template <int BM>
static inline int strip_rows(int W) { return (int)rup(BM + 2 * W + 2, 32); }

// Can this convolution run on the strip kernel?  (bf16; whole 256-column tiles; 16-channel chunks; the strip of a
// tile within the per-wave load slots; 32-bit byte offsets.)
template <int BM, int BN>
static inline bool conv_strip_fits(const GemmArgs& a) {
    if (a.cC % STRIP_KC || a.N % BN || a.K != 9 * a.cC || a.ln_stats) return false;
    if (strip_rows<BM>(a.cW) > 8 * STRIP_MAX_SLOTS * 32) return false;
    const int64_t rows = (int64_t)(a.M / (a.cH * a.cW) + 1) * a.a_istride + a.a_off;
    return rows * a.lda * 2 < (int64_t(1) << 31) && (int64_t)(a.N + 256) * a.K * 2 < (int64_t(1) << 31);
}

template <int BM, int BN, int WGM, int WGN, int OCC>
static inline hipError_t launch_conv_strip(const GemmArgs& a, hipStream_t s, bool configure_only = false) {
    constexpr int epi_b = WGM * WGN * 32 * (BN / WGN) * 4;
    constexpr int max_lds = 160 * 1024 / OCC;
    static bool configured = false;
    if (!configured) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_strip_kernel<BM, BN, WGM, WGN, OCC>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (rc != hipSuccess) return rc;
        configured = true;
    }
    if (configure_only) return hipSuccess;
    if (!conv_strip_fits<BM, BN>(a)) return hipErrorInvalidValue;
    const int sp = strip_rows<BM>(a.cW);
    const int ops_b = 2 * sp * 32 + 2 * 3 * BN * 32;
    const int lds = ops_b > epi_b ? ops_b : epi_b;
    if (lds > max_lds) return hipErrorInvalidValue;
    const int tiles = cdiv(a.M, BM) * cdiv(a.N, BN), nz = a.nz > 1 ? a.nz : 1;
    hipLaunchKernelGGL((conv_strip_kernel<BM, BN, WGM, WGN, OCC>), dim3(tiles, nz), dim3(64 * WGM * WGN), lds, s, a, sp);
    return hipGetLastError();
}

}  // namespace vpe
