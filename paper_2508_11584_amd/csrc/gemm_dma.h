// Large-tile MFMA GEMM for gfx950 with direct global->LDS loads (global_load_lds_dwordx4).
//
// Why a second kernel: on MI355X the register-staged 128 x 128 tiles stop at 750-840 TFLOP/s: the
// LDS write path (ds_write_b128 at ~80 bytes per clock per CU) and the global-load issue rate of
// 8 waves cannot keep four MFMA pipes fed at 64 FLOP per loaded byte.  Here a workgroup owns a
// 256 x BN tile (BN = 128 or 256), operands go from global memory straight into the swizzled LDS
// tile (global_load_lds_dwordx4: no VGPR staging, no ds_write), the next k-tile's loads are issued
// before the current tile's MFMAs, the LDS reads of k-step s + 1 are interleaved with the MFMAs of
// step s (sched_group_barrier), and the accumulators leave through a per-wave LDS staging block
// with 16-byte coalesced stores.  Measured: with the loads switched off the loop runs at 88 % of
// the MFMA rate; the loads are the limit, and their rate grows with the number of waves issuing
// them (4 waves: 670, 8 waves: 880, 16 waves per CU: 910-970 TFLOP/s on the 3x3 conv).
//
// Same operands, A modes and epilogues as gemm_kernel (see gemm.h); bf16 only.
#pragma once
#include <type_traits>

#include "gemm.h"

namespace vpe {

#define VPE_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define VPE_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// Epilogue of the wave-tiled kernels: each wave stages its MI x NI accumulator blocks 32 rows at a time in its own
// 32 x WN fp32 block of LDS (the operand buffers are free by now; the caller has put a barrier behind its last
// read of them) and leaves with 8-column chunks per lane.  lnrow: (mean, rstd) per tile row for GEMMs with a
// folded LayerNorm (ignored otherwise).
// Row index of a tile row in the output.  PADDED (the strip convolution): tile rows run over the padded pixel index
// ((image (H + 1) + y + 1) (W + 1) + x: one zero column behind every image row, one zero row between images); pad
// positions have no output (returned as a row past M).
template <bool PADDED>
__device__ __forceinline__ int epilogue_row(const GemmArgs& p, int r) {
    if (!PADDED) return r;
    const int wp = p.cW + 1, hp = p.cH + 1;
    const int line = r / wp, x = r - line * wp;
    const int img = line / hp, y = line - img * hp - 1;
    return (x < p.cW && y >= 0) ? (img * p.cH + y) * p.cW + x : 0x7fffffff;
}

// The same map for tile rows visited in increasing order with a fixed step: one pair of divisions at the start, then
// additions and compares (a ROWDOT lane visits every 64 / CG-th row of its wave tile).
template <bool PADDED>
struct EpilogueRows {
    int r, x, y, img, wp, hp;          // tile row; PADDED: its column, line within the image's H + 1 lines, image
    __device__ __forceinline__ EpilogueRows(const GemmArgs& p, int r0) : r(r0), x(0), y(0), img(0), wp(p.cW + 1), hp(p.cH + 1) {
        if (PADDED) {
            const int line = r0 / wp;
            x = r0 - line * wp;
            img = line / hp;
            y = line - img * hp;
        }
    }
    __device__ __forceinline__ int row(const GemmArgs& p) const {
        if (!PADDED) return r;
        return (x < p.cW && y >= 1) ? (img * p.cH + y - 1) * p.cW + x : 0x7fffffff;
    }
    __device__ __forceinline__ void advance(int step) {
        r += step;
        if (PADDED) {
            x += step;
            while (x >= wp) {
                x -= wp;
                if (++y == hp) { y = 0; ++img; }
            }
        }
    }
};

template <int MI, int NI, int WM, int WN, bool PADDED = false>
__device__ __forceinline__ void wave_tile_epilogue(const GemmArgs& p, f32x16 (&acc)[MI][NI], char* smem, const float* lnrow,
                                                   int wave, int wm, int wn, int lane, int m0, int n0) {
    typedef bf16 T;
    const int g = lane >> 5, li = lane & 31;
    float* sC = reinterpret_cast<float*>(smem) + wave * (32 * WN);
    const int wrow0 = m0 + wm * WM, wcol0 = n0 + wn * WN;
    // ROWDOT: a lane keeps one 8-column chunk (lane % CG) for all its rows -- its bias and projection values are
    // loaded once -- and visits rows lane / CG, + 64 / CG, ... of the wave tile in order, across the passes
    constexpr int RD_CG = WN / 8;
    f32x4 rd_b0 = {0, 0, 0, 0}, rd_b1 = rd_b0, rd_w0 = rd_b0, rd_w1 = rd_b0;
    EpilogueRows<PADDED> rd_rows(p, wrow0 + lane / RD_CG);
    const int rd_c = wcol0 + (lane % RD_CG) * 8;
    if (p.epi == EPI_ROWDOT && rd_c < p.N) {
        rd_b0 = *reinterpret_cast<const f32x4*>(p.bias + rd_c);
        rd_b1 = *reinterpret_cast<const f32x4*>(p.bias + rd_c + 4);
        rd_w0 = *reinterpret_cast<const f32x4*>(p.gamma + rd_c);
        rd_w1 = *reinterpret_cast<const f32x4*>(p.gamma + rd_c + 4);
    }
    // one pass per 32-row block of the wave tile; the block index is a compile-time constant of each pass (a
    // loop that the optimizer declines to unroll would turn the accumulators into an indexed array in scratch)
    auto pass = [&](auto I) {
        constexpr int i = decltype(I)::value;
        if (p.ln_stats) {
            // (column sums are loaded here, not before the k loop: this kernel has no registers to spare)
            float lncs[NI];
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int c = wcol0 + j * 32 + li;
                lncs[j] = c < p.N ? p.ln_colsum[c] : 0.0f;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * WM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                const f32x2 st = *reinterpret_cast<const f32x2*>(lnrow + 2 * row);
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j][v] = st[1] * (acc[i][j][v] - st[0] * lncs[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sC[(8 * (v >> 2) + 4 * g + (v & 3)) * WN + j * 32 + li] = acc[i][j][v];
        const int rblk = wrow0 + i * 32;
        if (p.epi == EPI_SWIGLU) {
            // groups of 64 physical columns: 32 gate columns, then their 32 linear partners
            constexpr int CG = WN / 16;                  // 8-wide gate chunks per row
            T* out = reinterpret_cast<T*>(p.out);
            for (int it = lane; it < 32 * CG; it += 64) {
                const int rr = it / CG, cg = it % CG, grp = cg >> 2, j0 = (cg & 3) * 8;
                const int r = epilogue_row<PADDED>(p, rblk + rr), ca = wcol0 + grp * 64 + j0;
                if (r < p.M && ca + 40 <= p.N) {
                    const float* src = sC + rr * WN + grp * 64 + j0;
                    float h[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float a = src[e] + p.bias[ca + e], b = src[32 + e] + p.bias[ca + 32 + e];
                        h[e] = swiglu_for<T>(a, b);
                    }
                    store8(out + (int64_t)r * p.ldo + (ca >> 6) * 32 + j0, h);
                }
            }
        } else if (p.epi == EPI_QKV && wcol0 >= 2 * p.dim) {
            // value columns, written transposed: one column and 8 consecutive tokens per lane
            T* vt = reinterpret_cast<T*>(p.out2);
            for (int it = lane; it < WN * 4; it += 64) {
                const int cc = it >> 2, rr = (it & 3) * 8;      // 4 lanes = 32 consecutive tokens of a column
                const int r = epilogue_row<PADDED>(p, rblk + rr), c2 = wcol0 + cc - 2 * p.dim;
                if (r < p.M && wcol0 + cc < p.N) {
                    const float bias = p.bias[wcol0 + cc];
                    float v[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = sC[(rr + k) * WN + cc] + bias;
                    store_tokens8<T>(p, vt, r, c2, v);
                }
            }
        } else if ((p.epi == EPI_RESID || p.epi == EPI_PATCH) && (p.st_out || p.xb_out)) {
            // 8 consecutive lanes hold the 8 chunks of one 64-column statistics group of a row
            if constexpr (WN % 64 == 0) {
                constexpr int CG = WN / 8;
#pragma unroll
                for (int it = lane; it < 32 * CG; it += 64) {
                    const int rr = it / CG, cg = it % CG;
                    const int r = epilogue_row<PADDED>(p, rblk + rr), c = wcol0 + cg * 8;
                    const bool active = r < p.M && c < p.N;
                    float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (active) {
                        const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * WN + cg * 8);
                        const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * WN + cg * 8 + 4);
                        v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
                        v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
                    }
                    resid_stats_chunk<T>(p, r, c, v, active, cg & 7);
                }
            }
        } else if (p.epi == EPI_ROWDOT) {
            // 8 consecutive lanes hold the 8 chunks of one 64-column projection group of a row
            if constexpr (WN % 64 == 0) {
                constexpr int CG = RD_CG;
                static_assert(64 % CG == 0, "a lane keeps its column chunk");
                float* out = reinterpret_cast<float*>(p.out);
#pragma unroll
                for (int n = 0; n < 32 * CG / 64; ++n) {
                    const int rr = lane / CG + n * (64 / CG);
                    const int r = rd_rows.row(p);
                    rd_rows.advance(64 / CG);
                    const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * WN + (lane % CG) * 8);
                    const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * WN + (lane % CG) * 8 + 4);
                    float sum = 0.0f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float a = lo[e] + rd_b0[e], b = hi[e] + rd_b1[e];
                        if (p.act == ACT_RELU) { a = fmaxf(a, 0.0f); b = fmaxf(b, 0.0f); }
                        sum += a * rd_w0[e] + b * rd_w1[e];
                    }
                    sum += __shfl_xor(sum, 1);
                    sum += __shfl_xor(sum, 2);
                    sum += __shfl_xor(sum, 4);
                    if ((lane & 7) == 0 && r < p.M && rd_c < p.N) out[(int64_t)r * p.ldo + (rd_c >> 6)] = sum;
                }
            }
        } else {
            constexpr int CG = WN / 8;
            for (int it = lane; it < 32 * CG; it += 64) {
                const int rr = it / CG, cg = it % CG;
                const int r = epilogue_row<PADDED>(p, rblk + rr), c = wcol0 + cg * 8;
                if (r < p.M && c < p.N) {
                    const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * WN + cg * 8);
                    const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * WN + cg * 8 + 4);
                    float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    epilogue_chunk<T>(p, r, c, v);
                }
            }
        }
    };
    pass(std::integral_constant<int, 0>{});
    if constexpr (MI > 1) pass(std::integral_constant<int, 1>{});
    if constexpr (MI > 2) pass(std::integral_constant<int, 2>{});
    if constexpr (MI > 3) pass(std::integral_constant<int, 3>{});
    static_assert(MI <= 4, "passes are written out up to four row blocks");
}

// BK = 64 or 32 elements per k-tile (LDS rows of 128 or 64 bytes), S LDS stages: the loads of tile
// kt + S - 1 are in flight while tile kt is multiplied, so a load has S - 1 tile times to arrive.
// OCC workgroups per CU (the launch bound is given in waves per SIMD: OCC * waves / 4).
// WGM x 2 waves: WGM = 2 gives 128-row wave tiles (256 accumulator registers, one wave per SIMD),
// WGM = 4 gives 64-row wave tiles and two waves per SIMD, i.e. twice as many waves issuing loads.
// Sum of a value over the two halves of a wave (lane l and lane l ^ 32), in both.
__device__ __forceinline__ float wave_halves_sum(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Projection epilogue (EPI_ROWDOT) of a wave tile whose MFMAs took the W operand first: a lane's accumulators are
// one tile row's columns (row = lane % 32 of a 32-row block, column 8 (v / 4) + 4 (lane / 32) + v % 4 of a 32-column
// block), so out[r][c / 64] = sum over the 64 columns of act(acc + bias) * w is a sum inside the lane plus one
// exchange between the lane halves, and the accumulators never go through LDS (staging a 384 x 256 tile there and
// reading it back, eight waves at once at the LDS's 128 bytes per clock, took 9 of 121 us).  Bias and projection vector
// of the tile's columns go to LDS first (the operand buffers are free; the caller's barrier is behind their last read)
// and come back by broadcast reads of four consecutive columns.
template <int MI, int NI, int WM, int WN, int BN, int THREADS, bool PADDED>
__device__ __forceinline__ void rowdot_epilogue_transposed(const GemmArgs& p, f32x16 (&acc)[MI][NI], char* smem, int wm, int wn,
                                                           int tid, int m0, int n0) {
    static_assert(NI % 2 == 0 && 2 * BN <= THREADS, "whole 64-column groups per wave; one value per thread");
    const int lane = tid & 63, g = lane >> 5, li = lane & 31;
    float* sbw = reinterpret_cast<float*>(smem);
    if (tid < BN) sbw[tid] = n0 + tid < p.N ? p.bias[n0 + tid] : 0.0f;
    else if (tid < 2 * BN) sbw[tid] = n0 + tid - BN < p.N ? p.gamma[n0 + tid - BN] : 0.0f;
    __syncthreads();
    float* out = reinterpret_cast<float*>(p.out);
    EpilogueRows<PADDED> rows(p, m0 + wm * WM + li);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int r = rows.row(p);
        rows.advance(32);
        float sum[NI / 2];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            float sj = 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = wn * WN + j * 32 + 8 * q + 4 * g;
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(sbw + ch), w4 = *reinterpret_cast<const f32x4*>(sbw + BN + ch);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float a = acc[i][j][4 * q + e] + b4[e];
                    if (p.act == ACT_RELU) a = fmaxf(a, 0.0f);
                    sj += a * w4[e];
                }
            }
            if (j & 1) sum[j >> 1] += sj; else sum[j >> 1] = sj;
            __builtin_amdgcn_sched_barrier(0);       // (keeps the scheduler from lifting every block's reads to the top: no registers for that)
        }
#pragma unroll
        for (int k = 0; k < NI / 2; ++k) {
            const float tot = wave_halves_sum(sum[k]);
            const int c = n0 + wn * WN + 64 * k;
            if (g == (k & 1) && r < p.M && c < p.N) out[(int64_t)r * p.ldo + (c >> 6)] = tot;
        }
    }
}

// RD: the instantiation for EPI_ROWDOT alone (MFMAs with the W operand first, projection epilogue without LDS staging).
template <int BN, int BK, int S, int WGM, int WGN, int OCC, int AMODE, int BM_ = 256, bool RD = false>
__global__ __launch_bounds__(64 * WGM * WGN, OCC * WGM * WGN / 4) void gemm_dma_kernel(const GemmArgs args) {
    const GemmArgs p = select_problem(args);
    typedef bf16 T;
    constexpr int BM = BM_, CE = 8, NW = WGN * WGM;
    static_assert((BM * BK * 2) % (1024 * NW) == 0 && (BN * BK * 2) % (1024 * NW) == 0 && BM % (32 * WGM) == 0, "loader / wave tiling");
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int ROWB = BK * 2, CPR = BK / 8, RPI = 64 / CPR;   // row bytes, chunks per row, rows per DMA instruction
    constexpr int KS = BK / 16;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int A_SLOTS = A_BYTES / (1024 * NW), B_SLOTS = B_BYTES / (1024 * NW);   // 1 KB DMA instructions per wave per k-tile
    constexpr int PD = S - 1;
    // chunk swizzle: 256 bytes of LDS (64 banks) hold 2 rows of 128 bytes or 4 rows of 64 bytes
    constexpr int SW_SHIFT = BK == 64 ? 1 : 2, SW_MASK = CPR - 1;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;

    int tm, tn;
    tile_coords(xcd_contiguous(blockIdx.x, gridDim.x), (p.M - p.m_begin + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
    const int m0 = p.m_begin + tm * BM, n0 = tn * BN;

    // folded LayerNorm: (mean, rstd) of this tile's rows live behind the stage / staging buffers
    constexpr int EPI_BYTES = NW * 32 * WN * 4;
    float* lnrow = reinterpret_cast<float*>(smem + (S * STAGE > EPI_BYTES ? S * STAGE : EPI_BYTES));

    const char* __restrict__ A = reinterpret_cast<const char*>(p.A);
    const char* __restrict__ W = reinterpret_cast<const char*>(p.W);

    // --- loader state.  DMA instruction `slot` of this wave fills 1 KB of LDS = RPI consecutive rows of
    // the A (or B) tile, row group rg = wave + NW slot: lane l lands on row rg*RPI + l/CPR, physical
    // chunk l%CPR, so it must fetch the logical chunk (l%CPR) ^ swizzle(row) of that row.
    int aoff[A_SLOTS];          // byte offset of the lane's chunk from A (k = 0; conv: centre pixel)
    int ay[A_SLOTS], ax[A_SLOTS];
    int boff[B_SLOTS];
#pragma unroll
    for (int s = 0; s < A_SLOTS; ++s) {
        const int row = (wave + NW * s) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ ((row >> SW_SHIFT) & SW_MASK);
        int r = m0 + row;
        r = r < p.M ? r : p.M - 1;
        ay[s] = ax[s] = 0;
        if (AMODE == A_PLAIN) {
            const int64_t ar = (int64_t)(r / p.a_rpi) * p.a_istride + p.a_off + r % p.a_rpi;
            aoff[s] = (int)((ar * p.lda + c * CE) * 2);
        } else {
            const int hw = p.cH * p.cW;
            const int b = r / hw, pix = r % hw;
            ay[s] = pix / p.cW;
            ax[s] = pix % p.cW;
            aoff[s] = (int)((((int64_t)b * p.a_istride + p.a_off + pix) * p.lda + c * CE) * 2);
        }
    }
#pragma unroll
    for (int s = 0; s < B_SLOTS; ++s) {
        const int row = (wave + NW * s) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ ((row >> SW_SHIFT) & SW_MASK);
        boff[s] = (int)(((int64_t)(n0 + row) * p.K + c * CE) * 2);
    }
    const char* zptr = reinterpret_cast<const char*>(p.zeros);

    auto dma = [&](int stage, int kt) {
        char* sA = smem + stage * STAGE;
        char* sB = sA + A_BYTES;
        const int k0 = kt * BK;
        if (AMODE == A_PLAIN) {
#pragma unroll
            for (int s = 0; s < A_SLOTS; ++s)
                __builtin_amdgcn_global_load_lds(VPE_GPTR(A + aoff[s] + k0 * 2), VPE_LPTR(sA + (wave + NW * s) * 1024), 16, 0, 0);
        } else {
            const int cc = kt / 9, tap = kt - cc * 9, c0 = cc * BK;    // chunk-major, tap-minor k order
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
            const int shift = ((dy * p.cW + dx) * (int)p.lda + c0) * 2;
#pragma unroll
            for (int s = 0; s < A_SLOTS; ++s) {
                const int yy = ay[s] + dy, xx = ax[s] + dx;
                const bool ok = yy >= 0 && yy < p.cH && xx >= 0 && xx < p.cW;
                const uint64_t mask = ok ? ~uint64_t(0) : uint64_t(0);
                const uint64_t addr = (reinterpret_cast<uint64_t>(A + aoff[s] + shift) & mask) |
                                      (reinterpret_cast<uint64_t>(zptr) & ~mask);
                __builtin_amdgcn_global_load_lds(VPE_GPTR(addr), VPE_LPTR(sA + (wave + NW * s) * 1024), 16, 0, 0);
            }
        }
        const int kw = AMODE == A_PLAIN ? k0 : (kt % 9) * p.cC + (kt / 9) * BK;   // weight column of this k-tile
#pragma unroll
        for (int s = 0; s < B_SLOTS; ++s)
            __builtin_amdgcn_global_load_lds(VPE_GPTR(W + boff[s] + kw * 2), VPE_LPTR(sB + (wave + NW * s) * 1024), 16, 0, 0);
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // --- MFMA operand reads.  Rows of one lane differ by multiples of 32, so the swizzle term is the
    // same for all of them: one lane offset per k-step, rows by immediates.
    const int arow0 = wm * WM + li, brow0 = wn * WN + li;
    const int asw = (arow0 >> SW_SHIFT) & SW_MASK, bsw = (brow0 >> SW_SHIFT) & SW_MASK;
    // Wave tiles of up to 6 fragments per k-step keep two fragment sets (the reads of step ks + 1 are in
    // flight during the MFMAs of step ks); larger wave tiles have no registers for the second set and read
    // each step's fragments just before its MFMAs (two waves per SIMD cover for each other).
    constexpr bool FRAG_DB = MI + NI <= 6;
    auto compute = [&](int stage) {
        const char* sA = smem + stage * STAGE + arow0 * ROWB;
        const char* sB = smem + stage * STAGE + A_BYTES + brow0 * ROWB;
        if constexpr (FRAG_DB) {
            bf16x8 fa[2][MI], fb[2][NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[0][i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * ROWB + ((g ^ asw) * 16));
#pragma unroll
            for (int j = 0; j < NI; ++j) fb[0][j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * ROWB + ((g ^ bsw) * 16));
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 1 < KS) {
                    const int ca = ((2 * (ks + 1) + g) ^ asw) * 16, cb = ((2 * (ks + 1) + g) ^ bsw) * 16;
#pragma unroll
                    for (int i = 0; i < MI; ++i) fa[(ks + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * ROWB + ca);
#pragma unroll
                    for (int j = 0; j < NI; ++j) fb[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * ROWB + cb);
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = RD ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
                // Issue order for the scheduler: the LDS reads of step ks + 1 are spread between the MFMAs
                // of step ks (one read per two MFMAs), so the only wave on this SIMD never waits on LDS
                // with an empty matrix pipe.  0x100 = DS read, 0x008 = MFMA.
                if (ks == 0) __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
                if (ks + 1 < KS) {
                    constexpr int PER = (MI * NI) / (MI + NI) > 0 ? (MI * NI) / (MI + NI) : 1;
                    constexpr int GROUPS = (MI * NI) / PER < MI + NI ? (MI * NI) / PER : MI + NI;
#pragma unroll
                    for (int n = 0; n < GROUPS; ++n) {
                        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x100, MI + NI - GROUPS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - GROUPS * PER, 0);
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x008, MI * NI, 0);
                }
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int ca = ((2 * ks + g) ^ asw) * 16, cb = ((2 * ks + g) ^ bsw) * 16;
                bf16x8 fa[MI], fb[NI];
#pragma unroll
                for (int i = 0; i < MI; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * ROWB + ca);
#pragma unroll
                for (int j = 0; j < NI; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * ROWB + cb);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = RD ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, MI * NI, 0);
            }
        }
    };

    // --- main loop: S LDS stages.  Iteration kt: wait until tile kt has landed (the S - 2 younger
    // tiles may still be in flight), barrier (which also tells everyone that the stage read in
    // iteration kt - 1 is free), issue the loads of tile kt + S - 1 into that free stage, multiply
    // tile kt.  Prefetches are unconditional (clamped index): every path has the same loads in flight.
    const int KT = p.K / BK;
#pragma unroll
    for (int s = 0; s < PD; ++s) dma(s, s < KT ? s : KT - 1);
    // behind the first tile loads, ordered before the epilogue by the loop's barriers
    if (p.ln_stats && tid < BM) ln_tile_row(p, m0, n0, tid, lnrow);
    for (int kt = 0; kt < KT; ++kt) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((PD - 1) * (A_SLOTS + B_SLOTS)));
        __syncthreads();
        dma((kt + PD) % S, kt + PD < KT ? kt + PD : KT - 1);
        __builtin_amdgcn_sched_barrier(0);
        compute(kt % S);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // drain the clamped tail prefetches before LDS is reused
    __syncthreads();

    if constexpr (WN % 64 != 0) {
        // Small tiles (32-column wave tiles): a wave does not hold whole 64-column groups, so the tile leaves
        // through the block-level epilogue of the register-staged kernels (whole tile staged in LDS).
        static_assert(BM * BN * 4 <= S * STAGE, "accumulator tile must fit the stage buffers");
        float lncs[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int c = n0 + wn * WN + j * 32 + li;
            lncs[j] = p.ln_stats && c < p.N ? p.ln_colsum[c] : 0.0f;
        }
        block_epilogue<T, BM, BN, WGM, WGN>(p, acc, smem, lnrow, lncs, m0, n0);
        return;
    }

    if constexpr (RD) rowdot_epilogue_transposed<MI, NI, WM, WN, BN, 64 * NW, false>(p, acc, smem, wm, wn, tid, m0, n0);
    else wave_tile_epilogue<MI, NI, WM, WN>(p, acc, smem, lnrow, wave, wm, wn, lane, m0, n0);
}

template <int BN, int BK, int S, int WGM = 2, int WGN = 2, int OCC = 1, int BM = 256, bool RD = false>
static inline hipError_t launch_gemm_dma(const GemmArgs& a, int amode, hipStream_t s, bool configure_only = false) {
    constexpr int stage_b = S * (BM + BN) * BK * 2, epi_b = WGM * WGN * 32 * (BN / WGN) * 4;
    constexpr int lds = (stage_b > epi_b ? stage_b : epi_b) + BM * 8;     // + (mean, rstd) of the tile's rows
    static_assert(lds * OCC <= 160 * 1024, "LDS budget of one CU");
    static bool configured = false;
    if (!configured) {
        hipError_t rc = hipSuccess;
        if (!RD) rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<BN, BK, S, WGM, WGN, OCC, A_PLAIN, BM, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc == hipSuccess)
            rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<BN, BK, S, WGM, WGN, OCC, A_CONV3, BM, RD>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc != hipSuccess) return rc;
        configured = true;
    }
    if (configure_only) return hipSuccess;
    // the projection-only instantiation exists for convolutions (the only users of that epilogue on these tiles)
    if (RD && (amode != A_CONV3 || a.epi != EPI_ROWDOT || a.ln_stats)) return hipErrorInvalidValue;
    const int tiles = cdiv(a.M - a.m_begin, BM) * cdiv(a.N, BN), nz = a.nz > 1 ? a.nz : 1;
    if (RD) hipLaunchKernelGGL((gemm_dma_kernel<BN, BK, S, WGM, WGN, OCC, A_CONV3, BM, RD>), dim3(tiles, nz), dim3(64 * WGM * WGN), lds, s, a);
    else if (amode == A_PLAIN) hipLaunchKernelGGL((gemm_dma_kernel<BN, BK, S, WGM, WGN, OCC, A_PLAIN, BM, false>), dim3(tiles, nz), dim3(64 * WGM * WGN), lds, s, a);
    else hipLaunchKernelGGL((gemm_dma_kernel<BN, BK, S, WGM, WGN, OCC, A_CONV3, BM, false>), dim3(tiles, nz), dim3(64 * WGM * WGN), lds, s, a);
    return hipGetLastError();
}

}  // namespace vpe
