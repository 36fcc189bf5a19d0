// Tiled MFMA GEMM for gfx950:  C[M][N] = A[M][K] * W^T  with W stored [N][K] (K contiguous),
// fp32 accumulation, and the layer's epilogue applied to the accumulators in registers.
//
// One kernel serves every dense contraction of the encoder and the heads (ViT blocks: fused
// QKV, out-projection, MLP; patch embedding after im2col; the heads' 1x1 and 3x3 convolutions):
//   * A operand: plain rows (optionally re-mapped so that only patch tokens of each image are
//     read) or an implicit im2col of a channels-last grid for 3x3 / pad 1 convolutions.
//   * operands in bf16 (v_mfma_f32_32x32x16_bf16) or fp32 (v_mfma_f32_32x32x2_f32).
//   * LDS: two stages of (BM + BN) rows x 128 bytes, 16-byte chunks XOR-swizzled by row.
//   * global -> register -> LDS software pipeline, one barrier per k-tile.
#pragma once
#include "common.h"

namespace vpe {

enum AMode { A_PLAIN = 0, A_CONV3 = 1 };
enum Epi { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3, EPI_PATCH = 4 };
enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

struct GemmArgs {
    const void* A;       // T
    int64_t lda;         // elements between consecutive A rows (PLAIN) / pixels (CONV3)
    const void* W;       // T [N rounded up to 128][K]
    const float* bias;   // [N] in the physical column order of W, may be null
    int M, N, K;         // K multiple of 64 (bf16) / 32 (fp32)
    // PLAIN: logical row r reads A row (r / a_rpi) * a_istride + a_off + r % a_rpi
    // CONV3: pixel (b, y, x) is A row b * a_istride + a_off + y * cW + x
    int a_rpi, a_istride, a_off;
    int cH, cW, cC;      // CONV3 grid and channels (K = 9 cC, cC multiple of the k-tile)
    int epi, act, out_f32;
    void* out;           // T or float (out_f32); RESID/PATCH: float residual stream
    int64_t ldo;
    int o_rpi, o_istride, o_off;   // output row map, as for A
    const float* gamma;  // RESID: LayerScale vector
    const float* pos;    // PATCH: positional rows [o_rpi][N]
    void* out2;          // QKV: transposed values  vt[(b * dim + c)][npad]
    int ntok, npad, dim; // QKV
};

template <typename T> struct Mma;

template <> struct Mma<bf16> {
    static constexpr int KS = 4;   // MFMA k-steps per 64-element k-tile
    typedef bf16x8 Frag;
    // lane half g supplies k elements 16 ks + 8 g .. + 7 of its row
    static __device__ __forceinline__ Frag load(const char* tile, int row, int ks, int g) {
        return *reinterpret_cast<const Frag*>(tile + (row * 8 + swz(row, 2 * ks + g)) * 16);
    }
    static __device__ __forceinline__ void mma(f32x16& c, const Frag& a, const Frag& b) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

template <> struct Mma<float> {
    static constexpr int KS = 2;   // macro k-steps (16 elements) per 32-element k-tile
    struct Frag { f32x4 lo, hi; };
    // lane half g supplies k elements 16 ks + 8 g .. + 7 of its row; the 8 MFMAs of a macro
    // step pair element kk of A with element kk of B, so the k order only has to agree.
    static __device__ __forceinline__ Frag load(const char* tile, int row, int ks, int g) {
        Frag f;
        f.lo = *reinterpret_cast<const f32x4*>(tile + (row * 8 + swz(row, 4 * ks + 2 * g)) * 16);
        f.hi = *reinterpret_cast<const f32x4*>(tile + (row * 8 + swz(row, 4 * ks + 2 * g + 1)) * 16);
        return f;
    }
    static __device__ __forceinline__ void mma(f32x16& c, const Frag& a, const Frag& b) {
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo[i], b.lo[i], c, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi[i], b.hi[i], c, 0, 0, 0);
    }
};

__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)); }

// Spread consecutive block ids (which the hardware deals round-robin to the 8 XCDs) so that
// each XCD works on one contiguous range of tiles and its L2 sees neighbouring A/W panels.
__device__ __forceinline__ int xcd_contiguous(int bid, int nb) {
    const int xcd = bid & 7, idx = bid >> 3, base = nb >> 3, rem = nb & 7;
    return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

template <typename T, int BM, int BN, int WGM, int WGN, int AMODE>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(const GemmArgs p) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr int CE = Elem<T>::CE;
    constexpr int BK = 8 * CE;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int RPP = NT / 8;
    constexpr int A_IT = BM / RPP, B_IT = BN / RPP;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must be a multiple of the loader pass");
    constexpr int STAGE = (BM + BN) * 128;
    __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    const int lrow = tid >> 3, lchunk = tid & 7;

    const int tiles_n = (p.N + BN - 1) / BN;
    const int lin = xcd_contiguous(blockIdx.x, gridDim.x);
    const int m0 = (lin / tiles_n) * BM, n0 = (lin % tiles_n) * BN;

    const T* __restrict__ A = reinterpret_cast<const T*>(p.A);
    const T* __restrict__ W = reinterpret_cast<const T*>(p.W);

    // per-thread A row state
    const T* aptr[A_IT];
    int ay[A_IT], ax[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int r = m0 + lrow + i * RPP;
        aptr[i] = nullptr;
        ay[i] = ax[i] = 0;
        if (r < p.M) {
            if (AMODE == A_PLAIN) {
                const int64_t ar = (int64_t)(r / p.a_rpi) * p.a_istride + p.a_off + r % p.a_rpi;
                aptr[i] = A + ar * p.lda + lchunk * CE;
            } else {
                const int hw = p.cH * p.cW;
                const int b = r / hw, pix = r % hw;
                ay[i] = pix / p.cW;
                ax[i] = pix % p.cW;
                aptr[i] = A + ((int64_t)b * p.a_istride + p.a_off + pix) * p.lda + lchunk * CE;
            }
        }
    }
    const T* wptr = W + (int64_t)(n0 + lrow) * p.K + lchunk * CE;

    u32x4 ra[A_IT], rb[B_IT];
    auto gload = [&](int kt) {
        const int k0 = kt * BK;
        if (AMODE == A_PLAIN) {
#pragma unroll
            for (int i = 0; i < A_IT; ++i)
                ra[i] = aptr[i] ? ld_global_16(aptr[i] + k0) : u32x4{0, 0, 0, 0};
        } else {
            const int tap = k0 / p.cC, c0 = k0 - tap * p.cC;
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
#pragma unroll
            for (int i = 0; i < A_IT; ++i) {
                const int yy = ay[i] + dy, xx = ax[i] + dx;
                const bool ok = aptr[i] && yy >= 0 && yy < p.cH && xx >= 0 && xx < p.cW;
                ra[i] = ok ? ld_global_16(aptr[i] + (int64_t)(dy * p.cW + dx) * p.lda + c0) : u32x4{0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) rb[i] = ld_global_16(wptr + (int64_t)i * RPP * p.K + k0);
    };
    auto sstore = [&](int buf) {
        char* sA = smem + buf * STAGE;
        char* sB = sA + BM * 128;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sA + (r * 8 + swz(r, lchunk)) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sB + (r * 8 + swz(r, lchunk)) * 16) = rb[i];
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int KT = p.K / BK;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) gload(kt + 1);
        const char* sA = smem + cur * STAGE;
        const char* sB = sA + BM * 128;
#pragma unroll
        for (int ks = 0; ks < Mma<T>::KS; ++ks) {
            typename Mma<T>::Frag fa[MI], fb[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[i] = Mma<T>::load(sA, wm * WM + i * 32 + li, ks, g);
#pragma unroll
            for (int j = 0; j < NI; ++j) fb[j] = Mma<T>::load(sB, wn * WN + j * 32 + li, ks, g);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) Mma<T>::mma(acc[i][j], fa[i], fb[j]);
        }
        if (kt + 1 < KT) sstore(cur ^ 1);
        __syncthreads();
    }

    // ---------------------------------------------------------------- epilogue
    // accumulator element v of lane (g, li) in block (i, j):
    //   row = 32 i + 8 (v / 4) + 4 g + v % 4,  col = 32 j + li
    const int rbase = m0 + wm * WM + 4 * g;
    const int cbase = n0 + wn * WN + li;
    if (p.epi == EPI_SWIGLU) {
        // physical columns come in groups of 64: 32 gate columns then their 32 linear partners
        if constexpr (NI % 2 == 0) {
            T* out = reinterpret_cast<T*>(p.out);
#pragma unroll
            for (int j = 0; j < NI; j += 2) {
                const int ca = cbase + j * 32, cb = ca + 32;
                if (cb >= p.N) continue;
                const float ba = p.bias[ca], bb = p.bias[cb];
                const int oc = (ca >> 6) * 32 + li;
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
                        if (r >= p.M) continue;
                        const float a = acc[i][j][v] + ba, b = acc[i][j + 1][v] + bb;
                        out[(int64_t)r * p.ldo + oc] = from_f32<T>(a / (1.0f + __expf(-a)) * b);
                    }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int c = cbase + j * 32;
        if (c >= p.N) continue;
        const float bias = p.bias ? p.bias[c] : 0.0f;
        const float gam = p.epi == EPI_RESID ? p.gamma[c] : 0.0f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
                if (r >= p.M) continue;
                float val = acc[i][j][v] + bias;
                if (p.epi == EPI_STORE) {
                    if (p.act == ACT_RELU) val = fmaxf(val, 0.0f);
                    else if (p.act == ACT_GELU) val = gelu_erf(val);
                    const int64_t orow = (int64_t)(r / p.o_rpi) * p.o_istride + p.o_off + r % p.o_rpi;
                    if (p.out_f32) reinterpret_cast<float*>(p.out)[orow * p.ldo + c] = val;
                    else reinterpret_cast<T*>(p.out)[orow * p.ldo + c] = from_f32<T>(val);
                } else if (p.epi == EPI_RESID) {
                    float* x = reinterpret_cast<float*>(p.out) + (int64_t)r * p.ldo + c;
                    *x = *x + gam * val;
                } else if (p.epi == EPI_PATCH) {
                    const int b = r / p.o_rpi, pp = r % p.o_rpi;
                    const int64_t orow = (int64_t)b * p.o_istride + p.o_off + pp;
                    reinterpret_cast<float*>(p.out)[orow * p.ldo + c] = val + p.pos[(int64_t)pp * p.N + c];
                } else {   // EPI_QKV
                    if (c < 2 * p.dim) {
                        reinterpret_cast<T*>(p.out)[(int64_t)r * p.ldo + c] = from_f32<T>(val);
                    } else {
                        const int b = r / p.ntok, n = r % p.ntok;
                        reinterpret_cast<T*>(p.out2)[((int64_t)b * p.dim + (c - 2 * p.dim)) * p.npad + n] =
                            from_f32<T>(val);
                    }
                }
            }
    }
}

template <typename T, int BM, int BN, int WGM, int WGN>
static inline hipError_t launch_tile(const GemmArgs& a, int amode, hipStream_t s) {
    const int tiles = cdiv(a.M, BM) * cdiv(a.N, BN);
    dim3 grid(tiles), block(64 * WGM * WGN);
    if (amode == A_PLAIN) hipLaunchKernelGGL((gemm_kernel<T, BM, BN, WGM, WGN, A_PLAIN>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((gemm_kernel<T, BM, BN, WGM, WGN, A_CONV3>), grid, block, 0, s, a);
    return hipGetLastError();
}

// Tile choice: the largest tile that still yields about two workgroups per CU; SwiGLU needs
// wave tiles of 64 columns (gate and linear partner in the same lane).
template <typename T>
static inline hipError_t launch_gemm_t(const GemmArgs& a, int amode, hipStream_t s) {
    const int64_t t128 = (int64_t)cdiv(a.M, 128) * cdiv(a.N, 128);
    const int64_t t64x128 = (int64_t)cdiv(a.M, 64) * cdiv(a.N, 128);
    if (t128 >= 384) return launch_tile<T, 128, 128, 2, 2>(a, amode, s);
    if (t64x128 >= 384 || a.epi == EPI_SWIGLU) return launch_tile<T, 64, 128, 2, 2>(a, amode, s);
    return launch_tile<T, 64, 64, 2, 2>(a, amode, s);
}

}  // namespace vpe
