// Tiled MFMA GEMM for gfx950:  C[M][N] = A[M][K] * W^T  with W stored [N][K] (K contiguous),
// fp32 accumulation, and the layer's epilogue applied to the accumulators in registers.
//
// One kernel serves every dense contraction of the encoder and the heads (ViT blocks: fused
// QKV, out-projection, MLP; patch embedding after im2col; the heads' 1x1 and 3x3 convolutions):
//   * A operand: plain rows (optionally re-mapped so that only patch tokens of each image are
//     read) or an implicit im2col of a channels-last grid for 3x3 / pad 1 convolutions.
//   * operands in bf16 (v_mfma_f32_32x32x16_bf16) or fp32 (v_mfma_f32_32x32x2_f32).
//   * LDS: two stages of (BM + BN) rows x 128 bytes, 16-byte chunks XOR-swizzled by row.
//   * global -> register -> LDS software pipeline two k-tiles deep, one barrier per k-tile.
#pragma once
#include "common.h"

namespace vpe {

enum AMode { A_PLAIN = 0, A_CONV3 = 1 };
enum Epi { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3, EPI_PATCH = 4, EPI_ROWDOT = 5 };
enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

struct GemmArgs {
    const void* A;       // T
    int64_t lda;         // elements between consecutive A rows (PLAIN) / pixels (CONV3)
    const void* W;       // T [N rounded up to 256][K]
    const float* bias;   // [N] in the physical column order of W, may be null
    int M, N, K;         // K multiple of 64 (bf16) / 32 (fp32)
    int m_begin;         // a launch covers rows m_begin .. M - 1 (row indices stay those of the whole problem)
    // PLAIN: logical row r reads A row (r / a_rpi) * a_istride + a_off + r % a_rpi
    // CONV3: pixel (b, y, x) is A row b * a_istride + a_off + y * cW + x
    int a_rpi, a_istride, a_off;
    int cH, cW, cC;      // CONV3 grid and channels (K = 9 cC, cC multiple of the k-tile)
    const void* zeros;   // CONV3: >= 16 bytes of zeros, read in place of out-of-image taps
    int epi, act, out_f32;
    void* out;           // T or float (out_f32); RESID/PATCH: float residual stream
    int64_t ldo;
    int o_rpi, o_istride, o_off;   // output row map, as for A
    const float* gamma;  // RESID: LayerScale vector.  ROWDOT: projection vector w[N]; the tile itself is not stored,
                         //   out (float) receives out[r * ldo + c / 64] = sum over the 64 columns of group c / 64 of
                         //   act(acc + bias)[col] * w[col]  (N multiple of 64; the caller adds the N / 64 partial sums)
    const float* pos;    // PATCH: positional rows [o_rpi][N]
    void* out2;          // QKV: transposed values  vt[(b * dim + c)][npad]
    int ntok, npad, dim; // QKV
    // LayerNorm folded into this GEMM (consumer side): A holds the UN-normalised rows (plain row map), W has
    // been scaled by the LayerNorm gain along k and bias holds b + beta W; the accumulator of (row r, column c)
    // becomes rstd_r * (acc - mean_r * ln_colsum[c]) before bias / activation, with ln_colsum[c] = sum_k W[c][k].
    // ln_stats [M][ln_groups][2]: (mean, sum of squared deviations from it) of every 64-column group of row r,
    // as written by the producer below; both sides work with differences, never with raw squares.
    const float* ln_stats;     // null: no LayerNorm
    const float* ln_colsum;
    int ln_groups;             // = K / 64
    float ln_eps;
    // A may hold the rows minus a per-row level (LayerNorm does not see a level common to a row, and a 16-bit
    // copy of x - level keeps its precision when the row sits far from zero): ln_level[r] is that level (null:
    // 0).  ln_level_out (may be null) receives the rows' means, written by the tiles of the first column
    // block: the level for the NEXT copy of these rows -- a different buffer from ln_level, which the other
    // column tiles are still reading.
    const float* ln_level;
    float* ln_level_out;
    // Producer side (RESID / PATCH, N a multiple of 64): besides the fp32 rows, write their copy in T
    // (xb_out, [rows][N], may be null) and the group statistics of the updated rows (st_out, may be null)
    void* xb_out;
    float* st_out;
    const float* xb_level;     // xb_out holds x - xb_level[row] (null: 0); statistics are of x itself
    // STORE only (N and ldo multiples of 8): fp32 tensors added after the activation, read through the output
    // row map with the output's row pitch (null: none); and a second copy of the result in T, optionally
    // through ReLU (the operand of a following convolution), same map and pitch (null: none)
    const float* add1;
    const float* add2;
    void* twin;
    int twin_relu;
    // batch of nz independent problems of the same shape in one launch (blockIdx.y = z): problem z uses
    // A + z * z_a, W + z * z_w, out + z * z_out (byte strides, may be negative) and bias + z * z_bias (elements);
    // with z_inner > 0 the output alone is addressed in two levels, out + (z % z_inner) * z_out + (z / z_inner) * z_out2
    int nz;
    int64_t z_a, z_w, z_out, z_bias;
    int z_inner;
    int64_t z_out2;
};

// The arguments of problem blockIdx.y of a batched launch (a plain copy when the launch is not batched).
__device__ __forceinline__ GemmArgs select_problem(const GemmArgs& in) {
    GemmArgs p = in;
    const int64_t z = blockIdx.y;
    p.A = reinterpret_cast<const char*>(in.A) + z * in.z_a;
    p.W = reinterpret_cast<const char*>(in.W) + z * in.z_w;
    p.out = in.z_inner > 0 ? reinterpret_cast<char*>(in.out) + (z % in.z_inner) * in.z_out + (z / in.z_inner) * in.z_out2
                           : reinterpret_cast<char*>(in.out) + z * in.z_out;
    if (in.bias) p.bias = in.bias + z * in.z_bias;
    return p;
}


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

// GELU in its exact (erf) form.  erf by the Abramowitz-Stegun 7.1.26 rational approximation
// (|error| <= 1.5e-7, i.e. fp32 rounding level): one reciprocal, one exponential and six FMAs
// instead of the ~40-instruction library erff, which made the GELU epilogue of a 256 x 256 tile as
// long as its k loop.
__device__ __forceinline__ float gelu_erf(float v) {
    const float x = fabsf(v) * 0.70710678118654752f;
    const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float erf_abs = 1.0f - poly * t * __expf(-x * x);
    return 0.5f * v * (1.0f + copysignf(erf_abs, v));
}

// The same function for results that are rounded to bf16: erf(x) = x P(x^2) on |x| <= 3, P of degree 9 (least-squares fit
// at Chebyshev nodes, |error of erf| <= 1.9e-5; beyond 3 the value at 3, 0.99998, clamped to 1), Horner in fp32: no
// reciprocal, no exponential (two quarter-rate instructions of the form above), 14 instead of 23 issue slots.  The
// result differs from the exact form by at most 1e-5 |v| -- 1/400 of a bf16 rounding step.
__device__ __forceinline__ float gelu_erf_bf16(float v) {
    const float x = fminf(fabsf(v) * 0.70710678118654752f, 3.0f);
    const float t = x * x;
    float p = fmaf(-4.469939086e-09f, t, 2.302152922e-07f);
    p = fmaf(p, t, -5.322654488e-06f);
    p = fmaf(p, t, 7.394709974e-05f);
    p = fmaf(p, t, -7.009955007e-04f);
    p = fmaf(p, t, 4.897189327e-03f);
    p = fmaf(p, t, -2.645343542e-02f);
    p = fmaf(p, t, 1.125671491e-01f);
    p = fmaf(p, t, -3.760564327e-01f);
    p = fmaf(p, t, 1.128376126e+00f);
    const float erf_abs = fminf(p * x, 1.0f);
    return 0.5f * v * (1.0f + copysignf(erf_abs, v));
}
template <typename T>
__device__ __forceinline__ float gelu_for(float v) { return sizeof(T) == 2 ? gelu_erf_bf16(v) : gelu_erf(v); }
// SiLU(a) * b.  For results rounded to bf16 the quotient is one v_rcp_f32 (1 ulp) and a product instead of the
// correctly rounded division sequence (about ten instructions).
template <typename T>
__device__ __forceinline__ float swiglu_for(float a, float b) {
    const float d = 1.0f + __expf(-a);
    return sizeof(T) == 2 ? a * __builtin_amdgcn_rcpf(d) * b : a / d * b;
}

// Spread consecutive block ids (which the hardware deals round-robin to the 8 XCDs) so that
// each XCD works on one contiguous range of tiles and its L2 sees neighbouring A/W panels.
__device__ __forceinline__ int xcd_contiguous(int bid, int nb) {
    const int xcd = bid & 7, idx = bid >> 3, base = nb >> 3, rem = nb & 7;
    return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

// Linear tile index -> (tile row, tile column) in groups of GM tile rows: the ~32 workgroups an XCD
// runs at a time then cover a GM x (32 / GM) block of tiles instead of one row of 32, so each A
// k-slice fetched into that XCD's L2 serves 32 / GM workgroups and each W k-slice GM of them.
// (Measured on the large tiles: with row-major order the loads ran at the XCD <-> memory-side
// fabric rate, about 13 TB/s in aggregate, not at the L2 rate.)
__device__ __forceinline__ void tile_coords(int lin, int tiles_m, int tiles_n, int& tm, int& tn) {
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = lin / per_group, rem = lin - group * per_group;
    const int first = group * GM;
    const int gsz = tiles_m - first < GM ? tiles_m - first : GM;
    tm = first + rem % gsz;
    tn = rem / gsz;
}

// 8 consecutive values of T (16 bytes of bf16, 32 bytes of fp32) to global memory.
__device__ __forceinline__ void store8(bf16* dst, const float* v) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16)v[i];
    *reinterpret_cast<bf16x8*>(dst) = o;
}
__device__ __forceinline__ void store8(float* dst, const float* v) {
    *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{v[4], v[5], v[6], v[7]};
}

// Epilogue of one row chunk: columns c .. c + 7 of logical row r (r < M, c < N, c % 8 == 0), the raw
// accumulators in v.  Full, aligned chunks go out as 16-byte stores; ragged ones element by element.
template <typename T>
__device__ __forceinline__ void epilogue_chunk(const GemmArgs& p, int r, int c, float* v) {
    const int nv = p.N - c < 8 ? p.N - c : 8;
    if (p.bias) {
        if (nv == 8) {
            const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + c), b1 = *reinterpret_cast<const f32x4*>(p.bias + c + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] += b0[i]; v[4 + i] += b1[i]; }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) if (i < nv) v[i] += p.bias[c + i];
        }
    }
    if (p.epi == EPI_STORE) {
        if (p.act == ACT_RELU) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = fmaxf(v[i], 0.0f);
        } else if (p.act == ACT_GELU) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = gelu_for<T>(v[i]);
        }
        const int64_t orow = (int64_t)(r / p.o_rpi) * p.o_istride + p.o_off + r % p.o_rpi;
        if (p.add1) {
            const float* a = p.add1 + orow * p.ldo + c;
            const f32x4 a0 = *reinterpret_cast<const f32x4*>(a), a1 = *reinterpret_cast<const f32x4*>(a + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] += a0[i]; v[4 + i] += a1[i]; }
        }
        if (p.add2) {
            const float* a = p.add2 + orow * p.ldo + c;
            const f32x4 a0 = *reinterpret_cast<const f32x4*>(a), a1 = *reinterpret_cast<const f32x4*>(a + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] += a0[i]; v[4 + i] += a1[i]; }
        }
        if (p.twin) {
            float t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = p.twin_relu ? fmaxf(v[i], 0.0f) : v[i];
            store8(reinterpret_cast<T*>(p.twin) + orow * p.ldo + c, t);
        }
        if (p.out_f32) {
            float* dst = reinterpret_cast<float*>(p.out) + orow * p.ldo + c;
            if (nv == 8 && (p.ldo & 3) == 0) store8(dst, v);
            else {
#pragma unroll
                for (int i = 0; i < 8; ++i) if (i < nv) dst[i] = v[i];
            }
        } else {
            T* dst = reinterpret_cast<T*>(p.out) + orow * p.ldo + c;
            if (nv == 8 && (p.ldo & 7) == 0) store8(dst, v);
            else {
#pragma unroll
                for (int i = 0; i < 8; ++i) if (i < nv) dst[i] = from_f32<T>(v[i]);
            }
        }
    } else if (p.epi == EPI_RESID || p.epi == EPI_PATCH) {
        // fp32 residual stream, N = ldo = model width (multiple of 64): always full aligned chunks
        int64_t orow = r;
        if (p.epi == EPI_PATCH) {
            const int b = r / p.o_rpi, pp = r % p.o_rpi;
            orow = (int64_t)b * p.o_istride + p.o_off + pp;
            const float* ps = p.pos + (int64_t)pp * p.N + c;
            const f32x4 p0 = *reinterpret_cast<const f32x4*>(ps), p1 = *reinterpret_cast<const f32x4*>(ps + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] += p0[i]; v[4 + i] += p1[i]; }
        }
        float* x = reinterpret_cast<float*>(p.out) + orow * p.ldo + c;
        if (p.epi == EPI_RESID) {
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(p.gamma + c), g1 = *reinterpret_cast<const f32x4*>(p.gamma + c + 4);
            const f32x4 x0 = *reinterpret_cast<const f32x4*>(x), x1 = *reinterpret_cast<const f32x4*>(x + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] = x0[i] + g0[i] * v[i]; v[4 + i] = x1[i] + g1[i] * v[4 + i]; }
        }
        store8(x, v);
    } else {   // EPI_QKV, query / key columns
        store8(reinterpret_cast<T*>(p.out) + (int64_t)r * p.ldo + c, v);
    }
}

// ROWDOT: contribution of 8 consecutive columns (starting at c) of one row to the row's projection.
__device__ __forceinline__ float rowdot_chunk(const GemmArgs& p, int c, const float* v) {
    const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + c), b1 = *reinterpret_cast<const f32x4*>(p.bias + c + 4);
    const f32x4 w0 = *reinterpret_cast<const f32x4*>(p.gamma + c), w1 = *reinterpret_cast<const f32x4*>(p.gamma + c + 4);
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float a = v[i] + b0[i], b = v[4 + i] + b1[i];
        if (p.act == ACT_RELU) { a = fmaxf(a, 0.0f); b = fmaxf(b, 0.0f); }
        s += a * w0[i] + b * w1[i];
    }
    return s;
}

// QKV epilogue, value columns: tokens r .. r + 7 (r a multiple of 8) of value column c2 go to the transposed
// buffer vt[(image * dim + c2)][token in image].  With several images whose token count is not a multiple of
// 8 the group starts at an odd offset inside its image: still one run of 8 when it does not cross into the
// next image, written with the widest stores its alignment allows; only a group that straddles two images
// (or the end of the matrix) goes element by element.
template <typename T>
__device__ __forceinline__ void store_tokens8(const GemmArgs& p, T* vt, int r, int c2, const float* v) {
    const int b = r / p.ntok, n = r - b * p.ntok;
    T* dst = vt + ((int64_t)b * p.dim + c2) * p.npad + n;
    if (n + 8 <= p.ntok && r + 8 <= p.M) {
        if ((n & 7) == 0) {
            store8(dst, v);
        } else if (sizeof(T) == 2 && (n & 1) == 0) {
#pragma unroll
            for (int k = 0; k < 8; k += 2) {
                const T lo = from_f32<T>(v[k]), hi = from_f32<T>(v[k + 1]);
                uint32_t w;
                w = (uint32_t)(*reinterpret_cast<const uint16_t*>(&lo)) | ((uint32_t)(*reinterpret_cast<const uint16_t*>(&hi)) << 16);
                *reinterpret_cast<uint32_t*>(dst + k) = w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) dst[k] = from_f32<T>(v[k]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int rk = r + k;
            if (rk < p.M) vt[((int64_t)(rk / p.ntok) * p.dim + c2) * p.npad + rk % p.ntok] = from_f32<T>(v[k]);
        }
    }
}

// (mean, rstd) of row r from its group statistics (mean_g, M2_g = sum of squared deviations from mean_g, of
// each 64-column group).  Groups are merged around the first group's mean, so a level common to the whole row
// cancels before anything is squared:
//   mean = m_0 + avg_g (m_g - m_0),   M2 = sum_g M2_g + 64 (sum_g (m_g - m_0)^2 - G (mean - m_0)^2).
// All loads are independent 16-byte loads of two groups each.
__device__ __forceinline__ void ln_row_stats(const GemmArgs& p, int r, float& mean, float& rstd) {
    const float* st = p.ln_stats + (int64_t)r * p.ln_groups * 2;
    const float m0 = st[0];
    float sd = 0.0f, sdd = 0.0f, sm2 = 0.0f;
    int g = 0;
#pragma unroll 4
    for (; g + 2 <= p.ln_groups; g += 2) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(st + 2 * g);
        const float d0 = v[0] - m0, d1 = v[2] - m0;
        sd += d0 + d1;
        sdd += d0 * d0 + d1 * d1;
        sm2 += v[1] + v[3];
    }
    if (g < p.ln_groups) {
        const float d = st[2 * g] - m0;
        sd += d; sdd += d * d; sm2 += st[2 * g + 1];
    }
    const float G = (float)p.ln_groups, dm = sd / G;
    mean = m0 + dm;
    const float m2 = sm2 + 64.0f * fmaxf(sdd - G * dm * dm, 0.0f);
    rstd = 1.0f / sqrtf(m2 / (64.0f * G) + p.ln_eps);
}

// Consumer prologue, one thread per tile row: (mean relative to the level A was stored against, rstd) into
// lnrow, and the row's mean handed on as the next level by the first column block's tiles.
__device__ __forceinline__ void ln_tile_row(const GemmArgs& p, int m0, int n0, int t, float* lnrow) {
    const bool real = m0 + t < p.M;
    const int r = real ? m0 + t : p.M - 1;
    float mean, rstd;
    ln_row_stats(p, r, mean, rstd);
    lnrow[2 * t] = mean - (p.ln_level ? p.ln_level[r] : 0.0f);
    lnrow[2 * t + 1] = rstd;
    if (p.ln_level_out && n0 == 0 && real) p.ln_level_out[r] = mean;
}

// RESID / PATCH chunk with the producer-side extras.  Called by all 8 lanes that hold the 8 chunks of one
// 64-column group of a row (consecutive lanes, chunk index = lane % 8); `active` is the same for all of them.
template <typename T>
__device__ __forceinline__ void resid_stats_chunk(const GemmArgs& p, int r, int c, float* v, bool active, int lane8) {
    int64_t orow = r;
    if (active) {
        epilogue_chunk<T>(p, r, c, v);         // leaves the updated residual values in v
        if (p.epi == EPI_PATCH) orow = (int64_t)(r / p.o_rpi) * p.o_istride + p.o_off + r % p.o_rpi;
        if (p.xb_out) {
            const float lev = p.xb_level ? p.xb_level[orow] : 0.0f;
            float rel[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) rel[i] = v[i] - lev;
            store8(reinterpret_cast<T*>(p.xb_out) + orow * p.ldo + c, rel);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    }
    if (!p.st_out) return;
    // group statistics around the group's first element (broadcast from the group's first lane), so that the
    // level of the data cancels before squaring: mean_g = v0 + s1 / 64, M2_g = s2 - s1^2 / 64
    const float v0 = __shfl(v[0], (int)(__lane_id() & ~7u));
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float d = v[i] - v0;
        s1 += d;
        s2 += d * d;
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
        s1 += __shfl_xor(s1, o);
        s2 += __shfl_xor(s2, o);
    }
    if (active && lane8 == 0)
        *reinterpret_cast<f32x2*>(p.st_out + (orow * (p.N >> 6) + (c >> 6)) * 2) =
            f32x2{v0 + s1 * (1.0f / 64.0f), fmaxf(s2 - s1 * s1 * (1.0f / 64.0f), 0.0f)};
}

// Block-level epilogue shared by the register-staged kernels.  The accumulators go through LDS
// (`smem`, free after the k loop, at least BM * BN * 4 bytes) as a row-major fp32 tile, so that
// each thread then owns 8 consecutive columns of a row: one row-index computation and 16-byte
// coalesced global accesses per chunk instead of 64 scattered 2-byte stores per lane.
// accumulator element v of lane (g, li) in block (i, j): row = 32 i + 8 (v / 4) + 4 g + v % 4, col = 32 j + li
// KG > 1: the workgroup holds KG groups of WGM x WGN waves, each with the partial sums of its share of the k
// range for the same tile; they are added in LDS in a fixed order (group 0, then 1, ...), and all KG groups'
// threads share the chunk work below.
template <typename T, int BM, int BN, int WGM, int WGN, int KG = 1>
__device__ __forceinline__ void block_epilogue(const GemmArgs& p, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32],
                                               char* smem, const float* lnrow, const float* lncs, int m0, int n0) {
    constexpr int NTG = 64 * WGM * WGN, NT = NTG * KG;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid % NTG) >> 6;
    const int kg = KG > 1 ? tid / NTG : 0;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    float* sC = reinterpret_cast<float*>(smem);
    if (p.ln_stats) {
        // folded LayerNorm: lnrow[2 row] = mean, lnrow[2 row + 1] = rstd of the tile's rows
        // lncs[j]: column sum of this lane's column in block j, loaded before the k loop
        // (the mean term belongs to the whole sum: only group 0 subtracts it)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * WM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                const f32x2 st = *reinterpret_cast<const f32x2*>(lnrow + 2 * row);
                const float mean = kg == 0 ? st[0] : 0.0f;
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j][v] = st[1] * (acc[i][j][v] - mean * lncs[j]);
            }
    }
#pragma unroll
    for (int k = 0; k < KG; ++k) {
        if (kg == k) {
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float* dst = sC + (wm * WM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * BN + wn * WN + j * 32 + li;
                        *dst = k == 0 ? acc[i][j][v] : *dst + acc[i][j][v];
                    }
        }
        __syncthreads();
    }

    if (p.epi == EPI_SWIGLU) {
        // physical columns come in groups of 64: 32 gate columns, then their 32 linear partners;
        // a thread takes 8 gate columns and their partners and writes 8 hidden units
        constexpr int CG = BN / 16, RPASS = NT / CG;
        const int cg = tid % CG, grp = cg >> 2, j0 = (cg & 3) * 8;
        const int ca = n0 + grp * 64 + j0;            // physical gate column
        if (ca + 40 <= p.N) {
            const int oc = (ca >> 6) * 32 + j0;       // hidden unit index
            T* out = reinterpret_cast<T*>(p.out);
            for (int rr = tid / CG; rr < BM; rr += RPASS) {
                const int r = m0 + rr;
                if (r >= p.M) break;
                const float* src = sC + rr * BN + grp * 64 + j0;
                float h[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float a = src[i] + p.bias[ca + i], b = src[32 + i] + p.bias[ca + 32 + i];
                    h[i] = swiglu_for<T>(a, b);
                }
                store8(out + (int64_t)r * p.ldo + oc, h);
            }
        }
        return;
    }
    if (p.epi == EPI_QKV && n0 >= 2 * p.dim) {
        // value columns: written transposed, vt[(b dim + c)][token].  A thread takes one column and 8
        // consecutive tokens (one 16-byte store); consecutive threads take consecutive token groups of
        // the same column, so a column's BM tokens leave as one contiguous run.
        constexpr int RGN = BM / 8;
        T* vt = reinterpret_cast<T*>(p.out2);
        for (int it = tid; it < BN * RGN; it += NT) {
            const int cc = it / RGN, rr = (it % RGN) * 8;
            const int r = m0 + rr, c2 = n0 + cc - 2 * p.dim;
            if (r >= p.M) continue;
            const float bias = p.bias[n0 + cc];
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = sC[(rr + k) * BN + cc] + bias;
            store_tokens8<T>(p, vt, r, c2, v);
        }
        return;
    }
    if ((p.epi == EPI_RESID || p.epi == EPI_PATCH) && (p.st_out || p.xb_out)) {
        constexpr int CG = BN / 8, RPASS = NT / CG;
        const int cg = tid % CG, c = n0 + cg * 8;
        for (int rr = tid / CG; rr < BM; rr += RPASS) {
            const int r = m0 + rr;
            const bool active = r < p.M && c < p.N;
            float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (active) {
                const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8 + 4);
                v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
                v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
            }
            resid_stats_chunk<T>(p, r, c, v, active, cg & 7);
        }
        return;
    }
    if (p.epi == EPI_ROWDOT) {
        // 8 consecutive lanes hold the 8 chunks of one 64-column group of a row: every lane takes part in
        // the exchange (out-of-range rows / columns contribute zero), the first lane of a group writes
        constexpr int CG = BN / 8, RPASS = NT / CG;
        const int cg = tid % CG, c = n0 + cg * 8;
        float* out = reinterpret_cast<float*>(p.out);
        for (int rr = tid / CG; rr < BM; rr += RPASS) {
            const int r = m0 + rr;
            float sum = 0.0f;
            if (r < p.M && c < p.N) {
                const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8 + 4);
                const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                sum = rowdot_chunk(p, c, v);
            }
            sum += __shfl_xor(sum, 1);
            sum += __shfl_xor(sum, 2);
            sum += __shfl_xor(sum, 4);
            if ((cg & 7) == 0 && r < p.M && c < p.N) out[(int64_t)r * p.ldo + (c >> 6)] = sum;
        }
        return;
    }
    {
        constexpr int CG = BN / 8, RPASS = NT / CG;
        const int cg = tid % CG, c = n0 + cg * 8;
        if (c < p.N) {
            for (int rr = tid / CG; rr < BM; rr += RPASS) {
                const int r = m0 + rr;
                if (r >= p.M) break;
                const f32x4 lo = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4*>(sC + rr * BN + cg * 8 + 4);
                float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                epilogue_chunk<T>(p, r, c, v);
            }
        }
    }
}

template <typename T, int BM, int BN, int WGM, int WGN, int AMODE>
__global__ __launch_bounds__(64 * WGM * WGN, 2) void gemm_kernel(const GemmArgs args) {
    const GemmArgs p = select_problem(args);
    constexpr int NT = 64 * WGM * WGN;
    constexpr int CE = Elem<T>::CE;
    constexpr int BK = 8 * CE;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int RPP = NT / 8;
    constexpr int A_IT = BM / RPP, B_IT = BN / RPP;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must be a multiple of the loader pass");
    constexpr int STAGE = (BM + BN) * 128;
    __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
    __shared__ __attribute__((aligned(8))) float lnrow[2 * BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    const int lrow = tid >> 3, lchunk = tid & 7;

    int tm, tn;
    tile_coords(xcd_contiguous(blockIdx.x, gridDim.x), (p.M - p.m_begin + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
    const int m0 = p.m_begin + tm * BM, n0 = tn * BN;


    const T* __restrict__ A = reinterpret_cast<const T*>(p.A);
    const T* __restrict__ W = reinterpret_cast<const T*>(p.W);

    // per-thread A row state.  Loads carry neither branches nor selects on the loaded value (either
    // would make the wave wait for the load right where it is issued): rows past M re-read row
    // M - 1 (their accumulators are never stored) and out-of-image conv taps read a page of zeros.
    const T* aptr[A_IT];
    int ay[A_IT], ax[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        int r = m0 + lrow + i * RPP;
        r = r < p.M ? r : p.M - 1;
        ay[i] = ax[i] = 0;
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
    const T* wptr = W + (int64_t)(n0 + lrow) * p.K + lchunk * CE;
    const T* zptr = reinterpret_cast<const T*>(p.zeros);

    // two register sets: the loads of k-tile kt + 2 are issued while tile kt is multiplied and tile
    // kt + 1 waits in the other set, so a global load has two tile times to arrive
    u32x4 ra[2][A_IT], rb[2][B_IT];
    auto gload = [&](int set, int kt) {
        const int k0 = kt * BK;
        if (AMODE == A_PLAIN) {
#pragma unroll
            for (int i = 0; i < A_IT; ++i) ra[set][i] = ld_global_16(aptr[i] + k0);
        } else {
            // k-tile order: channel chunk outer, tap inner -- the 9 taps of a chunk re-read the same
            // 128-byte slices of neighbouring pixels, which keeps a workgroup's L2 footprint small
            const int cc = kt / 9, tap = kt - cc * 9, c0 = cc * BK;
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
            const int64_t shift = (int64_t)(dy * p.cW + dx) * p.lda + c0;
#pragma unroll
            for (int i = 0; i < A_IT; ++i) {
                const int yy = ay[i] + dy, xx = ax[i] + dx;
                const bool ok = yy >= 0 && yy < p.cH && xx >= 0 && xx < p.cW;
                // bitwise pointer select: a ternary here is compiled to a branch around the address math
                const uint64_t mask = ok ? ~uint64_t(0) : uint64_t(0);
                const uint64_t addr = (reinterpret_cast<uint64_t>(aptr[i] + shift) & mask) |
                                      (reinterpret_cast<uint64_t>(zptr) & ~mask);
                ra[set][i] = ld_global_16(reinterpret_cast<const void*>(addr));
            }
        }
        const int kw = AMODE == A_PLAIN ? k0 : (kt % 9) * p.cC + (kt / 9) * BK;   // weight column of this k-tile
#pragma unroll
        for (int i = 0; i < B_IT; ++i) rb[set][i] = ld_global_16(wptr + (int64_t)i * RPP * p.K + kw);
    };
    auto sstore = [&](int set, int buf) {
        char* sA = smem + buf * STAGE;
        char* sB = sA + BM * 128;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sA + (r * 8 + swz(r, lchunk)) * 16) = ra[set][i];
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sB + (r * 8 + swz(r, lchunk)) * 16) = rb[set][i];
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // fragments of k-step ks + 1 are read from LDS before the MFMAs of step ks are issued
    auto compute = [&](int buf) {
        const char* sA = smem + buf * STAGE;
        const char* sB = sA + BM * 128;
        typename Mma<T>::Frag fa[2][MI], fb[2][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[0][i] = Mma<T>::load(sA, wm * WM + i * 32 + li, 0, g);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[0][j] = Mma<T>::load(sB, wn * WN + j * 32 + li, 0, g);
#pragma unroll
        for (int ks = 0; ks < Mma<T>::KS; ++ks) {
            if (ks + 1 < Mma<T>::KS) {
#pragma unroll
                for (int i = 0; i < MI; ++i) fa[(ks + 1) & 1][i] = Mma<T>::load(sA, wm * WM + i * 32 + li, ks + 1, g);
#pragma unroll
                for (int j = 0; j < NI; ++j) fb[(ks + 1) & 1][j] = Mma<T>::load(sB, wn * WN + j * 32 + li, ks + 1, g);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) Mma<T>::mma(acc[i][j], fa[ks & 1][i], fb[ks & 1][j]);
        }
    };

    // The prefetches are unconditional (tile index clamped to the last tile) so that the number of
    // loads in flight is the same on every path: with a conditional prefetch the compiler has to
    // assume it was skipped and waits for the newest loads before storing the older set.
    const int KT = p.K / BK;
    const int klast = KT - 1;
    gload(0, 0);
    gload(1, klast < 1 ? klast : 1);
    // folded LayerNorm: statistics of this tile's rows, read by the epilogue (the k loop's barriers order
    // them); placed behind the first tile loads so that it does not delay them
    float lncs[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) lncs[j] = 0.0f;
    if (p.ln_stats) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int c = n0 + wn * WN + j * 32 + li;
            if (c < p.N) lncs[j] = p.ln_colsum[c];
        }
        if (tid < BM) ln_tile_row(p, m0, n0, tid, lnrow);
    }
    sstore(0, 0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        gload(0, kt + 2 < klast ? kt + 2 : klast);
        compute(0);
        sstore(1, 1);
        __syncthreads();
        if (kt + 1 >= KT) break;
        gload(1, kt + 3 < klast ? kt + 3 : klast);
        compute(1);
        sstore(0, 0);
        __syncthreads();
    }

    static_assert(BM * BN * 4 <= 2 * STAGE, "accumulator tile must fit the stage buffers");
    block_epilogue<T, BM, BN, WGM, WGN>(p, acc, smem, lnrow, lncs, m0, n0);
}

// The same tile computed by KG groups of WGM x WGN waves, each over 1 / KG of the k range (group g the k-tiles
// [g ceil(KT / KG), (g + 1) ceil(KT / KG))), with its own pair of LDS buffers; the partial sums are added in
// LDS in a fixed order by the epilogue.  For problems with less than one tile per CU and a long k loop (the
// ViT-S fc2 GEMM, the 3x3 convolutions on the patch grid): such a loop is a serial chain of load, barrier, LDS
// read and MFMA in one wave per SIMD, and the second group's chain runs in the gaps of the first.
// Dynamic LDS: 2 KG * STAGE + 8 * BM bytes.
template <typename T, int BM, int BN, int WGM, int WGN, int AMODE, int KG>
__global__ __launch_bounds__(64 * KG * WGM * WGN, KG * WGM * WGN / 4) void gemm_splitk_kernel(const GemmArgs args) {
    const GemmArgs p = select_problem(args);
    constexpr int NTG = 64 * WGM * WGN;
    constexpr int CE = Elem<T>::CE;
    constexpr int BK = 8 * CE;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int RPP = NTG / 8;
    constexpr int A_IT = BM / RPP, B_IT = BN / RPP;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must be a multiple of the loader pass");
    constexpr int STAGE = (BM + BN) * 128;
    extern __shared__ __attribute__((aligned(16))) char smem_all[];
    float* lnrow = reinterpret_cast<float*>(smem_all + KG * 2 * STAGE);

    const int tid = threadIdx.x, kg = tid / NTG, gt = tid % NTG;
    char* smem = smem_all + kg * 2 * STAGE;
    const int lane = gt & 63, wave = gt >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int g = lane >> 5, li = lane & 31;
    const int lrow = gt >> 3, lchunk = gt & 7;

    int tm, tn;
    tile_coords(xcd_contiguous(blockIdx.x, gridDim.x), (p.M - p.m_begin + BM - 1) / BM, (p.N + BN - 1) / BN, tm, tn);
    const int m0 = p.m_begin + tm * BM, n0 = tn * BN;

    const T* __restrict__ A = reinterpret_cast<const T*>(p.A);
    const T* __restrict__ W = reinterpret_cast<const T*>(p.W);

    // loader state as in gemm_kernel: no branches or selects on loaded values, rows past M re-read row M - 1,
    // out-of-image taps read the page of zeros
    const T* aptr[A_IT];
    int ay[A_IT], ax[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        int r = m0 + lrow + i * RPP;
        r = r < p.M ? r : p.M - 1;
        ay[i] = ax[i] = 0;
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
    const T* wptr = W + (int64_t)(n0 + lrow) * p.K + lchunk * CE;
    const T* zptr = reinterpret_cast<const T*>(p.zeros);

    // this group's k-tiles: [kbeg, kbeg + kcnt) of the KT tiles; all groups run ceil(KT / KG) iterations (the
    // barriers are common), a group with fewer tiles re-loads its last one and skips the multiply
    const int KT = p.K / BK, KH = (KT + KG - 1) / KG;
    const int kbeg = kg * KH;
    const int kcnt = KT - kbeg < KH ? (KT - kbeg > 0 ? KT - kbeg : 0) : KH;
    auto tile_of = [&](int local) {
        const int t = kbeg + (local < kcnt ? local : kcnt - 1);
        return t < 0 ? 0 : (t < KT ? t : KT - 1);
    };

    u32x4 ra[2][A_IT], rb[2][B_IT];
    auto gload = [&](int set, int local) {
        const int kt = tile_of(local);
        const int k0 = kt * BK;
        if (AMODE == A_PLAIN) {
#pragma unroll
            for (int i = 0; i < A_IT; ++i) ra[set][i] = ld_global_16(aptr[i] + k0);
        } else {
            const int cc = kt / 9, tap = kt - cc * 9, c0 = cc * BK;
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
            const int64_t shift = (int64_t)(dy * p.cW + dx) * p.lda + c0;
#pragma unroll
            for (int i = 0; i < A_IT; ++i) {
                const int yy = ay[i] + dy, xx = ax[i] + dx;
                const bool ok = yy >= 0 && yy < p.cH && xx >= 0 && xx < p.cW;
                const uint64_t mask = ok ? ~uint64_t(0) : uint64_t(0);
                const uint64_t addr = (reinterpret_cast<uint64_t>(aptr[i] + shift) & mask) |
                                      (reinterpret_cast<uint64_t>(zptr) & ~mask);
                ra[set][i] = ld_global_16(reinterpret_cast<const void*>(addr));
            }
        }
        const int kw = AMODE == A_PLAIN ? k0 : (kt % 9) * p.cC + (kt / 9) * BK;
#pragma unroll
        for (int i = 0; i < B_IT; ++i) rb[set][i] = ld_global_16(wptr + (int64_t)i * RPP * p.K + kw);
    };
    auto sstore = [&](int set, int buf) {
        char* sA = smem + buf * STAGE;
        char* sB = sA + BM * 128;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sA + (r * 8 + swz(r, lchunk)) * 16) = ra[set][i];
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int r = lrow + i * RPP;
            *reinterpret_cast<u32x4*>(sB + (r * 8 + swz(r, lchunk)) * 16) = rb[set][i];
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto compute = [&](int buf) {
        const char* sA = smem + buf * STAGE;
        const char* sB = sA + BM * 128;
        typename Mma<T>::Frag fa[2][MI], fb[2][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[0][i] = Mma<T>::load(sA, wm * WM + i * 32 + li, 0, g);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[0][j] = Mma<T>::load(sB, wn * WN + j * 32 + li, 0, g);
#pragma unroll
        for (int ks = 0; ks < Mma<T>::KS; ++ks) {
            if (ks + 1 < Mma<T>::KS) {
#pragma unroll
                for (int i = 0; i < MI; ++i) fa[(ks + 1) & 1][i] = Mma<T>::load(sA, wm * WM + i * 32 + li, ks + 1, g);
#pragma unroll
                for (int j = 0; j < NI; ++j) fb[(ks + 1) & 1][j] = Mma<T>::load(sB, wn * WN + j * 32 + li, ks + 1, g);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) Mma<T>::mma(acc[i][j], fa[ks & 1][i], fb[ks & 1][j]);
        }
    };

    gload(0, 0);
    gload(1, 1);
    float lncs[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) lncs[j] = 0.0f;
    if (p.ln_stats) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int c = n0 + wn * WN + j * 32 + li;
            if (c < p.N) lncs[j] = p.ln_colsum[c];
        }
        if (tid < BM) ln_tile_row(p, m0, n0, tid, lnrow);
    }
    sstore(0, 0);
    __syncthreads();
    for (int kt = 0; kt < KH; kt += 2) {
        gload(0, kt + 2);
        if (kt < kcnt) compute(0);              // uniform per wave
        sstore(1, 1);
        __syncthreads();
        if (kt + 1 >= KH) break;
        gload(1, kt + 3);
        if (kt + 1 < kcnt) compute(1);
        sstore(0, 0);
        __syncthreads();
    }

    static_assert(BM * BN * 4 <= 2 * STAGE, "accumulator tile must fit the stage buffers");
    block_epilogue<T, BM, BN, WGM, WGN, KG>(p, acc, smem_all, lnrow, lncs, m0, n0);
}

template <typename T, int BM, int BN, int WGM, int WGN, int KG>
static inline hipError_t launch_tile_splitk(const GemmArgs& a, int amode, hipStream_t s, bool configure_only = false) {
    constexpr int lds = KG * 2 * (BM + BN) * 128 + 8 * BM;
    static_assert(lds <= 160 * 1024 && 64 * KG * WGM * WGN <= 1024, "LDS and workgroup size limits");
    static_assert(BM <= 64 * WGM * WGN, "the row statistics are taken by the first BM threads (group 0)");
    static bool configured = false;
    if (!configured) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_splitk_kernel<T, BM, BN, WGM, WGN, A_PLAIN, KG>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc == hipSuccess)
            rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_splitk_kernel<T, BM, BN, WGM, WGN, A_CONV3, KG>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc != hipSuccess) return rc;
        configured = true;
    }
    if (configure_only) return hipSuccess;
    const int tiles = cdiv(a.M - a.m_begin, BM) * cdiv(a.N, BN);
    dim3 grid(tiles, a.nz > 1 ? a.nz : 1), block(64 * KG * WGM * WGN);
    if (amode == A_PLAIN) hipLaunchKernelGGL((gemm_splitk_kernel<T, BM, BN, WGM, WGN, A_PLAIN, KG>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((gemm_splitk_kernel<T, BM, BN, WGM, WGN, A_CONV3, KG>), grid, block, lds, s, a);
    return hipGetLastError();
}

template <typename T, int BM, int BN, int WGM, int WGN>
static inline hipError_t launch_tile(const GemmArgs& a, int amode, hipStream_t s) {
    const int tiles = cdiv(a.M - a.m_begin, BM) * cdiv(a.N, BN);
    dim3 grid(tiles, a.nz > 1 ? a.nz : 1), block(64 * WGM * WGN);
    if (amode == A_PLAIN) hipLaunchKernelGGL((gemm_kernel<T, BM, BN, WGM, WGN, A_PLAIN>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((gemm_kernel<T, BM, BN, WGM, WGN, A_CONV3>), grid, block, 0, s, a);
    return hipGetLastError();
}

// Tile choice: the largest tile that still yields about two workgroups per CU; SwiGLU needs
// wave tiles of 64 columns (gate and linear partner in the same lane).
template <typename T>
static inline hipError_t launch_gemm_t(const GemmArgs& a, int amode, hipStream_t s) {
    const int nz = a.nz > 1 ? a.nz : 1;
    const int64_t t128 = (int64_t)cdiv(a.M, 128) * cdiv(a.N, 128) * nz;
    const int64_t t64x128 = (int64_t)cdiv(a.M, 64) * cdiv(a.N, 128) * nz;
    if (t128 >= 384) return launch_tile<T, 128, 128, 2, 2>(a, amode, s);
    if (t64x128 >= 384 || a.epi == EPI_SWIGLU) return launch_tile<T, 64, 128, 2, 2>(a, amode, s);
    return launch_tile<T, 64, 64, 2, 2>(a, amode, s);
}

}  // namespace vpe
