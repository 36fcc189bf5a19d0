// Bilinear resampling kernels (half-pixel centres, no corner alignment), channels-last.
// For output index y of an axis resized from `in` to `out` samples:
//   s = (y + 0.5) * in / out - 0.5 clamped to [0, in - 1];  i0 = floor(s);  i1 = min(i0 + 1, in - 1);
//   weight of i1 = s - i0.
#pragma once
#include "common.h"

namespace vpe {

struct Tap { int i0, i1; float w1; };

__device__ __forceinline__ Tap bilinear_tap(int y, int in, int out) {
    // s = ((2 y + 1) in - out) / (2 out), in exact integers: the tap index is an integer quotient and the
    // weight a single rounded ratio (a float s would carry an absolute error that grows with the image size)
    const int n = (2 * y + 1) * in - out, d = 2 * out;
    Tap t;
    if (n <= 0) {                       // s <= 0: clamped to the first sample
        t.i0 = 0;
        t.w1 = 0.0f;
    } else {
        // quotient by a float reciprocal, made exact by one correction step (|estimate - n / d| < 1 for the
        // image sizes that fit the 32-bit numerator)
        const float rd = __builtin_amdgcn_rcpf((float)d);      // 1 ulp; the correction step below absorbs it
        int q = (int)((float)n * rd);
        int rem = n - q * d;
        if (rem < 0) { --q; rem += d; }
        else if (rem >= d) { ++q; rem -= d; }
        t.i0 = q;
        t.w1 = (float)rem * rd;
        if (t.i0 >= in - 1) {           // s >= in - 1: clamped to the last sample
            t.i0 = in - 1;
            t.w1 = 0.0f;
        }
    }
    t.i1 = t.i0 + 1 < in ? t.i0 + 1 : in - 1;
    return t;
}

template <typename T, int CE> struct Vec;
template <> struct Vec<bf16, 8> {
    static __device__ __forceinline__ void load(const bf16* p, float* f) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (float)v[i];
    }
    static __device__ __forceinline__ void store(bf16* p, const float* f) {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (bf16)f[i];
        *reinterpret_cast<bf16x8*>(p) = v;
    }
};
template <> struct Vec<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float* f) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = v[i];
    }
    static __device__ __forceinline__ void store(float* p, const float* f) {
        *reinterpret_cast<f32x4*>(p) = f32x4{f[0], f[1], f[2], f[3]};
    }
};

// Depth-head stage input  z = bilinear(p: gh x gw -> Hs x Ws) + bilinear(r: Hs/2 x Ws/2 -> Hs x Ws),
// channels-last with C channels; r may be null (first stage with a resized tap).
//
// One thread per (2 x 2 output block at even coordinates, 16-byte channel group).  The four outputs of a
// block read overlapping source pixels, so the block is formed from at most 3 x 3 loads per source map
// instead of 4 x 4, or from 2 x 2 when the map is enlarged by a multiple of 4 (both rows and both columns
// of the block then fall between the same two source samples: `SHARED`).  Arithmetic per output
// is the plain separable form: horizontal blend of each source row, then the vertical blend.
template <typename T, int CE>
struct BlockSrc {
    // source rows a <= b <= c and, for the block's second output row, which of them its taps are
    int ra, rb, rc;
    bool lo1_is_a, hi1_is_b;
    float w0, w1;
    __device__ __forceinline__ void init(int y0, int in, int out) {
        const Tap t0 = bilinear_tap(y0, in, out), t1 = bilinear_tap(y0 + 1, in, out);
        ra = t0.i0; rb = t0.i1; rc = t1.i1;
        lo1_is_a = t1.i0 == t0.i0;
        hi1_is_b = t1.i1 == t0.i1;
        w0 = t0.w1; w1 = t1.w1;
    }
};

template <typename T, bool SHARED>
__device__ __forceinline__ void add_block(const T* __restrict__ src, int b, int h, int w, int C, int cg, int y0, int x0,
                                          int Hs, int Ws, float (&acc)[2][2][Elem<T>::CE]) {
    constexpr int CE = Elem<T>::CE;
    BlockSrc<T, CE> ys, xs;
    ys.init(y0, h, Hs);
    xs.init(x0, w, Ws);
    const T* base = src + (int64_t)b * h * w * C + cg * CE;     // offsets inside one image fit 32 bits (checked by the launcher)
    const int rows[3] = {ys.ra, ys.rb, ys.rc};
    const int xa = xs.ra * C, xb = xs.rb * C, xc = xs.rc * C;
    // horizontal blends of each source row for the block's two output columns
    float hz[3][2][CE];
#pragma unroll
    for (int i = 0; i < (SHARED ? 2 : 3); ++i) {
        const T* rp = base + rows[i] * w * C;
        float va[CE], vb[CE], vc[CE];
        Vec<T, CE>::load(rp + xa, va);
        Vec<T, CE>::load(rp + xb, vb);
        if (!SHARED) Vec<T, CE>::load(rp + xc, vc);
#pragma unroll
        for (int e = 0; e < CE; ++e) {
            hz[i][0][e] = (1.0f - xs.w0) * va[e] + xs.w0 * vb[e];
            if (SHARED) {
                hz[i][1][e] = (1.0f - xs.w1) * va[e] + xs.w1 * vb[e];
            } else {
                const float lo = xs.lo1_is_a ? va[e] : vb[e], hi = xs.hi1_is_b ? vb[e] : vc[e];
                hz[i][1][e] = (1.0f - xs.w1) * lo + xs.w1 * hi;
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < CE; ++e) {
            acc[0][k][e] += (1.0f - ys.w0) * hz[0][k][e] + ys.w0 * hz[1][k][e];
            if (SHARED) {
                acc[1][k][e] += (1.0f - ys.w1) * hz[0][k][e] + ys.w1 * hz[1][k][e];
            } else {
                const float lo = ys.lo1_is_a ? hz[0][k][e] : hz[1][k][e], hi = ys.hi1_is_b ? hz[1][k][e] : hz[2][k][e];
                acc[1][k][e] += (1.0f - ys.w1) * lo + ys.w1 * hi;
            }
        }
}

// The r map is enlarged by exactly 2: output rows 2 i and 2 i + 1 are 1/4 in[i - 1] + 3/4 in[i] and 3/4 in[i] + 1/4 in[i + 1]
// (indices clamped to the map, which is what clamping the sample position gives), likewise along x -- fixed weights and
// fixed roles of the three source rows and columns: no tap arithmetic, no selects.
template <typename T>
__device__ __forceinline__ void add_block_x2(const T* __restrict__ src, int b, int h, int w, int C, int cg, int i, int j,
                                             float (&acc)[2][2][Elem<T>::CE]) {
    constexpr int CE = Elem<T>::CE;
    const T* base = src + (int64_t)b * h * w * C + cg * CE;
    const int rows[3] = {i > 0 ? i - 1 : 0, i, i + 1 < h ? i + 1 : h - 1};
    const int ca = (j > 0 ? j - 1 : 0) * C, cb = j * C, cc = (j + 1 < w ? j + 1 : w - 1) * C;
    float hz[3][2][CE];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const T* rp = base + rows[k] * w * C;
        float va[CE], vb[CE], vc[CE];
        Vec<T, CE>::load(rp + ca, va);
        Vec<T, CE>::load(rp + cb, vb);
        Vec<T, CE>::load(rp + cc, vc);
#pragma unroll
        for (int e = 0; e < CE; ++e) {
            hz[k][0][e] = fmaf(0.75f, vb[e], 0.25f * va[e]);
            hz[k][1][e] = fmaf(0.75f, vb[e], 0.25f * vc[e]);
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < CE; ++e) {
            acc[0][k][e] += fmaf(0.75f, hz[1][k][e], 0.25f * hz[0][k][e]);
            acc[1][k][e] += fmaf(0.75f, hz[1][k][e], 0.25f * hz[2][k][e]);
        }
}

// PSHARED: the p map is enlarged by a multiple of 4 in both directions (decided by the launcher).
// Grid: x over (block column, channel group) pairs, y = block row, z = image: the row, the image and the row's taps
// are the same for a whole workgroup, and a thread's only division is by the number of channel groups.
template <typename T, bool PSHARED>
__global__ __launch_bounds__(256) void fuse_upsample_kernel(const T* __restrict__ p, int gh, int gw,
                                                            const T* __restrict__ r, int B, int Hs, int Ws,
                                                            int C, T* __restrict__ z) {
    constexpr int CE = Elem<T>::CE;
    const int groups = C / CE, bw = Ws / 2, bh = Hs / 2;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= bw * groups) return;
    const int xb = t / groups, cg = t - xb * groups;
    const int x0 = 2 * xb, yb = blockIdx.y, y0 = 2 * yb, b = blockIdx.z;
    float acc[2][2][CE];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int e = 0; e < CE; ++e) acc[i][k][e] = 0.0f;
    add_block<T, PSHARED>(p, b, gh, gw, C, cg, y0, x0, Hs, Ws, acc);
    if (r) add_block_x2<T>(r, b, bh, bw, C, cg, yb, xb, acc);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 2; ++k)
            Vec<T, CE>::store(z + ((((int64_t)b * Hs + y0 + i) * Ws + x0 + k) * C) + cg * CE, acc[i][k]);
}

// Segmentation output: class[b][y][x] = argmax_c bilinear(logits[b] : gh x gw -> H x W)[c],
// ties to the lowest index.  logits fp32 channels-last [B][gh][gw][C]; one thread per pixel.
__global__ __launch_bounds__(256) void seg_upsample_argmax_kernel(const float* __restrict__ logits, int B,
                                                                  int gh, int gw, int C, int H, int W,
                                                                  uint8_t* __restrict__ cls) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * H * W) return;
    const int x = (int)(idx % W);
    const int y = (int)((idx / W) % H), b = (int)(idx / ((int64_t)W * H));
    const Tap ty = bilinear_tap(y, gh, H), tx = bilinear_tap(x, gw, W);
    const float* base = logits + (int64_t)b * gh * gw * C;
    const float* p00 = base + ((int64_t)ty.i0 * gw + tx.i0) * C;
    const float* p01 = base + ((int64_t)ty.i0 * gw + tx.i1) * C;
    const float* p10 = base + ((int64_t)ty.i1 * gw + tx.i0) * C;
    const float* p11 = base + ((int64_t)ty.i1 * gw + tx.i1) * C;
    int best = 0;
    float bv = -INFINITY;
    for (int c = 0; c < C; ++c) {
        const float top = (1.0f - tx.w1) * p00[c] + tx.w1 * p01[c];
        const float bot = (1.0f - tx.w1) * p10[c] + tx.w1 * p11[c];
        const float v = (1.0f - ty.w1) * top + ty.w1 * bot;
        if (v > bv) { bv = v; best = c; }
    }
    cls[idx] = (uint8_t)best;
}

// The same output for an enlargement by an even integer factor S (S * S <= 256), the case of the 14 x 14
// patches: all output pixels y in [S k - S/2, S k + S/2) blend the same two source rows k - 1 and k (clamped;
// likewise along x), so one workgroup takes one such S x S cell, puts the four source logit vectors in LDS once
// and every thread (one output pixel) walks the classes reading them by broadcast -- 4 LDS reads per class
// instead of 4 global loads.  Weights come from bilinear_tap as before (at the image border it returns weight 0
// for the clamped side, so the duplicated row / column does not matter); arithmetic and tie rule are unchanged.
__global__ __launch_bounds__(256) void seg_upsample_argmax_cell_kernel(const float* __restrict__ logits, int B,
                                                                       int gh, int gw, int C, int S,
                                                                       uint8_t* __restrict__ cls) {
    extern __shared__ float sv[];                 // [4][C]: (r0, c0), (r0, c1), (r1, c0), (r1, c1)
    const int H = gh * S, W = gw * S;
    const int cj = blockIdx.x % (gw + 1), ci = (blockIdx.x / (gw + 1)) % (gh + 1), b = blockIdx.x / ((gw + 1) * (gh + 1));
    const int r0 = ci > 0 ? ci - 1 : 0, r1 = ci < gh ? ci : gh - 1;
    const int c0 = cj > 0 ? cj - 1 : 0, c1 = cj < gw ? cj : gw - 1;
    const float* base = logits + (int64_t)b * gh * gw * C;
    for (int i = threadIdx.x; i < 4 * C; i += 256) {
        const int q = i / C, c = i - q * C;
        sv[i] = base[((int64_t)(q < 2 ? r0 : r1) * gw + ((q & 1) ? c1 : c0)) * C + c];
    }
    __syncthreads();
    const int ly = threadIdx.x / S, lx = threadIdx.x - ly * S;
    const int y = ci * S - S / 2 + ly, x = cj * S - S / 2 + lx;
    if (ly >= S || y < 0 || y >= H || x < 0 || x >= W) return;
    const Tap ty = bilinear_tap(y, gh, H), tx = bilinear_tap(x, gw, W);
    int best = 0;
    float bv = -INFINITY;
    for (int c = 0; c < C; ++c) {
        const float top = (1.0f - tx.w1) * sv[c] + tx.w1 * sv[C + c];
        const float bot = (1.0f - tx.w1) * sv[2 * C + c] + tx.w1 * sv[3 * C + c];
        const float v = (1.0f - ty.w1) * top + ty.w1 * bot;
        if (v > bv) { bv = v; best = c; }
    }
    cls[((int64_t)b * H + y) * W + x] = (uint8_t)best;
}

// Depth output: depth = ReLU(bilinear(bilinear_x2(d) -> H x W)) with d fp32 [B][h8][w8] given as
// d = bias + the sum of the `nparts` partial values stored per pixel (the convolution before it leaves the
// 1-channel projection as one partial sum per 64 channels; summed here in index order, so the result does
// not depend on scheduling).  NP = 4: the four partials are one 16-byte load; NP = 0: any count.
// The x2 map is evaluated on the fly at the four positions the final resize reads.
template <int NP>
__global__ __launch_bounds__(256) void depth_output_kernel(const float* __restrict__ d, int nparts, float bias,
                                                           int B, int h8, int w8, int H, int W,
                                                           float* __restrict__ depth) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * H * W) return;
    const int x = (int)(idx % W);
    const int y = (int)((idx / W) % H), b = (int)(idx / ((int64_t)W * H));
    const int h16 = 2 * h8, w16 = 2 * w8;
    const float* src = d + (int64_t)b * h8 * w8 * nparts;
    auto at = [&](int i) {
        if (NP == 4) {
            const f32x4 q = *reinterpret_cast<const f32x4*>(src + 4 * (int64_t)i);
            return (((bias + q[0]) + q[1]) + q[2]) + q[3];
        }
        float v = bias;
        for (int k = 0; k < nparts; ++k) v += src[(int64_t)i * nparts + k];
        return v;
    };
    auto up2 = [&](int yy, int xx) {
        const Tap ty = bilinear_tap(yy, h8, h16), tx = bilinear_tap(xx, w8, w16);
        const float top = (1.0f - tx.w1) * at(ty.i0 * w8 + tx.i0) + tx.w1 * at(ty.i0 * w8 + tx.i1);
        const float bot = (1.0f - tx.w1) * at(ty.i1 * w8 + tx.i0) + tx.w1 * at(ty.i1 * w8 + tx.i1);
        return (1.0f - ty.w1) * top + ty.w1 * bot;
    };
    const Tap ty = bilinear_tap(y, h16, H), tx = bilinear_tap(x, w16, W);
    const float top = (1.0f - tx.w1) * up2(ty.i0, tx.i0) + tx.w1 * up2(ty.i0, tx.i1);
    const float bot = (1.0f - tx.w1) * up2(ty.i1, tx.i0) + tx.w1 * up2(ty.i1, tx.i1);
    depth[idx] = fmaxf((1.0f - ty.w1) * top + ty.w1 * bot, 0.0f);
}

// ---- operators of the full DPT head (maps are pixel-major: [B][h][w][ld] with C <= ld channels in use) ----

// Bilinear resize with aligned corners, TI -> TO, 8 channels per thread.  The tap tables (AcTap per output
// row and per output column) are filled on the host in exact integer arithmetic when the engine is created.
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void resize_ac_kernel(const TI* __restrict__ src, int B, int h, int w, int ld_in, int C,
                                                        const AcTap* __restrict__ ty, const AcTap* __restrict__ tx,
                                                        int H, int W, int ld_out, TO* __restrict__ dst) {
    const int cgs = C >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * H * W * cgs) return;
    const int cg = (int)(idx % cgs);
    const int64_t pix = idx / cgs;
    const int x = (int)(pix % W), y = (int)((pix / W) % H), b = (int)(pix / ((int64_t)W * H));
    const AcTap a = ty[y], c = tx[x];
    const int y1 = a.i0 + 1 < h ? a.i0 + 1 : h - 1, x1 = c.i0 + 1 < w ? c.i0 + 1 : w - 1;
    const TI* base = src + (int64_t)b * h * w * ld_in + cg * 8;
    float v00[8], v01[8], v10[8], v11[8], o[8];
    auto load = [&](int yy, int xx, float* v) {
        const TI* q = base + ((int64_t)yy * w + xx) * ld_in;
#pragma unroll
        for (int i = 0; i < 8; i += Elem<TI>::CE) Vec<TI, Elem<TI>::CE>::load(q + i, v + i);
    };
    load(a.i0, c.i0, v00); load(a.i0, x1, v01); load(y1, c.i0, v10); load(y1, x1, v11);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float top = (1.0f - c.w1) * v00[i] + c.w1 * v01[i], bot = (1.0f - c.w1) * v10[i] + c.w1 * v11[i];
        o[i] = (1.0f - a.w1) * top + a.w1 * bot;
    }
    TO* out = dst + pix * ld_out + cg * 8;
#pragma unroll
    for (int i = 0; i < 8; i += Elem<TO>::CE) Vec<TO, Elem<TO>::CE>::store(out + i, o + i);
}

// Operand of a 3x3 convolution with stride 2 and padding 1, gathered: dst [B ho wo][9 ld] with column
// tap * ld + c = src[b][2 y + tap / 3 - 1][2 x + tap % 3 - 1][c] (zero outside the image); 16-byte chunks.
template <typename T>
__global__ __launch_bounds__(256) void gather3x3s2_kernel(const T* __restrict__ src, int B, int h, int w, int ld,
                                                          int ho, int wo, T* __restrict__ dst) {
    constexpr int CE = Elem<T>::CE;
    const int chunks = ld / CE;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * ho * wo * 9 * chunks) return;
    const int ch = (int)(idx % chunks), tap = (int)((idx / chunks) % 9);
    const int64_t pix = idx / (9 * chunks);
    const int x = (int)(pix % wo), y = (int)((pix / wo) % ho), b = (int)(pix / ((int64_t)wo * ho));
    const int sy = 2 * y + tap / 3 - 1, sx = 2 * x + tap % 3 - 1;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (sy >= 0 && sy < h && sx >= 0 && sx < w)
        v = ld_global_16(src + (((int64_t)b * h + sy) * w + sx) * ld + ch * CE);
    *reinterpret_cast<u32x4*>(dst + (pix * 9 + tap) * ld + ch * CE) = v;
}

// depth[i] = max(bias + sum of the nparts partial projections of pixel i, 0).
__global__ __launch_bounds__(256) void rowsum_relu_kernel(const float* __restrict__ d, int nparts, float bias, int64_t n,
                                                          float* __restrict__ depth) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    float v = bias;
    for (int k = 0; k < nparts; ++k) v += d[idx * nparts + k];
    depth[idx] = fmaxf(v, 0.0f);
}

// Camera-frame transform (paper, Sec. "Transforms": type conversion, resizing and normalisation in front of
// the foundation model): src uint8 [B][sh][sw][3] interleaved RGB -> dst fp32 [B][3][H][W] with
//   dst[c] = (bilinear(src[..., c] / 255 : sh x sw -> H x W) - mean[c]) / std[c],
// half-pixel centres, no antialiasing filter.  scale[c] = 1 / (255 std[c]), shift[c] = -mean[c] / std[c].
// One thread per output pixel; the three channel planes are written with unit stride along x.
struct Affine3 { float scale[3], shift[3]; };

__global__ __launch_bounds__(256) void preprocess_u8_kernel(const uint8_t* __restrict__ src, int B, int sh, int sw,
                                                            int H, int W, Affine3 a, float* __restrict__ dst) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * H * W) return;
    const int x = (int)(idx % W);
    const int y = (int)((idx / W) % H), b = (int)(idx / ((int64_t)W * H));
    const Tap ty = bilinear_tap(y, sh, H), tx = bilinear_tap(x, sw, W);
    const uint8_t* base = src + (int64_t)b * sh * sw * 3;
    const uint8_t* p00 = base + ((int64_t)ty.i0 * sw + tx.i0) * 3;
    const uint8_t* p01 = base + ((int64_t)ty.i0 * sw + tx.i1) * 3;
    const uint8_t* p10 = base + ((int64_t)ty.i1 * sw + tx.i0) * 3;
    const uint8_t* p11 = base + ((int64_t)ty.i1 * sw + tx.i1) * 3;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const float top = (1.0f - tx.w1) * (float)p00[c] + tx.w1 * (float)p01[c];
        const float bot = (1.0f - tx.w1) * (float)p10[c] + tx.w1 * (float)p11[c];
        const float v = (1.0f - ty.w1) * top + ty.w1 * bot;
        dst[(((int64_t)b * 3 + c) * H + y) * W + x] = v * a.scale[c] + a.shift[c];
    }
}

}  // namespace vpe
