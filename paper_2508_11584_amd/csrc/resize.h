// Bilinear resampling kernels (half-pixel centres, no corner alignment), channels-last.
// For output index y of an axis resized from `in` to `out` samples:
//   s = (y + 0.5) * in / out - 0.5 clamped to [0, in - 1];  i0 = floor(s);  i1 = min(i0 + 1, in - 1);
//   weight of i1 = s - i0.
#pragma once
#include "common.h"

namespace vpe {

struct Tap { int i0, i1; float w1; };

__device__ __forceinline__ Tap bilinear_tap(int y, int in, int out) {
    // (2 y + 1) * in is exact in integers; one division, one subtraction
    float s = (float)((2 * y + 1) * in) / (float)(2 * out) - 0.5f;
    s = fminf(fmaxf(s, 0.0f), (float)(in - 1));
    Tap t;
    t.i0 = (int)s;
    t.i1 = t.i0 + 1 < in ? t.i0 + 1 : in - 1;
    t.w1 = s - (float)t.i0;
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
// channels-last with C channels; r may be null (first stage with a resized tap).  One thread
// per (pixel, 16-byte channel group).
template <typename T>
__global__ __launch_bounds__(256) void fuse_upsample_kernel(const T* __restrict__ p, int gh, int gw,
                                                            const T* __restrict__ r, int B, int Hs, int Ws,
                                                            int C, T* __restrict__ z) {
    constexpr int CE = Elem<T>::CE;
    const int groups = C / CE;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * Hs * Ws * groups) return;
    const int cg = (int)(idx % groups);
    int64_t pix = idx / groups;
    const int x = (int)(pix % Ws);
    pix /= Ws;
    const int y = (int)(pix % Hs), b = (int)(pix / Hs);
    float acc[CE];
#pragma unroll
    for (int i = 0; i < CE; ++i) acc[i] = 0.0f;
    auto add = [&](const T* src, int h, int w) {
        const Tap ty = bilinear_tap(y, h, Hs), tx = bilinear_tap(x, w, Ws);
        const T* base = src + (int64_t)b * h * w * C + cg * CE;
        float v00[CE], v01[CE], v10[CE], v11[CE];
        Vec<T, CE>::load(base + ((int64_t)ty.i0 * w + tx.i0) * C, v00);
        Vec<T, CE>::load(base + ((int64_t)ty.i0 * w + tx.i1) * C, v01);
        Vec<T, CE>::load(base + ((int64_t)ty.i1 * w + tx.i0) * C, v10);
        Vec<T, CE>::load(base + ((int64_t)ty.i1 * w + tx.i1) * C, v11);
#pragma unroll
        for (int i = 0; i < CE; ++i) {
            const float top = (1.0f - tx.w1) * v00[i] + tx.w1 * v01[i];
            const float bot = (1.0f - tx.w1) * v10[i] + tx.w1 * v11[i];
            acc[i] += (1.0f - ty.w1) * top + ty.w1 * bot;
        }
    };
    add(p, gh, gw);
    if (r) add(r, Hs / 2, Ws / 2);
    Vec<T, CE>::store(z + ((((int64_t)b * Hs + y) * Ws + x) * C) + cg * CE, acc);
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

// Depth output: depth = ReLU(bilinear(bilinear_x2(d) -> H x W)) with d fp32 [B][h8][w8] given as
// d = bias + the sum of `nparts` partial maps `part_stride` floats apart (the convolution before it leaves
// the 1-channel projection as one partial sum per 64 channels).  The x2 map is evaluated on the fly at the
// four positions the final resize reads.
__global__ __launch_bounds__(256) void depth_output_kernel(const float* __restrict__ d, int nparts,
                                                           int64_t part_stride, float bias, int B, int h8, int w8,
                                                           int H, int W, float* __restrict__ depth) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * H * W) return;
    const int x = (int)(idx % W);
    const int y = (int)((idx / W) % H), b = (int)(idx / ((int64_t)W * H));
    const int h16 = 2 * h8, w16 = 2 * w8;
    const float* src = d + (int64_t)b * h8 * w8;
    auto at = [&](int i) {
        float v = bias;
        for (int k = 0; k < nparts; ++k) v += src[k * part_stride + i];     // fixed order: deterministic
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

}  // namespace vpe
