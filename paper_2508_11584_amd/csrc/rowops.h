// Bandwidth-bound row kernels: LayerNorm, patch gathering (im2col), weight re-layout at
// engine creation and channel argmax.  All are coalesced along the
// contiguous (channel) axis; one wavefront owns one row.
#pragma once
#include "common.h"

namespace vpe {

// Stand-alone MLP activation over a hidden buffer h [rows][cols] in place, 8 elements per thread: the bandwidth-bound
// pass that the GEMM epilogues make unnecessary (kept for measuring what the fusion saves).  gated == 0: erf-GELU of
// every element; gated != 0: column j < cols / 2 becomes SiLU(h[j]) * h[j + cols / 2] (cols multiple of 16).
template <typename T>
__global__ __launch_bounds__(256) void activation_kernel(T* __restrict__ h, int64_t rows, int cols, int gated) {
    const int per_row = (gated ? cols / 2 : cols) / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * per_row) return;
    const int64_t r = idx / per_row;
    const int c = (int)(idx - r * per_row) * 8;
    T* p = h + r * cols + c;
    float v[8], w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = to_f32(p[i]);
    if (gated) {
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = to_f32(p[cols / 2 + i]);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = swiglu_for<T>(v[i], w[i]);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = gelu_for<T>(v[i]);
    }
    store8(p, v);
}


// LayerNorm over the last axis of the fp32 residual stream: y = g (x - mean) / sqrt(var + eps) + b
// with the biased variance; statistics in fp32 (mean first, then centred second moment, both
// from registers).  One wave per row, 4 rows per workgroup.  D multiple of 64, D <= 64 * 32.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_kernel(const float* __restrict__ x, int rows, int D,
                                                        const float* __restrict__ gam,
                                                        const float* __restrict__ bet, float eps,
                                                        T* __restrict__ y) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= rows) return;
    constexpr int MAXV = 16;                     // float2 per lane -> D <= 2048
    const int nv = D >> 7;                       // full float2 passes (128 elements each)
    const bool tail = (D & 64) != 0;             // one extra pass of single floats
    const float* xr = x + (int64_t)row * D;
    f32x2 v[MAXV];
    float t = 0.0f, sum = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i)
        if (i < nv) {
            v[i] = *reinterpret_cast<const f32x2*>(xr + i * 128 + 2 * lane);
            sum += v[i][0] + v[i][1];
        }
    if (tail) { t = xr[nv * 128 + lane]; sum += t; }
    const float mean = wave_sum(sum) / D;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i)
        if (i < nv) {
            const float a = v[i][0] - mean, b = v[i][1] - mean;
            sq += a * a + b * b;
        }
    if (tail) sq += (t - mean) * (t - mean);
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / D + eps);
    T* yr = y + (int64_t)row * D;
#pragma unroll
    for (int i = 0; i < MAXV; ++i)
        if (i < nv) {
            const int c = i * 128 + 2 * lane;
            const f32x2 gg = *reinterpret_cast<const f32x2*>(gam + c);
            const f32x2 bb = *reinterpret_cast<const f32x2*>(bet + c);
            yr[c] = from_f32<T>(gg[0] * (v[i][0] - mean) * rstd + bb[0]);
            yr[c + 1] = from_f32<T>(gg[1] * (v[i][1] - mean) * rstd + bb[1]);
        }
    if (tail) {
        const int c = nv * 128 + lane;
        yr[c] = from_f32<T>(gam[c] * (t - mean) * rstd + bet[c]);
    }
}

// Patch gathering for the 14x14 stride-14 embedding: row (b, p) of `cols` receives the 588
// pixels of patch p in (channel, row, column) order, zero-padded to kpad columns.  The same
// launch also fills the non-patch rows of the residual stream (CLS + pos[0], then registers)
// from the `special` table [1 + R][D], together with their copy in T minus the row's level (xb, level; may be
// null) and the (mean, sum
// of squared deviations) of each of their 64-column groups (stats [rows][D / 64][2], may be null) -- what
// the GEMM epilogues produce for the other rows.  blocks [0, B*P) gather; the rest write special rows.
template <typename T>
__global__ __launch_bounds__(256) void im2col_kernel(const float* __restrict__ img, int B, int H, int W,
                                                     int kpad, T* __restrict__ cols,
                                                     const float* __restrict__ special, int nspecial,
                                                     int ntok, int D, float* __restrict__ x,
                                                     T* __restrict__ xb, float* __restrict__ stats,
                                                     const float* __restrict__ level) {
    const int gw = W / 14, P = (H / 14) * gw;
    int blk = blockIdx.x;
    if (blk < B * P) {
        const int b = blk / P, p = blk % P, pi = p / gw, pj = p % gw;
        const float* src = img + (int64_t)b * 3 * H * W;
        for (int k = threadIdx.x; k < kpad; k += 256) {
            float v = 0.0f;
            if (k < 588) {
                const int c = k / 196, u = (k % 196) / 14, w = k % 14;
                v = src[((int64_t)c * H + pi * 14 + u) * W + pj * 14 + w];
            }
            cols[(int64_t)blk * kpad + k] = from_f32<T>(v);
        }
    } else {
        blk -= B * P;
        const int b = blk / nspecial, r = blk % nspecial;
        const int64_t row = (int64_t)b * ntok + r;
        const int lane = threadIdx.x & 63;
        for (int grp = threadIdx.x >> 6; grp < D / 64; grp += 4) {      // one wave per 64-column group
            const int d = grp * 64 + lane;
            const float v = special[(int64_t)r * D + d];
            x[row * D + d] = v;
            if (xb) xb[row * D + d] = from_f32<T>(v - (level ? level[row] : 0.0f));
            const float mean = wave_sum(v) * (1.0f / 64.0f);
            const float m2 = wave_sum((v - mean) * (v - mean));
            if (stats && lane == 0) {
                stats[(row * (D / 64) + grp) * 2] = mean;
                stats[(row * (D / 64) + grp) * 2 + 1] = m2;
            }
        }
    }
}

// Weight re-layout at engine creation: dst[(row_off + n)][col_off + k] = src element (n, k).
//   mode 0: src index = n * rs + k * cs                       (any strided 2-D view)
//   mode 1: src is a conv kernel [n][cin][3][3]; k = tap * cin + ci -> src[(n * cin + ci) * 9 + tap], written to
//           column tap * cs + ci when cs > 0 (channel pitch of a zero-padded operand), else to column k
//   swiglu != 0: physical row n reads logical row  32 (n / 64) + n % 64          if n % 64 < 32
//                                                  half + 32 (n / 64) + n % 64 - 32   otherwise
//   kscale != null: element (n, k) is multiplied by kscale[k] before rounding (a LayerNorm gain folded in)
__device__ __forceinline__ int swiglu_row(int n, int swiglu_half) {
    if (!swiglu_half) return n;
    const int grp = n >> 6, j = n & 63;
    return j < 32 ? 32 * grp + j : swiglu_half + 32 * grp + j - 32;
}

template <typename T>
__global__ __launch_bounds__(256) void relayout_kernel(const float* __restrict__ src, T* __restrict__ dst,
                                                       int n_rows, int n_cols, int64_t rs, int64_t cs,
                                                       int mode, int cin, int swiglu_half, int64_t dst_ld,
                                                       int row_off, int col_off, const float* __restrict__ kscale) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)n_rows * n_cols) return;
    const int n = (int)(idx / n_cols), k = (int)(idx % n_cols);
    const int nl = swiglu_row(n, swiglu_half);
    int64_t si;
    int kd = k;
    if (mode == 0) si = nl * rs + k * cs;
    else {
        const int tap = k / cin, ci = k % cin;
        si = ((int64_t)nl * cin + ci) * 9 + tap;
        if (cs > 0) kd = tap * (int)cs + ci;
    }
    dst[(int64_t)(row_off + n) * dst_ld + col_off + kd] = from_f32<T>(kscale ? src[si] * kscale[k] : src[si]);
}

// Companion of a re-layout with a folded LayerNorm (y = LN(x) W + b with gain g and shift beta):
//   colsum[n] = sum_k w'[n][k]  with w' = the re-laid, gain-scaled and ROUNDED weight (what the MFMA multiplies),
//   bias[n]  += sum_k beta[k] * w[k][n]   (unscaled, unrounded weight),
// for physical row n (SwiGLU order as in relayout_kernel).  src is the linear weight [K][n_out] in fp32.
// One thread per output column; the K-long sums run in double.
template <typename T>
__global__ __launch_bounds__(256) void ln_fold_kernel(const float* __restrict__ src, int K, int n_out, int swiglu_half,
                                                      const float* __restrict__ gain, const float* __restrict__ beta,
                                                      float* __restrict__ colsum, float* __restrict__ bias) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= n_out) return;
    const int nl = swiglu_row(n, swiglu_half);
    double cs = 0.0, bb = 0.0;
    for (int k = 0; k < K; ++k) {
        const float w = src[(int64_t)k * n_out + nl];
        cs += (double)to_f32(from_f32<T>(w * gain[k]));
        bb += (double)beta[k] * (double)w;
    }
    colsum[n] = (float)cs;
    bias[n] += (float)bb;
}

// Per-row argmax over the first C of `ld` fp32 values (ties -> lowest index); one wave per row:
// each lane scans a strided subset in ascending order, then a butterfly keeps the larger value and,
// among equal values, the lower index.
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ in, int64_t rows, int C,
                                                          int ld, uint8_t* __restrict__ out) {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= rows) return;
    const float* p = in + r * ld;
    float bv = -INFINITY;
    int best = 0x7fffffff;
    for (int c = lane; c < C; c += 64) {
        const float v = p[c];
        if (v > bv) { bv = v; best = c; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(best, o);
        if (ov > bv || (ov == bv && oi < best)) { bv = ov; best = oi; }
    }
    if (lane == 0) out[r] = (uint8_t)best;
}

}  // namespace vpe
