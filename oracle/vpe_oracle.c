/*
 * CPU oracle operators for the Visual Perception Engine hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product (the HIP library or its
 * Python binding) may include, link or call this file; it exists so the tests,
 * the smoke check and the benchmark's cpu_baseline leg have a slow, plain,
 * independently written statement of what the path computes.
 *
 * The paper (Sec. "Example implementation") names the networks -- a DINOv2-style
 * ViT encoder whose final and three intermediate feature maps feed a DPT depth
 * head, a linear segmentation head and a detection head -- but prints no
 * formulas.  Each operator below is therefore the textbook definition of the
 * named layer, in fp64, one loop nest per definition, no blocking or fusion.
 * OpenMP only splits the outermost independent index (rows / output channels).
 *
 * All tensors are dense row-major double arrays.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int vo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void vo_set_num_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Patch embedding: a ps x ps convolution of stride ps (ViT tokeniser).
 * img [3][H][W], w [D][3][ps][ps], b [D]  ->  out [(H/ps)*(W/ps)][D], patches row-major. */
void vo_patch_embed(const double* img, int H, int W, int ps, const double* w, const double* b, int D,
                    double* out) {
    const int gh = H / ps, gw = W / ps;
#pragma omp parallel for schedule(static)
    for (int p = 0; p < gh * gw; ++p) {
        const int i = p / gw, j = p % gw;
        for (int d = 0; d < D; ++d) {
            double acc = b[d];
            for (int c = 0; c < 3; ++c)
                for (int u = 0; u < ps; ++u)
                    for (int v = 0; v < ps; ++v)
                        acc += w[((d * 3 + c) * ps + u) * ps + v] *
                               img[((size_t)c * H + (size_t)(i * ps + u)) * W + (size_t)(j * ps + v)];
            out[(size_t)p * D + d] = acc;
        }
    }
}

/* LayerNorm over the last axis: y = g * (x - mean) / sqrt(var + eps) + b, biased variance.
 * x,y [T][D]. */
void vo_layernorm(const double* x, int T, int D, const double* g, const double* b, double eps, double* y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const double* xr = x + (size_t)t * D;
        double mean = 0.0;
        for (int d = 0; d < D; ++d) mean += xr[d];
        mean /= D;
        double var = 0.0;
        for (int d = 0; d < D; ++d) var += (xr[d] - mean) * (xr[d] - mean);
        var /= D;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int d = 0; d < D; ++d) y[(size_t)t * D + d] = g[d] * (xr[d] - mean) * rstd + b[d];
    }
}

/* Affine map y = x W + b.  x [T][K], w [K][N], b [N] (may be NULL), y [T][N]. */
void vo_linear(const double* x, int T, int K, const double* w, const double* b, int N, double* y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* yr = y + (size_t)t * N;
        for (int n = 0; n < N; ++n) yr[n] = b ? b[n] : 0.0;
        for (int k = 0; k < K; ++k) {
            const double xv = x[(size_t)t * K + k];
            const double* wr = w + (size_t)k * N;
            for (int n = 0; n < N; ++n) yr[n] += xv * wr[n];
        }
    }
}

/* Multi-head softmax attention, no mask.  qkv [N][3*D] with D = nh*dh: columns
 * [0,D) queries, [D,2D) keys, [2D,3D) values, head i owns columns dh*i..dh*i+dh-1 of each.
 * out [N][D] = concat_i softmax(q_i k_i^T / sqrt(dh)) v_i.
 * probs (optional, may be NULL): [nh][N][N] attention weights. */
void vo_attention(const double* qkv, int N, int nh, int dh, double* out, double* probs) {
    const int D = nh * dh;
    const double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(static) collapse(2)
        for (int hd = 0; hd < nh; ++hd) {
            for (int i = 0; i < N; ++i) {
                const double* q = qkv + (size_t)i * 3 * D + hd * dh;
                double mx = -INFINITY;
                for (int j = 0; j < N; ++j) {
                    const double* k = qkv + (size_t)j * 3 * D + D + hd * dh;
                    double acc = 0.0;
                    for (int e = 0; e < dh; ++e) acc += q[e] * k[e];
                    s[j] = acc * scale;
                    if (s[j] > mx) mx = s[j];
                }
                double den = 0.0;
                for (int j = 0; j < N; ++j) {
                    s[j] = exp(s[j] - mx);
                    den += s[j];
                }
                for (int j = 0; j < N; ++j) s[j] /= den;
                if (probs) memcpy(probs + ((size_t)hd * N + i) * N, s, sizeof(double) * (size_t)N);
                double* o = out + (size_t)i * D + hd * dh;
                for (int e = 0; e < dh; ++e) o[e] = 0.0;
                for (int j = 0; j < N; ++j) {
                    const double* v = qkv + (size_t)j * 3 * D + 2 * D + hd * dh;
                    for (int e = 0; e < dh; ++e) o[e] += s[j] * v[e];
                }
            }
        }
        free(s);
    }
}

/* GELU, exact form: 0.5 x (1 + erf(x / sqrt 2)).  In place. */
void vo_gelu(double* x, int64_t n) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) x[i] = 0.5 * x[i] * (1.0 + erf(x[i] / sqrt(2.0)));
}

/* SwiGLU gate: h [T][2M] = [a | b]  ->  out [T][M] = silu(a) * b, silu(a) = a / (1 + e^-a). */
void vo_swiglu(const double* h, int T, int M, double* out) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int m = 0; m < M; ++m) {
            const double a = h[(size_t)t * 2 * M + m], b = h[(size_t)t * 2 * M + M + m];
            out[(size_t)t * M + m] = a / (1.0 + exp(-a)) * b;
        }
}

/* LayerScale residual update x <- x + gamma * m, elementwise over [T][D]. */
void vo_scale_residual(double* x, const double* m, const double* gamma, int T, int D) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int d = 0; d < D; ++d) x[(size_t)t * D + d] += gamma[d] * m[(size_t)t * D + d];
}

/* 3x3 convolution, stride 1, zero padding 1.  in [Cin][H][W], w [Cout][Cin][3][3], b [Cout],
 * out [Cout][H][W]; relu != 0 applies max(0, .) after the bias. */
void vo_conv3x3(const double* in, int Cin, int H, int W, const double* w, const double* b, int Cout,
                int relu, double* out) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int co = 0; co < Cout; ++co) {
        double* o = out + (size_t)co * H * W;
        for (size_t i = 0; i < (size_t)H * W; ++i) o[i] = b ? b[co] : 0.0;
        for (int ci = 0; ci < Cin; ++ci) {
            const double* src = in + (size_t)ci * H * W;
            for (int ky = 0; ky < 3; ++ky)
                for (int kx = 0; kx < 3; ++kx) {
                    const double wv = w[((size_t)(co * Cin + ci) * 3 + ky) * 3 + kx];
                    for (int y = 0; y < H; ++y) {
                        const int sy = y + ky - 1;
                        if (sy < 0 || sy >= H) continue;
                        for (int x = 0; x < W; ++x) {
                            const int sx = x + kx - 1;
                            if (sx < 0 || sx >= W) continue;
                            o[(size_t)y * W + x] += wv * src[(size_t)sy * W + sx];
                        }
                    }
                }
        }
        if (relu)
            for (size_t i = 0; i < (size_t)H * W; ++i) o[i] = o[i] > 0.0 ? o[i] : 0.0;
    }
}

/* 1x1 convolution = per-pixel affine map.  in [Cin][HW], w [Cout][Cin], b [Cout], out [Cout][HW]. */
void vo_conv1x1(const double* in, int Cin, int64_t HW, const double* w, const double* b, int Cout, double* out) {
#pragma omp parallel for schedule(static)
    for (int co = 0; co < Cout; ++co) {
        double* o = out + (size_t)co * HW;
        for (int64_t i = 0; i < HW; ++i) o[i] = b ? b[co] : 0.0;
        for (int ci = 0; ci < Cin; ++ci) {
            const double wv = w[(size_t)co * Cin + ci];
            const double* src = in + (size_t)ci * HW;
            for (int64_t i = 0; i < HW; ++i) o[i] += wv * src[i];
        }
    }
}

/* Bilinear resize with half-pixel centres (no corner alignment).  For output row y:
 * sy = (y + 0.5) * h / H - 0.5 clamped to [0, h-1]; y0 = floor(sy); y1 = min(y0 + 1, h-1); a = sy - y0;
 * likewise along x.  in [C][h][w] -> out [C][H][W]. */
void vo_bilinear(const double* in, int C, int h, int w, int H, int W, double* out) {
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c)
        for (int y = 0; y < H; ++y) {
            double sy = (y + 0.5) * (double)h / (double)H - 0.5;
            if (sy < 0.0) sy = 0.0;
            if (sy > h - 1) sy = h - 1;
            const int y0 = (int)floor(sy);
            const int y1 = y0 + 1 < h ? y0 + 1 : h - 1;
            const double a = sy - y0;
            for (int x = 0; x < W; ++x) {
                double sx = (x + 0.5) * (double)w / (double)W - 0.5;
                if (sx < 0.0) sx = 0.0;
                if (sx > w - 1) sx = w - 1;
                const int x0 = (int)floor(sx);
                const int x1 = x0 + 1 < w ? x0 + 1 : w - 1;
                const double bx = sx - x0;
                const double* p = in + (size_t)c * h * w;
                const double top = (1.0 - bx) * p[(size_t)y0 * w + x0] + bx * p[(size_t)y0 * w + x1];
                const double bot = (1.0 - bx) * p[(size_t)y1 * w + x0] + bx * p[(size_t)y1 * w + x1];
                out[((size_t)c * H + y) * W + x] = (1.0 - a) * top + a * bot;
            }
        }
}

/* 3x3 convolution, stride 2, zero padding 1: out[co][y][x] = b[co] + sum_{ci,ky,kx} w[co][ci][ky][kx] *
 * in[ci][2y + ky - 1][2x + kx - 1] (terms outside the image are zero).  in [Cin][H][W] ->
 * out [Cout][Ho][Wo] with Ho = floor((H - 1) / 2) + 1, Wo likewise. */
void vo_conv3x3_s2(const double* in, int Cin, int H, int W, const double* w, const double* b, int Cout, double* out) {
    const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int co = 0; co < Cout; ++co)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x) {
                double acc = b ? b[co] : 0.0;
                for (int ci = 0; ci < Cin; ++ci)
                    for (int ky = 0; ky < 3; ++ky)
                        for (int kx = 0; kx < 3; ++kx) {
                            const int sy = 2 * y + ky - 1, sx = 2 * x + kx - 1;
                            if (sy < 0 || sy >= H || sx < 0 || sx >= W) continue;
                            acc += w[((size_t)(co * Cin + ci) * 3 + ky) * 3 + kx] * in[((size_t)ci * H + sy) * W + sx];
                        }
                out[((size_t)co * Ho + y) * Wo + x] = acc;
            }
}

/* Transposed convolution whose kernel size equals its stride s (no overlap, no padding): every input pixel
 * paints its own s x s block,  out[co][s y + dy][s x + dx] = b[co] + sum_ci in[ci][y][x] * w[ci][co][dy][dx].
 * in [Cin][H][W], w [Cin][Cout][s][s] (input channel first, as transposed convolutions are stored),
 * out [Cout][s H][s W]. */
void vo_conv_transpose(const double* in, int Cin, int H, int W, const double* w, const double* b, int Cout, int s,
                       double* out) {
#pragma omp parallel for schedule(static)
    for (int co = 0; co < Cout; ++co)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x)
                for (int dy = 0; dy < s; ++dy)
                    for (int dx = 0; dx < s; ++dx) {
                        double acc = b ? b[co] : 0.0;
                        for (int ci = 0; ci < Cin; ++ci)
                            acc += in[((size_t)ci * H + y) * W + x] * w[(((size_t)ci * Cout + co) * s + dy) * s + dx];
                        out[((size_t)co * s * H + (size_t)s * y + dy) * s * W + (size_t)s * x + dx] = acc;
                    }
}

/* Bilinear resize with aligned corners: output sample y sits at source coordinate sy = y (h - 1) / (H - 1)
 * (0 when H == 1), so the four corner samples are copied and the rest interpolate linearly between the two
 * nearest source rows / columns.  in [C][h][w] -> out [C][H][W]. */
void vo_bilinear_ac(const double* in, int C, int h, int w, int H, int W, double* out) {
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c)
        for (int y = 0; y < H; ++y) {
            const double sy = H > 1 ? (double)y * (double)(h - 1) / (double)(H - 1) : 0.0;
            int y0 = (int)floor(sy);
            if (y0 > h - 1) y0 = h - 1;
            const int y1 = y0 + 1 < h ? y0 + 1 : h - 1;
            const double a = sy - y0;
            for (int x = 0; x < W; ++x) {
                const double sx = W > 1 ? (double)x * (double)(w - 1) / (double)(W - 1) : 0.0;
                int x0 = (int)floor(sx);
                if (x0 > w - 1) x0 = w - 1;
                const int x1 = x0 + 1 < w ? x0 + 1 : w - 1;
                const double bx = sx - x0;
                const double* p = in + (size_t)c * h * w;
                const double top = (1.0 - bx) * p[(size_t)y0 * w + x0] + bx * p[(size_t)y0 * w + x1];
                const double bot = (1.0 - bx) * p[(size_t)y1 * w + x0] + bx * p[(size_t)y1 * w + x1];
                out[((size_t)c * H + y) * W + x] = (1.0 - a) * top + a * bot;
            }
        }
}

/* Channel argmax, ties to the lowest index.  in [C][HW] -> out [HW] (int32). */
void vo_argmax_channels(const double* in, int C, int64_t HW, int32_t* out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < HW; ++i) {
        int best = 0;
        double bv = in[i];
        for (int c = 1; c < C; ++c) {
            const double v = in[(size_t)c * HW + i];
            if (v > bv) { bv = v; best = c; }
        }
        out[i] = best;
    }
}
