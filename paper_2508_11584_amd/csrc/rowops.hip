// Launchers of the bandwidth-bound kernels (LayerNorm, im2col, re-layout, resampling, argmax).
#include "kernels.h"
#include "resize.h"
#include "rowops.h"

namespace vpe {

static inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

hipError_t launch_layernorm(int dtype, const float* x, int rows, int D, const float* g, const float* b,
                            float eps, void* y, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (dtype) hipLaunchKernelGGL(layernorm_kernel<bf16>, dim3(blocks_for(rows, 4)), dim3(256), 0, s, x, rows, D, g, b, eps, (bf16*)y);
    else hipLaunchKernelGGL(layernorm_kernel<float>, dim3(blocks_for(rows, 4)), dim3(256), 0, s, x, rows, D, g, b, eps, (float*)y);
    return hipGetLastError();
}

hipError_t launch_activation(int dtype, void* h, int64_t rows, int cols, int gated, hipStream_t s) {
    if (rows <= 0 || cols % 16) return rows <= 0 ? hipSuccess : hipErrorInvalidValue;
    const int64_t n = rows * ((gated ? cols / 2 : cols) / 8);
    const unsigned nb = (unsigned)((n + 255) / 256);
    if (dtype) hipLaunchKernelGGL(activation_kernel<bf16>, dim3(nb), dim3(256), 0, s, (bf16*)h, rows, cols, gated);
    else hipLaunchKernelGGL(activation_kernel<float>, dim3(nb), dim3(256), 0, s, (float*)h, rows, cols, gated);
    return hipGetLastError();
}

hipError_t launch_im2col(int dtype, const float* img, int B, int H, int W, int kpad, void* cols,
                         const float* special, int nspecial, int ntok, int D, float* x, void* xb, float* stats,
                         const float* level, hipStream_t s) {
    const int P = (H / 14) * (W / 14);
    const unsigned nb = (unsigned)(B * P + B * nspecial);
    if (dtype) hipLaunchKernelGGL(im2col_kernel<bf16>, dim3(nb), dim3(256), 0, s, img, B, H, W, kpad, (bf16*)cols, special, nspecial, ntok, D, x, (bf16*)xb, stats, level);
    else hipLaunchKernelGGL(im2col_kernel<float>, dim3(nb), dim3(256), 0, s, img, B, H, W, kpad, (float*)cols, special, nspecial, ntok, D, x, (float*)xb, stats, level);
    return hipGetLastError();
}

hipError_t launch_relayout(int dtype, const float* src, void* dst, int n_rows, int n_cols, int64_t rs,
                           int64_t cs, int mode, int cin, int swiglu_half, int64_t dst_ld, int row_off,
                           int col_off, const float* kscale, hipStream_t s) {
    const int64_t n = (int64_t)n_rows * n_cols;
    if (n <= 0) return hipSuccess;
    if (dtype) hipLaunchKernelGGL(relayout_kernel<bf16>, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, (bf16*)dst, n_rows, n_cols, rs, cs, mode, cin, swiglu_half, dst_ld, row_off, col_off, kscale);
    else hipLaunchKernelGGL(relayout_kernel<float>, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, (float*)dst, n_rows, n_cols, rs, cs, mode, cin, swiglu_half, dst_ld, row_off, col_off, kscale);
    return hipGetLastError();
}

hipError_t launch_ln_fold(int dtype, const float* src, int K, int n_out, int swiglu_half, const float* gain,
                          const float* beta, float* colsum, float* bias, hipStream_t s) {
    if (dtype) hipLaunchKernelGGL(ln_fold_kernel<bf16>, dim3(blocks_for(n_out, 256)), dim3(256), 0, s, src, K, n_out, swiglu_half, gain, beta, colsum, bias);
    else hipLaunchKernelGGL(ln_fold_kernel<float>, dim3(blocks_for(n_out, 256)), dim3(256), 0, s, src, K, n_out, swiglu_half, gain, beta, colsum, bias);
    return hipGetLastError();
}

hipError_t launch_argmax_rows(const float* in, int64_t rows, int C, int ld, uint8_t* out, hipStream_t s) {
    hipLaunchKernelGGL(argmax_rows_kernel, dim3(blocks_for(rows, 4)), dim3(256), 0, s, in, rows, C, ld, out);
    return hipGetLastError();
}

hipError_t launch_fuse_upsample(int dtype, const void* p, int gh, int gw, const void* r, int B, int Hs, int Ws,
                                int C, void* z, hipStream_t s) {
    if (Hs % 2 || Ws % 2 || Hs < 2 * gh || Ws < 2 * gw) return hipErrorInvalidValue;   // 2 x 2 output blocks of an enlargement
    if ((int64_t)Hs * Ws * C >= (int64_t(1) << 31)) return hipErrorInvalidValue;          // 32-bit offsets inside an image
    // both rows (columns) of an even-aligned block fall between the same two source samples when the factor f
    // is a multiple of 4: a sample boundary lies between outputs y and y + 1 only if f (2 j + 1) = 2 y + 2,
    // and for even y the right side is 2 mod 4
    const bool shared = Hs % (4 * gh) == 0 && Ws % (4 * gw) == 0;
    const int64_t per_row = (int64_t)(Ws / 2) * (C / (dtype ? 8 : 4));
    if (per_row >= (int64_t(1) << 31) || Hs / 2 > 65535 || B > 65535) return hipErrorInvalidValue;   // grid y, z limits
    const dim3 grid(blocks_for(per_row, 256), Hs / 2, B), block(256);
    if (dtype) {
        if (shared) hipLaunchKernelGGL((fuse_upsample_kernel<bf16, true>), grid, block, 0, s, (const bf16*)p, gh, gw, (const bf16*)r, B, Hs, Ws, C, (bf16*)z);
        else hipLaunchKernelGGL((fuse_upsample_kernel<bf16, false>), grid, block, 0, s, (const bf16*)p, gh, gw, (const bf16*)r, B, Hs, Ws, C, (bf16*)z);
    } else {
        if (shared) hipLaunchKernelGGL((fuse_upsample_kernel<float, true>), grid, block, 0, s, (const float*)p, gh, gw, (const float*)r, B, Hs, Ws, C, (float*)z);
        else hipLaunchKernelGGL((fuse_upsample_kernel<float, false>), grid, block, 0, s, (const float*)p, gh, gw, (const float*)r, B, Hs, Ws, C, (float*)z);
    }
    return hipGetLastError();
}

hipError_t launch_seg_upsample_argmax(const float* logits, int B, int gh, int gw, int C, int H, int W,
                                      uint8_t* cls, hipStream_t s) {
    const int S = H / gh;
    if (H == S * gh && W == S * gw && S >= 2 && S % 2 == 0 && S * S <= 256 && C <= 2048) {
        const unsigned cells = (unsigned)(B * (gh + 1) * (gw + 1));
        hipLaunchKernelGGL(seg_upsample_argmax_cell_kernel, dim3(cells), dim3(256), 4 * C * sizeof(float), s, logits, B, gh, gw, C, S, cls);
    } else {
        hipLaunchKernelGGL(seg_upsample_argmax_kernel, dim3(blocks_for((int64_t)B * H * W, 256)), dim3(256), 0, s, logits, B, gh, gw, C, H, W, cls);
    }
    return hipGetLastError();
}

hipError_t launch_depth_output(const float* d, int nparts, float bias, int B, int h8, int w8,
                               int H, int W, float* depth, hipStream_t s) {
    const dim3 grid(blocks_for((int64_t)B * H * W, 256)), block(256);
    if (nparts == 4) hipLaunchKernelGGL(depth_output_kernel<4>, grid, block, 0, s, d, nparts, bias, B, h8, w8, H, W, depth);
    else hipLaunchKernelGGL(depth_output_kernel<0>, grid, block, 0, s, d, nparts, bias, B, h8, w8, H, W, depth);
    return hipGetLastError();
}

hipError_t launch_resize_ac(int dtype, int out_f32, const void* src, int B, int h, int w, int ld_in, int C,
                            const void* ty, const void* tx, int H, int W, int ld_out, void* dst, hipStream_t s) {
    if (C % 8 || ld_in % 8 || ld_out % 8 || C > ld_in || C > ld_out) return hipErrorInvalidValue;
    const dim3 grid(blocks_for((int64_t)B * H * W * (C / 8), 256)), block(256);
    const AcTap *a = (const AcTap*)ty, *b = (const AcTap*)tx;
    if (!dtype) hipLaunchKernelGGL((resize_ac_kernel<float, float>), grid, block, 0, s, (const float*)src, B, h, w, ld_in, C, a, b, H, W, ld_out, (float*)dst);
    else if (out_f32) hipLaunchKernelGGL((resize_ac_kernel<bf16, float>), grid, block, 0, s, (const bf16*)src, B, h, w, ld_in, C, a, b, H, W, ld_out, (float*)dst);
    else hipLaunchKernelGGL((resize_ac_kernel<bf16, bf16>), grid, block, 0, s, (const bf16*)src, B, h, w, ld_in, C, a, b, H, W, ld_out, (bf16*)dst);
    return hipGetLastError();
}

hipError_t launch_gather3x3s2(int dtype, const void* src, int B, int h, int w, int ld, void* dst, hipStream_t s) {
    if (ld % 8) return hipErrorInvalidValue;
    const int ho = (h - 1) / 2 + 1, wo = (w - 1) / 2 + 1;
    const int64_t n = (int64_t)B * ho * wo * 9 * (ld / (dtype ? 8 : 4));
    if (dtype) hipLaunchKernelGGL(gather3x3s2_kernel<bf16>, dim3(blocks_for(n, 256)), dim3(256), 0, s, (const bf16*)src, B, h, w, ld, ho, wo, (bf16*)dst);
    else hipLaunchKernelGGL(gather3x3s2_kernel<float>, dim3(blocks_for(n, 256)), dim3(256), 0, s, (const float*)src, B, h, w, ld, ho, wo, (float*)dst);
    return hipGetLastError();
}

hipError_t launch_rowsum_relu(const float* d, int nparts, float bias, int64_t n, float* depth, hipStream_t s) {
    hipLaunchKernelGGL(rowsum_relu_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, d, nparts, bias, n, depth);
    return hipGetLastError();
}

hipError_t launch_preprocess_u8(const uint8_t* src, int B, int sh, int sw, int H, int W, const float* mean,
                                const float* stdev, float* dst, hipStream_t s) {
    Affine3 a;
    for (int c = 0; c < 3; ++c) {
        a.scale[c] = 1.0f / (255.0f * stdev[c]);
        a.shift[c] = -mean[c] / stdev[c];
    }
    hipLaunchKernelGGL(preprocess_u8_kernel, dim3(blocks_for((int64_t)B * H * W, 256)), dim3(256), 0, s, src, B, sh, sw, H, W, a, dst);
    return hipGetLastError();
}

}  // namespace vpe
