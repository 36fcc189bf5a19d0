// Host-callable launchers of the gfx950 kernels, one translation unit per kernel family so
// the heavy MFMA templates compile in parallel.  dtype: 0 = fp32, 1 = bf16 (vpe_dtype).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attention.h"
#include "gemm.h"

namespace vpe {

hipError_t launch_gemm(int dtype, const GemmArgs& a, int amode, hipStream_t s);
hipError_t launch_attention(int dtype, const AttnArgs& a, hipStream_t s);
hipError_t configure_attention();
hipError_t configure_gemm();
hipError_t configure_gemm_bf16();
hipError_t configure_gemm_f32();

hipError_t launch_layernorm(int dtype, const float* x, int rows, int D, const float* g, const float* b,
                            float eps, void* y, hipStream_t s);
hipError_t launch_activation(int dtype, void* h, int64_t rows, int cols, int gated, hipStream_t s);
hipError_t launch_im2col(int dtype, const float* img, int B, int H, int W, int kpad, void* cols,
                         const float* special, int nspecial, int ntok, int D, float* x, void* xb, float* stats,
                         const float* level, hipStream_t s);
hipError_t launch_relayout(int dtype, const float* src, void* dst, int n_rows, int n_cols, int64_t rs,
                           int64_t cs, int mode, int cin, int swiglu_half, int64_t dst_ld, int row_off,
                           int col_off, const float* kscale, hipStream_t s);
hipError_t launch_ln_fold(int dtype, const float* src, int K, int n_out, int swiglu_half, const float* gain,
                          const float* beta, float* colsum, float* bias, hipStream_t s);
hipError_t launch_argmax_rows(const float* in, int64_t rows, int C, int ld, uint8_t* out, hipStream_t s);
hipError_t launch_fuse_upsample(int dtype, const void* p, int gh, int gw, const void* r, int B, int Hs, int Ws,
                                int C, void* z, hipStream_t s);
hipError_t launch_seg_upsample_argmax(const float* logits, int B, int gh, int gw, int C, int H, int W,
                                      uint8_t* cls, hipStream_t s);
hipError_t launch_depth_output(const float* d, int nparts, float bias, int B, int h8, int w8,
                               int H, int W, float* depth, hipStream_t s);

// Operators of the full DPT head; `tables` are AcTap arrays on the device (see resize.h).
// out_f32 != 0: fp32 output from an input in the engine dtype.  C multiple of 8, pitches multiples of 8.
hipError_t launch_resize_ac(int dtype, int out_f32, const void* src, int B, int h, int w, int ld_in, int C,
                            const void* ty, const void* tx, int H, int W, int ld_out, void* dst, hipStream_t s);
hipError_t launch_gather3x3s2(int dtype, const void* src, int B, int h, int w, int ld, void* dst, hipStream_t s);
hipError_t launch_rowsum_relu(const float* d, int nparts, float bias, int64_t n, float* depth, hipStream_t s);

hipError_t launch_preprocess_u8(const uint8_t* src, int B, int sh, int sw, int H, int W, const float* mean,
                                const float* stdev, float* dst, hipStream_t s);

}  // namespace vpe
