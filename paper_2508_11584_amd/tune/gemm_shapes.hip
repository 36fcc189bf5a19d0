// Calibration harness for the GEMM tile choice in csrc/gemm_bf16.hip: times every tiling on the GEMM and
// 3x3-convolution shapes of the five benchmark configurations (random bf16 operands, plain store epilogue) and
// prints one line per shape.  Pipe the output into fit_tile_model.py to refit the coefficients.
//
//   hipcc -O3 --offload-arch=gfx950 -std=c++17 -I../csrc -I../../include \
//         -Xclang -target-feature -Xclang -packed-fp32-ops gemm_shapes.hip -o gemm_shapes
//   ./gemm_shapes | python fit_tile_model.py
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "gemm_dma.h"
using namespace vpe;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)

template <typename F> float timeit(F f, int reps) {
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    f(); f();
    hipEventRecord(e0);
    for (int i = 0; i < reps; ++i) f();
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    hipError_t e = hipGetLastError(); if (e != hipSuccess) printf("ERR %s\n", hipGetErrorString(e));
    return ms / reps;
}

__global__ void fill(uint16_t* p, size_t n, uint32_t seed) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    uint32_t x = (uint32_t)i * 2654435761u + seed; x ^= x >> 13; x *= 0x5bd1e995u; x ^= x >> 15;
    float v = ((x & 0xffff) / 65536.0f - 0.5f) * 0.25f;
    uint32_t b = __float_as_uint(v);
    p[i] = (uint16_t)(b >> 16);
}

int main(int argc, char** argv) {
    struct Shape { int M, N, K; const char* name; int cH = 0, cW = 0, cC = 0; };
    std::vector<Shape> shapes = {
        {1531, 1152, 384, "cfg2 qkv"}, {1531, 384, 384, "cfg2 proj"}, {1531, 1536, 384, "cfg2 fc1"}, {1531, 384, 1536, "cfg2 fc2"},
        {1530, 384, 640, "cfg2 patch"}, {1530, 256, 384, "cfg2 tapproj"},
        {97920, 256, 2304, "cfg2 conv3", 272, 360, 256}, {24480, 256, 2304, "cfg2 conv2", 136, 180, 256},
        {6120, 256, 2304, "cfg2 conv1", 68, 90, 256}, {1530, 256, 2304, "cfg2 conv0", 34, 45, 256},
        {1530, 512, 3456, "cfg2 det", 34, 45, 384},
        {87616, 256, 2304, "cfg3 conv3", 296, 296, 256}, {21904, 256, 2304, "cfg3 conv2", 148, 148, 256},
        {350464, 256, 2304, "cfg4 conv3", 296, 296, 256},
        {1370, 2304, 768, "cfg3 qkv"}, {1370, 768, 768, "cfg3 proj"}, {1370, 3072, 768, "cfg3 fc1"}, {1370, 768, 3072, "cfg3 fc2"},
        {5496, 3072, 1024, "cfg4 qkv"}, {5496, 1024, 1024, "cfg4 proj"}, {5496, 4096, 1024, "cfg4 fc1"}, {5496, 1024, 4096, "cfg4 fc2"},
        {10992, 4608, 1536, "cfg5 qkv"}, {10992, 1536, 1536, "cfg5 proj"}, {10992, 8192, 1536, "cfg5 fc1"}, {10992, 1536, 4096, "cfg5 fc2"},
        {5476, 256, 1024, "cfg4 tapproj"}, {5476, 512, 9216, "cfg4 det conv-as-gemm"},
    };
    size_t maxA = 0, maxW = 0, maxO = 0;
    for (auto& s : shapes) { maxA = std::max(maxA, (size_t)s.M * (s.cC ? s.cC : s.K)); maxW = std::max(maxW, (size_t)(s.N + 256) * s.K); maxO = std::max(maxO, (size_t)s.M * s.N); }
    uint16_t *A, *W, *O; float* bias;
    CK(hipMalloc(&A, maxA * 2)); CK(hipMalloc(&W, maxW * 2)); CK(hipMalloc(&O, maxO * 2)); CK(hipMalloc(&bias, 16384 * 4));
    fill<<<(maxA + 255) / 256, 256>>>(A, maxA, 1); fill<<<(maxW + 255) / 256, 256>>>(W, maxW, 2);
    CK(hipMemset(bias, 0, 16384 * 4));
    CK(hipDeviceSynchronize());
    for (auto& s : shapes) {
        GemmArgs a{};
        a.A = A; a.lda = s.K; a.W = W; a.bias = bias; a.M = s.M; a.N = s.N; a.K = s.K;
        a.a_rpi = s.M; a.o_rpi = s.M; a.epi = EPI_STORE; a.act = ACT_NONE; a.out = O; a.ldo = s.N;
        const int amode = s.cC ? A_CONV3 : A_PLAIN;
        if (s.cC) { a.lda = s.cC; a.cH = s.cH; a.cW = s.cW; a.cC = s.cC; a.a_istride = s.cH * s.cW; a.zeros = bias; a.act = ACT_RELU; }
        const double fl = 2.0 * s.M * s.N * s.K;
        const int reps = 20;
        float t[8];
        t[0] = timeit([&] { launch_gemm_dma<128, 32, 2, 4, 2, 2>(a, amode, 0); }, reps);
        t[1] = timeit([&] { launch_gemm_dma<256, 64, 2, 4, 2, 1>(a, amode, 0); }, reps);
        t[2] = timeit([&] { launch_gemm_dma<256, 32, 2, 4, 2, 1, 384>(a, amode, 0); }, reps);
        t[3] = timeit([&] { launch_tile<bf16, 128, 128, 2, 2>(a, amode, 0); }, reps);
        t[4] = timeit([&] { launch_tile<bf16, 64, 128, 2, 2>(a, amode, 0); }, reps);
        t[5] = timeit([&] { launch_tile<bf16, 64, 64, 2, 2>(a, amode, 0); }, reps);
        t[6] = timeit([&] { launch_gemm_dma<64, 64, 2, 2, 2, 2, 64>(a, amode, 0); }, reps);
        t[7] = timeit([&] { launch_gemm_dma<128, 64, 2, 2, 2, 2, 64>(a, amode, 0); }, reps);
        printf("%-22s M=%5d N=%5d K=%5d |", s.name, s.M, s.N, s.K);
        const char* names[8] = {"d256x128", "d256x256", "d384x256", "r128x128", "r64x128", "r64x64", "d64x64", "d64x128"};
        for (int k = 0; k < 8; ++k) printf(" %s %7.1fus %4.0fTF |", names[k], t[k] * 1e3, fl / t[k] / 1e9);
        printf("\n");
        fflush(stdout);
    }
    return 0;
}
