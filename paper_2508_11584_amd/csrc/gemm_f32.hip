// fp32-operand instantiations of the MFMA GEMM, plus the dtype dispatch.
#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s);
hipError_t launch_gemm(int dtype, const GemmArgs& a, int amode, hipStream_t s) {
    return dtype ? launch_gemm_bf16(a, amode, s) : launch_gemm_t<float>(a, amode, s);
}
}  // namespace vpe
