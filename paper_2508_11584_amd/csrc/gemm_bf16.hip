// bf16-operand instantiations of the MFMA GEMM.
#include "kernels.h"
namespace vpe {
hipError_t launch_gemm_bf16(const GemmArgs& a, int amode, hipStream_t s) { return launch_gemm_t<bf16>(a, amode, s); }
}  // namespace vpe
