// Instantiations of the flash-style attention kernel.
#include "kernels.h"
namespace vpe {
hipError_t launch_attention(int dtype, const AttnArgs& a, hipStream_t s) {
    return dtype ? launch_attention_t<bf16>(a, s) : launch_attention_t<float>(a, s);
}
}  // namespace vpe
