// Instantiations of the flash-style attention kernel and the choice of workgroup shape.
#include <cstdlib>

#include "kernels.h"
namespace vpe {

// variant = QB * 100 + QW * 10 + KW
template <typename T>
static hipError_t launch_variant(int variant, const AttnArgs& a, hipStream_t s, bool cfg = false) {
    switch (variant) {
        case 114: return launch_attention_variant<T, 1, 1, 4>(a, s, cfg);
        case 141: return launch_attention_variant<T, 1, 4, 1>(a, s, cfg);
        default: break;
    }
    if constexpr (sizeof(T) == 2) {
        switch (variant) {
            case 214: return launch_attention_variant<T, 2, 1, 4>(a, s, cfg);
            case 122: return launch_attention_variant<T, 1, 2, 2>(a, s, cfg);
            case 124: return launch_attention_variant<T, 1, 2, 4>(a, s, cfg);
            case 224: return launch_attention_variant<T, 2, 2, 4>(a, s, cfg);
            default: break;
        }
    }
    return hipErrorInvalidValue;
}

// VPE_ATTN_VARIANT = 100 QB + 10 QW + KW overrides the choice of shape (tuning aid; read when an engine is created).
static int g_forced_variant = 0;

// LDS opt-in for every instantiation; called once at engine creation, outside any stream capture.
hipError_t configure_attention() {
    const char* env = getenv("VPE_ATTN_VARIANT");
    g_forced_variant = env ? atoi(env) : 0;
    static const int all[] = {114, 141, 214, 122, 124, 224};
    AttnArgs a{};
    for (int v : all) {
        hipError_t rc = launch_variant<bf16>(v, a, nullptr, true);
        if (rc != hipSuccess) return rc;
    }
    hipError_t rc = launch_variant<float>(114, a, nullptr, true);
    if (rc != hipSuccess) return rc;
    return launch_variant<float>(141, a, nullptr, true);
}

hipError_t launch_attention(int dtype, const AttnArgs& a, hipStream_t s) {
    const int forced = g_forced_variant;
    // Workgroup shapes measured on MI355X (QB, QW, KW = query blocks per wave, query waves, key waves), us:
    //                                         (1,2,4) (1,2,2) (2,2,4) (1,4,1) (1,4,2) (1,8,1)
    //   ViT-S 476x630   (6 x N 1531)            14.0    15.1    22.3    23.5    19.6      -
    //   ViT-B 518x518   (12 x N 1370)           25.9    20.3    22.4    22.7      -     31.1
    //   ViT-L 518x518 x4 (64 x N 1374)          80.2    59.0    67.6    50.9      -     76.2
    //   ViT-g 518x518 x8 (192 x N 1374)        217.0   153.6   190.7   145.0   164.3   182.0
    // Few (head, 32-query block) pairs want the key axis split over waves to fill the chip; many want four
    // query waves sharing each key tile and no merge.  Wider workgroups (eight query waves, or two query blocks per
    // wave) halve the L2 -> LDS traffic and are slower all the same; narrower ones (two waves) double it and are
    // slower too.
    // Beside other streams' kernels the footprint counts for more than the time alone: (1,2,4) holds a CU's LDS
    // (128 KB) for itself, (1,2,2) takes half and four waves.  ViT-S 476x630, three encoder lanes + heads: 1968 against
    // 1888 frames/s with (1,2,2), although the kernel alone takes 14.3 against 13.0 us (and frame latency 1.069
    // against 1.058 ms); even (1,4,1) -- 32 KB, 22.5 us alone -- gives 1941.
    const int64_t qblocks = (int64_t)cdiv(a.N, 32) * a.B * a.heads;
    int variant = qblocks >= 2048 ? 141 : (qblocks >= 400 || a.shared_gpu) ? 122 : 124;
    if (forced) variant = forced;
    return dtype ? launch_variant<bf16>(variant, a, s) : launch_variant<float>(forced == 141 || qblocks >= 2048 ? 141 : 114, a, s);
}
}  // namespace vpe
