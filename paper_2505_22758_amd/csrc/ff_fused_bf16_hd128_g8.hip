// Fused decode kernel instances: bf16 weights, head_dim 128, 8 query heads per kv head.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_bf16_hd128_g8(const FusedLaunch& a, const char** what) { return launch_fused_family<W_BF16, 128, 8>(a, what); }
}  // namespace ff
