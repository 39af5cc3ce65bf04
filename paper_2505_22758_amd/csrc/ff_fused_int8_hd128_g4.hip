// Fused decode kernel instances: int8 weights, head_dim 128, 4 query heads per kv head.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_int8_hd128_g4(const FusedLaunch& a, const char** what) { return launch_fused_family<W_INT8, 128, 4>(a, what); }
}  // namespace ff
