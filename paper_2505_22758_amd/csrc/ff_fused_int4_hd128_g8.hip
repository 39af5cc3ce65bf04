// Fused decode kernel instances: int4 weights, head_dim 128, 8 query heads per kv head.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_int4_hd128_g8(const FusedLaunch& a, const char** what) { return launch_fused_family<W_INT4, 128, 8>(a, what); }
}  // namespace ff
