// Fused decode kernel instances for bf16 weights.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_bf16(const FusedLaunch& a, const char** what) { return launch_fused_family<W_BF16>(a, what); }
}  // namespace ff
