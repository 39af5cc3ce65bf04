// Fused decode kernel instances for int8 weights.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_int8(const FusedLaunch& a, const char** what) { return launch_fused_family<W_INT8>(a, what); }
}  // namespace ff
