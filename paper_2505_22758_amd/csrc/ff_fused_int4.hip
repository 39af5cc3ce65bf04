// Fused decode kernel instances for int4 weights.
#include "ff_fused.h"
namespace ff {
hipError_t launch_fused_int4(const FusedLaunch& a, const char** what) { return launch_fused_family<W_INT4>(a, what); }
}  // namespace ff
