// Stand-ins for the kernel launchers of libspa2 in the host-sanitizer build of the argument checks: a rejected
// call must never reach one of them, so each aborts.
#include <cstdio>
#include <cstdlib>

#include "spa2_internal.h"

namespace spa2 {
[[noreturn]] static void reached(const char* what) {
  std::fprintf(stderr, "a rejected call reached %s\n", what);
  std::abort();
}
hipError_t launch_pool(const void*, const void*, const Dims&, float*, float*, hipStream_t) { reached("launch_pool"); }
hipError_t launch_select(const float*, const float*, const Dims&, int, float, float, uint8_t*, int32_t*, int32_t*, float*,
                         hipStream_t) { reached("launch_select"); }
hipError_t launch_columns(const uint8_t*, const Dims&, int32_t*, int32_t*, int32_t*, hipStream_t) { reached("launch_columns"); }
hipError_t launch_pattern_full(const Dims&, uint8_t*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, hipStream_t) {
  reached("launch_pattern_full");
}
hipError_t launch_fwd(const void*, const void*, const void*, const Dims&, const int32_t*, const int32_t*, const int32_t*,
                      float, void*, void*, float*, const SplitPlan&, hipStream_t) { reached("launch_fwd"); }
size_t fwd_slot_bytes(const Dims& m) { return (size_t)(256 * (m.d / 2) + 512) * 4; }
size_t dq_slot_bytes(const Dims& m) { return (size_t)256 * (m.d / 2) * 4; }
size_t dkdv_slot_bytes(const Dims& m) { return (size_t)4 * (m.d / 32) * 16 * 64 * 4; }
hipError_t launch_bwd_delta(const void*, const void*, const void*, const Dims&, float*, hipStream_t) { reached("launch_bwd_delta"); }
hipError_t launch_bwd_dq(const void*, const void*, const void*, const void*, const float*, const float*, const Dims&,
                         const int32_t*, const int32_t*, const int32_t*, float, void*, const SplitPlan&, hipStream_t) {
  reached("launch_bwd_dq");
}
hipError_t launch_bwd_dkdv(const void*, const void*, const void*, const void*, const float*, const float*, const Dims&,
                           const int32_t*, const int32_t*, const int32_t*, float, void*, void*, const SplitPlan&, hipStream_t) {
  reached("launch_bwd_dkdv");
}
size_t error_ws_bytes(const Dims& m) { return (size_t)m.B * m.H * 64; }
hipError_t launch_error_terms(const void*, const void*, const float*, const float*, const Dims&, double*, void*, hipStream_t) {
  reached("launch_error_terms");
}
size_t vd_ws_bytes() { return 2048 * 8; }
hipError_t launch_vd_loss(const void*, const void*, int64_t, bool, double, double*, void*, hipStream_t) { reached("launch_vd_loss"); }
hipError_t launch_vd_grad(const void*, const void*, int64_t, bool, double, const double*, void*, hipStream_t) {
  reached("launch_vd_grad");
}
}  // namespace spa2
