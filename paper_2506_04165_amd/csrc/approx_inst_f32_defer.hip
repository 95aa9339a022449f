// Explicit instantiations of the fused approximate Top-K kernel: group F32_DEFER.
#include "approx_kernel.h"
#include "approx_instances.h"

namespace atk {
#define ATK_X(TAG, T, KP, V, R, P) ATK_DEFINE_LAUNCH(T, KP, V, R, P)
ATK_INSTANCES_F32_DEFER(ATK_X)
#undef ATK_X
}  // namespace atk
