// Explicit instantiations of the fused approximate Top-K kernel: group I32_WIDE.
#include "approx_kernel.h"
#include "approx_instances.h"

namespace atk {
#define ATK_X(TAG, T, KP, V, R, P) ATK_DEFINE_LAUNCH(T, KP, V, R, P)
ATK_INSTANCES_I32_WIDE(ATK_X)
#undef ATK_X
}  // namespace atk
