// Explicit instantiations of the fused approximate Top-K kernel: group BF16_LONG.
#include "approx_kernel.h"
#include "approx_instances.h"

namespace atk {
#define ATK_X(TAG, T, KP, V, R, P) ATK_DEFINE_LAUNCH(T, KP, V, R, P)
ATK_INSTANCES_BF16_LONG(ATK_X)
#undef ATK_X
}  // namespace atk
