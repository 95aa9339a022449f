// Matmul-fused stage 1 (Section 7.3): the instantiations with lists of three and four.  Compiled with the
// default register classes: at this register pressure the accumulator-register form of the
// matrix instruction measured faster.
#include "mips_fused_kernel.h"

namespace atk {

hipError_t launch_mips_stage1_long(const MipsParams& p, int KP, hipStream_t stream) {
    return KP == 3 ? launch_for<3>(p, stream) : launch_for<4>(p, stream);
}

}  // namespace atk
