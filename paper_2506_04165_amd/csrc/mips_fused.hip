// Matmul-fused stage 1 (Section 7.3): instantiations with short lists (K' <= 2) and the
// dispatcher.  This file is compiled with matrix results kept in ordinary VGPRs (see the build
// script): with short lists there are registers to spare and the move per score it saves shows.
#include "mips_fused_kernel.h"

namespace atk {

hipError_t launch_mips_stage1_long(const MipsParams& p, int KP, hipStream_t stream);   // mips_fused_long.hip

hipError_t launch_mips_stage1(const MipsParams& p, int KP, hipStream_t stream) {
    switch (KP) {
        case 1: return launch_for<1>(p, stream);
        case 2: return launch_for<2>(p, stream);
        case 3: case 4: return launch_mips_stage1_long(p, KP, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace atk
