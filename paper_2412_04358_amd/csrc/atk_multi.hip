// The lean kernel's launches with several helpers per finisher (kLeanMulti, see atk_lean_kernel.h).
#include "atk_lean_kernel.h"

namespace atk {

hipError_t launch_lean_multi(const Plan &pl, const LeanParams &prm, hipStream_t stream) {
    if (pl.dtype == ATK_F32) return launch_lean_mode<ATK_F32, kLeanMulti>(pl, prm, stream);
    return launch_lean_mode<ATK_BF16, kLeanMulti>(pl, prm, stream);
}

}  // namespace atk
