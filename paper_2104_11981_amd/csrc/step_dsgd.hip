// Instantiations of the fused step kernel (step_impl.hpp) for: ALGO_DSGD.
#define DL_STEP_KERNEL_IMPL
#include "step_impl.hpp"

namespace dl {
namespace step {

template <>
int launch_method<ALGO_DSGD>(int vec, int format, bool norms, const StepCall& s) {
    return launch_extras<ALGO_DSGD>(vec, format, norms, s);
}

}  // namespace step
}  // namespace dl
