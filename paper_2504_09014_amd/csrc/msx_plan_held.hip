// The plan interpreter with room for the sums of a read phase (see k_plan_executor in msx_kernels_plan.hpp).
#include <hip/hip_runtime.h>

#include "msx_phased.hpp"
#include "msx_plan.hpp"

namespace msx {

const void* plan_executor_held(bool f32)
{
    return f32 ? (const void*)k_plan_executor<0, kPhasedHeld> : (const void*)k_plan_executor<1, kPhasedHeld>;
}

}  // namespace msx
