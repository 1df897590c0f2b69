// Selector of the plan interpreter's instantiation with held sums (defined in msx_plan_held.hip, a translation
// unit of its own: that instantiation is as long as the phased kernels; used by the host code in msx_host.hip).
#pragma once
#include "msx_kernels_plan.hpp"

namespace msx {

const void* plan_executor_held(bool f32);

}  // namespace msx
