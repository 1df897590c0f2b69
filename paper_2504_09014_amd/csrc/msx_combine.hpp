// Selector of the phased combine kernel (defined in msx_combine_dealt.hip, used by the host code in msx_host.hip).
#pragma once
#include "msx_moe_common.hpp"

namespace msx {

// sums (vectors) a thread holds per phase, as many as the phased AllReduce
constexpr int kCombineHeld = 64;

typedef void (*CombineKernel)(MoeArgs, DevCtx);
CombineKernel combine_dealt_kernel(bool f32);

}  // namespace msx
