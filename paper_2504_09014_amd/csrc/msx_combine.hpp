// Selector of the phased combine kernel (defined in msx_combine_dealt.hip, used by the host code in msx_host.hip).
#pragma once
#include "msx_moe_common.hpp"

namespace msx {

// sums (vectors) a thread holds per phase: beside them it keeps eight row offsets per tile, so a few less than
// the 64 of the phased AllReduce fit without spilling
constexpr int kCombineHeld = 56;

typedef void (*CombineKernel)(MoeArgs, DevCtx);
CombineKernel combine_dealt_kernel(bool f32);

}  // namespace msx
