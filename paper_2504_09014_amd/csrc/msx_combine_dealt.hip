// The phased combine's instantiations (see msx_kernels_combine.hpp), in a translation unit of their own: each is
// tens of thousands of instructions and compiles beside the rest.
#include <hip/hip_runtime.h>

#include "msx_combine.hpp"
#include "msx_kernels_combine.hpp"

namespace msx {

CombineKernel combine_dealt_kernel(bool f32)
{
    return f32 ? (CombineKernel)k_moe_combine_dealt<0, kCombineHeld> : (CombineKernel)k_moe_combine_dealt<1, kCombineHeld>;
}

}  // namespace msx
