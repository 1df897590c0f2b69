// Part of the phased HB kernels' instantiations (see msx_kernels_phased.hpp, msx_phased.hpp): the AllReduce
// for 2 to 4 ranks with the rank count as a template argument (paced, with the condition-free copy of a round).
#include <hip/hip_runtime.h>

#include "msx_kernels_phased.hpp"
#include "msx_phased.hpp"

namespace msx {

#define MSX_PN(NR) (f32 ? (PhasedKernel)k_allreduce_hb_phased<0, NR, 0, kPhasedHeld, 0> : (PhasedKernel)k_allreduce_hb_phased<1, NR, 0, kPhasedHeld, 0>)

PhasedKernel phased_allreduce_2_to_4(bool f32, int nranks)
{
    return nranks == 2 ? MSX_PN(2) : nranks == 3 ? MSX_PN(3) : nranks == 4 ? MSX_PN(4) : nullptr;
}

}  // namespace msx
