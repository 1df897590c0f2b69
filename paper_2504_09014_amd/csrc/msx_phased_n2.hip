// Part of the phased HB kernels' instantiations (see msx_kernels_phased.hpp, msx_phased.hpp): the AllReduce
// for 5 to 7 ranks with the rank count as a template argument (paced, with the condition-free copy of a round).
#include <hip/hip_runtime.h>

#include "msx_kernels_phased.hpp"
#include "msx_phased.hpp"

namespace msx {

#define MSX_PN(NR) (f32 ? (PhasedKernel)k_allreduce_hb_phased<0, NR, 0, kPhasedHeld, 0> : (PhasedKernel)k_allreduce_hb_phased<1, NR, 0, kPhasedHeld, 0>)

PhasedKernel phased_allreduce_5_to_7(bool f32, int nranks)
{
    return nranks == 5 ? MSX_PN(5) : nranks == 6 ? MSX_PN(6) : nranks == 7 ? MSX_PN(7) : nullptr;
}

}  // namespace msx
