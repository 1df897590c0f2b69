// Part of the phased HB kernels' instantiations (see msx_kernels_phased.hpp, msx_phased.hpp): the AllReduce
// for 2 and 4 ranks with the rank count as a template argument (paced, with the condition-free copy of a round).
#include <hip/hip_runtime.h>

#include "msx_kernels_phased.hpp"
#include "msx_phased.hpp"

namespace msx {

PhasedKernel phased_allreduce_2_or_4(bool f32, int nranks)
{
    if (nranks == 4) return f32 ? (PhasedKernel)k_allreduce_hb_phased<0, 4, 0, kPhasedHeld, 0> : (PhasedKernel)k_allreduce_hb_phased<1, 4, 0, kPhasedHeld, 0>;
    if (nranks == 2) return f32 ? (PhasedKernel)k_allreduce_hb_phased<0, 2, 0, kPhasedHeld, 0> : (PhasedKernel)k_allreduce_hb_phased<1, 2, 0, kPhasedHeld, 0>;
    return nullptr;
}

}  // namespace msx
