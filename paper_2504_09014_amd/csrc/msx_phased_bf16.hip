// Part of the phased HB kernels' instantiations (see msx_kernels_phased.hpp, msx_phased.hpp).
#include <hip/hip_runtime.h>

#include "msx_kernels_phased.hpp"
#include "msx_phased.hpp"

namespace msx {

#define MSX_P(DT, RES, KIND) (nranks == 8 ? (PhasedKernel)k_allreduce_hb_phased<DT, 8, RES, kPhasedHeld, KIND> \
                                          : (PhasedKernel)k_allreduce_hb_phased<DT, 0, RES, kPhasedHeld, KIND>)

PhasedKernel phased_allreduce_bf16(int nranks, int res) { return res ? MSX_P(1, 1, 0) : MSX_P(1, 0, 0); }

}  // namespace msx
