// Selectors of the phased HB kernels, and the all-gather's instantiations (see msx_kernels_phased.hpp).
#include <hip/hip_runtime.h>

#include "msx_kernels_phased.hpp"
#include "msx_phased.hpp"

namespace msx {

PhasedKernel phased_reduce_kernel(bool f32, int nranks, int res, int kind)
{
    if (kind == 1) return phased_reducescatter(f32, nranks);
    if (res == 0 && nranks >= 2 && nranks <= 4) return phased_allreduce_2_to_4(f32, nranks);
    if (res == 0 && nranks >= 5 && nranks <= 7) return phased_allreduce_5_to_7(f32, nranks);
    return f32 ? phased_allreduce_f32(nranks, res) : phased_allreduce_bf16(nranks, res);
}

PhasedKernel phased_allgather_kernel(int nranks)
{
    return nranks == 8 ? (PhasedKernel)k_allgather_hb_phased<8, kPhasedHeld> : (PhasedKernel)k_allgather_hb_phased<0, kPhasedHeld>;
}

}  // namespace msx
