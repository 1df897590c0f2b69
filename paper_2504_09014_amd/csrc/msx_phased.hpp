// Selectors of the phased kernels (defined in msx_phased.hip, used by the host code in msx_host.hip).
#pragma once
#include "msx_hb_common.hpp"

namespace msx {

typedef void (*PhasedKernel)(HbArgs, DevCtx);

// sums (vectors) a thread holds per phase: 64 fill the register file of a CU that runs one workgroup
constexpr int kPhasedHeld = 64;

// dt: MSX_F32 or MSX_BF16; kind 0 AllReduce (res: 0 none, 1 one residual shared by all ranks), 1 ReduceScatter.
// The rank count is a template argument for 8 ranks (and, for the AllReduce without a residual, for 2 to 7)
// and a run-time value otherwise.
PhasedKernel phased_reduce_kernel(bool f32, int nranks, int res, int kind);
PhasedKernel phased_allgather_kernel(int nranks);

// the instantiations, spread over several translation units so that they compile side by side
PhasedKernel phased_allreduce_f32(int nranks, int res);
PhasedKernel phased_allreduce_bf16(int nranks, int res);
PhasedKernel phased_reducescatter(bool f32, int nranks);
PhasedKernel phased_allreduce_2_to_4(bool f32, int nranks);    // no residual; nullptr for other rank counts
PhasedKernel phased_allreduce_5_to_7(bool f32, int nranks);

}  // namespace msx
