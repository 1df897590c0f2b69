// What the HB-protocol kernels share: their argument block, element access for the scalar tails, and the
// per-rank load / sum loops.
#pragma once
#include "msx_device.hpp"

namespace msx {

struct HbArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    const void* res[kMaxRanks];
    size_t count;       // elements per rank (allreduce) / per block (others)
    int n;              // ranks
    int chans;          // workgroups per rank
    int has_res;        // add a residual
    int res_shared;     // all residual pointers are the same buffer
    int barriers;       // run the start / end rank barriers
    int peer_outer;     // two-phase all-gather: one hb_put per peer instead of peer-inner
    int pace;           // phased kernels: hold the write phase to a common schedule
};

template <int DT> __device__ __forceinline__ float load_elem(const void* p, size_t e)
{
    if constexpr (DT == 0) return ((const float*)p)[e];
    else return __uint_as_float((unsigned)((const unsigned short*)p)[e] << 16);
}
template <int DT> __device__ __forceinline__ void store_elem(void* p, size_t e, float v)
{
    if constexpr (DT == 0) ((float*)p)[e] = v;
    else ((unsigned short*)p)[e] = (unsigned short)bf16_round(v);
}

// Elements past the last whole 16-byte vector: summed and written to every rank by the
// first threads of rank 0, channel 0 (ordinary stores: that workgroup releases for real).
template <int DT>
__device__ __forceinline__ void allreduce_tail(const HbArgs& a, int n_l, size_t first, size_t count)
{
    for (size_t e = first + threadIdx.x; e < count; e += blockDim.x) {
        float acc = load_elem<DT>(a.in[0], e);
#pragma unroll
        for (int j = 1; j < kMaxRanks; ++j)
            if (j < n_l) acc += load_elem<DT>(a.in[j], e);
        float r[kMaxRanks];
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            r[p] = (p < n_l && a.has_res) ? load_elem<DT>(a.res[a.res_shared ? 0 : p], e) : 0.0f;
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l) store_elem<DT>(a.out[p], e, a.has_res ? acc + r[p] : acc);
    }
}

#define MSX_LOAD_ALL(v, ptrs, idx)                                   \
    _Pragma("unroll") for (int j = 0; j < kMaxRanks; ++j)            \
        if (j < n_l) v[j] = ld16(ptrs[j], idx);

#define MSX_SUM_ALL(acc, v)                                          \
    acc.set(v[0]);                                                   \
    _Pragma("unroll") for (int j = 1; j < kMaxRanks; ++j)            \
        if (j < n_l) acc.add(v[j]);

}  // namespace msx
