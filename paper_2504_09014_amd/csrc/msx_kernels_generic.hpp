// Element types and operators beyond the tuned paths: fp16, int32, and max / min next to sum (the DSL
// carries a ReduceOp; the Collective API mirrors NCCL's).  One fused all-pairs HB kernel and one
// reduce-scatter kernel, same structure as the tuned ones (every rank reads its chunk from all
// ranks, combines in rank order in fp32, puts the result everywhere with write-through stores),
// one vector per thread and pass, rank count at run time.  Sum rounds once at the end; max / min
// keep the earlier value unless the later one is strictly greater / smaller.  int32 is combined as
// integers: the sum modulo 2^32, max / min signed.
#pragma once
#include <hip/hip_fp16.h>
#include "msx_device.hpp"
#include "msx_kernels_hb.hpp"

namespace msx {

template <int OP> __device__ __forceinline__ float combine(float acc, float v)
{
    if constexpr (OP == 0) return acc + v;
    else if constexpr (OP == 1) return v > acc ? v : acc;
    else return v < acc ? v : acc;
}

template <int OP> __device__ __forceinline__ unsigned combine_i32(unsigned acc, unsigned v)
{
    if constexpr (OP == 0) return acc + v;                                  // wraps modulo 2^32
    else if constexpr (OP == 1) return (int)v > (int)acc ? v : acc;
    else return (int)v < (int)acc ? v : acc;
}

// fp16 <-> fp32 through the hardware converters (round to nearest even, subnormals kept)
__device__ __forceinline__ float f16_lo(unsigned w) { return __half2float(__ushort_as_half((unsigned short)(w & 0xffffu))); }
__device__ __forceinline__ float f16_hi(unsigned w) { return __half2float(__ushort_as_half((unsigned short)(w >> 16))); }
__device__ __forceinline__ unsigned f16_round(float f) { return (unsigned)__half_as_ushort(__float2half_rn(f)); }

// elements of one 32-bit word for dtype DT (0 fp32, 1 bf16, 2 fp16)
template <int DT> __device__ __forceinline__ void unpack_word(unsigned w, float& a, float& b)
{
    if constexpr (DT == 0) { a = __uint_as_float(w); b = 0.0f; }
    else if constexpr (DT == 1) { a = bf16_lo(w); b = bf16_hi(w); }
    else { a = f16_lo(w); b = f16_hi(w); }
}
template <int DT> __device__ __forceinline__ unsigned pack_word(float a, float b)
{
    if constexpr (DT == 0) return __float_as_uint(a);
    else if constexpr (DT == 1) return bf16_round(a) | (bf16_round(b) << 16);
    else return f16_round(a) | (f16_round(b) << 16);
}

template <int DT, int OP> struct VecAccG {
    float a[4], b[4];
    unsigned w[4];        // DT == 3 (int32): the words themselves
    __device__ __forceinline__ void set(u32x4 v)
    {
        if constexpr (DT == 3) { w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
        else {
            unpack_word<DT>(v.x, a[0], b[0]); unpack_word<DT>(v.y, a[1], b[1]);
            unpack_word<DT>(v.z, a[2], b[2]); unpack_word<DT>(v.w, a[3], b[3]);
        }
    }
    __device__ __forceinline__ void add(u32x4 v)
    {
        if constexpr (DT == 3) {
            w[0] = combine_i32<OP>(w[0], v.x); w[1] = combine_i32<OP>(w[1], v.y);
            w[2] = combine_i32<OP>(w[2], v.z); w[3] = combine_i32<OP>(w[3], v.w);
        } else {
            float x[4], y[4];
            unpack_word<DT>(v.x, x[0], y[0]); unpack_word<DT>(v.y, x[1], y[1]);
            unpack_word<DT>(v.z, x[2], y[2]); unpack_word<DT>(v.w, x[3], y[3]);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                a[k] = combine<OP>(a[k], x[k]);
                if constexpr (DT != 0) b[k] = combine<OP>(b[k], y[k]);
            }
        }
    }
    __device__ __forceinline__ u32x4 pack() const
    {
        if constexpr (DT == 3) return u32x4{w[0], w[1], w[2], w[3]};
        else return u32x4{pack_word<DT>(a[0], b[0]), pack_word<DT>(a[1], b[1]), pack_word<DT>(a[2], b[2]), pack_word<DT>(a[3], b[3])};
    }
};

// one element, as the accumulator type of the scalar paths: float, or the int32 bits in an unsigned
template <int DT> struct ElemG { typedef float type; };
template <> struct ElemG<3> { typedef unsigned type; };
template <int DT, int OP> __device__ __forceinline__ typename ElemG<DT>::type combine_elem(typename ElemG<DT>::type acc, typename ElemG<DT>::type v)
{
    if constexpr (DT == 3) return combine_i32<OP>(acc, v);
    else return combine<OP>(acc, v);
}

template <int DT> __device__ __forceinline__ typename ElemG<DT>::type load_elem_g(const void* p, size_t e)
{
    if constexpr (DT == 0) return ((const float*)p)[e];
    else if constexpr (DT == 1) return __uint_as_float((unsigned)((const unsigned short*)p)[e] << 16);
    else if constexpr (DT == 2) return __half2float(__ushort_as_half(((const unsigned short*)p)[e]));
    else return ((const unsigned*)p)[e];
}
template <int DT> __device__ __forceinline__ void store_elem_g(void* p, size_t e, typename ElemG<DT>::type v)
{
    if constexpr (DT == 0) ((float*)p)[e] = v;
    else if constexpr (DT == 1) ((unsigned short*)p)[e] = (unsigned short)bf16_round(v);
    else if constexpr (DT == 2) ((unsigned short*)p)[e] = (unsigned short)f16_round(v);
    else ((unsigned*)p)[e] = v;
}

// AllReduce (mode 0: result to every rank, a.count = elements per rank; mode 2: the same element by element,
// for pointers that are only element-aligned) or ReduceScatter (mode 1: a.count = elements per block,
// a.out[r] = rank r's block, vec as in k_reducescatter_hb).
template <int DT, int OP>
__global__ __launch_bounds__(256) void k_reduce_generic(HbArgs a, DevCtx c, int mode, int vec)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    constexpr size_t epv = (DT == 0 || DT == 3) ? 4 : 8;
    constexpr size_t esz = (DT == 0 || DT == 3) ? 4 : 2;
    if (a.barriers && n > 1 && !rank_barrier<true>(c, rank, n, chan, 600, false, false)) return;
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;
    bool plain_stores = false;
    if (mode == 0) {
        const size_t V = a.count / epv;
        const size_t lo = chunk_begin(V, rank, n), hi = chunk_begin(V, rank + 1, n);
        for (size_t idx = lo + rt; idx < hi; idx += RT) {
            u32x4 v[kMaxRanks];
            MSX_LOAD_ALL(v, a.in, idx)
            VecAccG<DT, OP> acc;
            MSX_SUM_ALL(acc, v)
            const u32x4 o = acc.pack();
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l) st16_wt(a.out[p], idx, o);
        }
        if (rank == 0 && chan == 0 && V * epv < a.count) {
            plain_stores = true;
            for (size_t e = V * epv + threadIdx.x; e < a.count; e += blockDim.x) {
                auto acc = load_elem_g<DT>(a.in[0], e);
                for (int j = 1; j < n; ++j) acc = combine_elem<DT, OP>(acc, load_elem_g<DT>(a.in[j], e));
                for (int p = 0; p < n; ++p) store_elem_g<DT>(a.out[p], e, acc);
            }
        }
    } else if (mode == 2) {
        // AllReduce element by element, for rows that do not start on 16-byte boundaries: rank r combines its
        // share of the elements and stores them to every rank (in place is safe: an element is read and
        // written by one thread only).  Ordinary stores, so the end barrier releases.
        plain_stores = true;
        const size_t lo = a.count * (size_t)rank / (size_t)n, hi = a.count * (size_t)(rank + 1) / (size_t)n;
        for (size_t e = lo + rt; e < hi; e += RT) {
            auto acc = load_elem_g<DT>(a.in[0], e);
            for (int j = 1; j < n; ++j) acc = combine_elem<DT, OP>(acc, load_elem_g<DT>(a.in[j], e));
            for (int p = 0; p < n; ++p) store_elem_g<DT>(a.out[p], e, acc);
        }
    } else {
        const size_t blk = a.count;
        if (vec) {
            const size_t cv = blk / epv;
            const void* src[kMaxRanks];
#pragma unroll
            for (int j = 0; j < kMaxRanks; ++j) src[j] = j < n ? (const char*)a.in[j] + (size_t)rank * blk * esz : nullptr;
            for (size_t idx = rt; idx < cv; idx += RT) {
                u32x4 v[kMaxRanks];
                MSX_LOAD_ALL(v, src, idx)
                VecAccG<DT, OP> acc;
                MSX_SUM_ALL(acc, v)
                st16(a.out[rank], idx, acc.pack());
            }
        } else {
            for (size_t k = rt; k < blk; k += RT) {
                const size_t e = (size_t)rank * blk + k;
                auto acc = load_elem_g<DT>(a.in[0], e);
                for (int j = 1; j < n; ++j) acc = combine_elem<DT, OP>(acc, load_elem_g<DT>(a.in[j], e));
                store_elem_g<DT>(a.out[rank], k, acc);
            }
        }
    }
    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 601, plain_stores, false);
}

}  // namespace msx
