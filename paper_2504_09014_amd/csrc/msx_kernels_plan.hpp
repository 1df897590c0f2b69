// Plan interpreter: ONE generic kernel that runs an AllReduce from an execution plan, the
// analogue of the paper's Executor (DSL section, "Executor": a single kernel interprets any
// plan, with the primitives inlined).  A plan is a list of operations per workgroup (per rank
// and channel), produced on the host by a small lowering step for a fixed size and rank count;
// buffers are named by kind and rank, so one plan serves any pointers of that shape.  The same
// algorithms exist as hand-written kernels; running both gives the interpreter's overhead.
#pragma once
#include "msx_device.hpp"

namespace msx {

enum PlanCode : int {
    kOpEnd = 0,
    kOpBarrier = 1,     // rank barrier on this channel; flags bit 0 release, bit 1 acquire
    kOpSignal = 2,      // signal `peer`; flags bit 0: release fence first
    kOpWait = 3,        // wait for `peer`; flags bit 1: acquire
    kOpReducePut = 4,   // for each vector of the range: sum the sources in list order, store to every destination
    kOpDrain = 5        // every wave waits for its outstanding stores (before a fence-less signal)
};

enum BufKind : int { kBufIn = 0, kBufOut = 1, kBufScratch = 2 };

struct PlanRef { short kind; short rank; };   // which buffer: kind of rank

struct alignas(16) PlanOp {
    int code;
    int peer;
    int flags;
    int nsrc, ndst;
    PlanRef src[kMaxRanks + 1];
    PlanRef dst[kMaxRanks];
    int dst_wt;                 // bit d: destination d is written through (visible to peers without a fence)
    unsigned long long first;   // first vector this thread block touches is first + threadIdx.x
    unsigned long long end;     // one past the last vector of the range
    unsigned long long step;    // distance between consecutive vectors of one thread
};

struct PlanArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    void* scratch[kMaxRanks];
    const PlanOp* ops;          // all workgroups' lists, back to back
    const unsigned* start;      // [grid + 1] index of each workgroup's first op, and the total
    int n;
};

// Buffer table in LDS, [kind][rank]: indexed at run time without spilling the kernel arguments to
// private memory (a launch that needs private memory costs several microseconds more).
struct PlanBufs { const void* p[3][kMaxRanks]; };

__device__ __forceinline__ const void* plan_buf(const PlanBufs& a, PlanRef r) { return a.p[r.kind][r.rank]; }

// The data-moving operation, specialised on the list lengths so that the pointer tables stay in
// registers and all loads of one vector are issued together (two vectors per thread in flight).
// NS / ND = 0 means "take the length at run time" (the general, slower form).
template <int DT, int NS, int ND>
__device__ __forceinline__ void plan_reduce_put_run(const PlanBufs& a, const PlanOp* op)
{
    constexpr int MS = NS ? NS : kMaxRanks + 1, MD = ND ? ND : kMaxRanks;
    const int ns = NS ? NS : op->nsrc, nd = ND ? ND : op->ndst;
    const void* src[MS];
    void* dst[MD];
#pragma unroll
    for (int k = 0; k < MS; ++k) src[k] = k < ns ? plan_buf(a, op->src[k]) : nullptr;
#pragma unroll
    for (int k = 0; k < MD; ++k) dst[k] = k < nd ? const_cast<void*>(plan_buf(a, op->dst[k])) : nullptr;
    const int wt = op->dst_wt;
    const unsigned long long end = op->end, step = op->step;
    for (unsigned long long i = op->first + threadIdx.x; i < end; i += 2 * step) {
        const unsigned long long i1 = i + step;
        const bool two = i1 < end;
        u32x4 v0[MS], v1[MS];
#pragma unroll
        for (int k = 0; k < MS; ++k)
            if (k < ns) {
                v0[k] = ld16(src[k], i);
                if (two) v1[k] = ld16(src[k], i1);
            }
        u32x4 o0 = v0[0], o1 = v1[0];                // a single source is a plain copy
        if (ns > 1) {
            VecAcc<DT> a0, a1;
            a0.set(v0[0]);
            if (two) a1.set(v1[0]);
#pragma unroll
            for (int k = 1; k < MS; ++k)
                if (k < ns) {
                    a0.add(v0[k]);
                    if (two) a1.add(v1[k]);
                }
            o0 = a0.pack();
            if (two) o1 = a1.pack();
        }
#pragma unroll
        for (int k = 0; k < MD; ++k)
            if (k < nd) {
                if (wt & (1 << k)) { st16_wt(dst[k], i, o0); if (two) st16_wt(dst[k], i1, o1); }
                else { st16(dst[k], i, o0); if (two) st16(dst[k], i1, o1); }
            }
    }
}

// General form for list lengths without a specialisation: no tables, one vector at a time.
template <int DT>
__device__ __forceinline__ void plan_reduce_put_any(const PlanBufs& a, const PlanOp* op)
{
    const int ns = op->nsrc, nd = op->ndst, wt = op->dst_wt;
    const unsigned long long end = op->end, step = op->step;
    for (unsigned long long i = op->first + threadIdx.x; i < end; i += step) {
        u32x4 o = ld16(plan_buf(a, op->src[0]), i);
        if (ns > 1) {
            VecAcc<DT> acc;
            acc.set(o);
            for (int k = 1; k < ns; ++k) acc.add(ld16(plan_buf(a, op->src[k]), i));
            o = acc.pack();
        }
        for (int k = 0; k < nd; ++k) {
            void* d = const_cast<void*>(plan_buf(a, op->dst[k]));
            if (wt & (1 << k)) st16_wt(d, i, o);
            else st16(d, i, o);
        }
    }
}

template <int DT>
__global__ __launch_bounds__(256) void k_plan_executor(PlanArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    // the workgroup's list is fetched into LDS in one sweep, so stepping through it costs no
    // memory round trip per operation (lists longer than the LDS copy are read in place)
    constexpr unsigned kLdsOps = 96;
    __shared__ PlanOp lds_ops[kLdsOps];
    __shared__ PlanBufs bufs;
    if (threadIdx.x < (unsigned)kMaxRanks) {
#pragma unroll
        for (int r = 0; r < kMaxRanks; ++r)
            if ((int)threadIdx.x == r) {
                bufs.p[kBufIn][r] = a.in[r];
                bufs.p[kBufOut][r] = a.out[r];
                bufs.p[kBufScratch][r] = a.scratch[r];
            }
    }
    const unsigned first_op = a.start[blockIdx.x], n_ops = a.start[blockIdx.x + 1] - first_op;
    const PlanOp* list = a.ops + first_op;
    if (n_ops <= kLdsOps) {
        const unsigned nv = n_ops * (unsigned)(sizeof(PlanOp) / 16);
        const u32x4* g = (const u32x4*)list;
        u32x4* l = (u32x4*)lds_ops;
        for (unsigned i = threadIdx.x; i < nv; i += blockDim.x) l[i] = g[i];
        list = lds_ops;
    }
    __syncthreads();
    for (const PlanOp* op = list; op->code != kOpEnd; ++op) {
        switch (op->code) {
            case kOpBarrier:
                if (!rank_barrier<true>(c, rank, n, chan, 400, (op->flags & 1) != 0, (op->flags & 2) != 0)) return;
                break;
            case kOpSignal:
                channel_signal(c, rank, op->peer, chan, 401, (op->flags & 1) != 0);
                break;
            case kOpWait:
                // a wait that runs out ends the list: what it guards must not be consumed
                if (!channel_wait(c, rank, op->peer, chan, (op->flags & 2) ? 402 : 403, (op->flags & 2) != 0)) return;
                break;
            case kOpDrain:
                put_drain();
                break;
            case kOpReducePut: {
                const int ns = op->nsrc, nd = op->ndst;
                if (ns == 8 && nd == 8) plan_reduce_put_run<DT, 8, 8>(bufs, op);
                else if (ns == 1 && nd == 1) plan_reduce_put_run<DT, 1, 1>(bufs, op);
                else if (ns == 2 && nd == 1) plan_reduce_put_run<DT, 2, 1>(bufs, op);
                else if (ns == 2 && nd == 2) plan_reduce_put_run<DT, 2, 2>(bufs, op);
                else plan_reduce_put_any<DT>(bufs, op);
                break;
            }
            default:
                break;
        }
    }
}

}  // namespace msx
