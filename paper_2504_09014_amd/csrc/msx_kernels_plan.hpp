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

struct PlanOp {
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
    const unsigned* start;      // [grid] index of each workgroup's first op
    int n;
};

__device__ __forceinline__ const void* plan_buf(const PlanArgs& a, PlanRef r)
{
    return r.kind == kBufIn ? a.in[r.rank] : r.kind == kBufOut ? (const void*)a.out[r.rank] : (const void*)a.scratch[r.rank];
}

template <int DT>
__global__ __launch_bounds__(256) void k_plan_executor(PlanArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    for (const PlanOp* op = a.ops + a.start[blockIdx.x]; op->code != kOpEnd; ++op) {
        switch (op->code) {
            case kOpBarrier:
                rank_barrier(c, rank, n, chan, 400, (op->flags & 1) != 0, (op->flags & 2) != 0);
                break;
            case kOpSignal:
                channel_signal(c, rank, op->peer, chan, 401, (op->flags & 1) != 0);
                break;
            case kOpWait:
                if (op->flags & 2) channel_wait(c, rank, op->peer, chan, 402);
                else {
                    if (threadIdx.x == 0) {
                        const unsigned idx = sem_index(rank, op->peer, chan);
                        const unsigned want = c.expected[idx] + 1u;
                        c.expected[idx] = want;
                        sem_spin(c, c.sem + (size_t)idx * kSemStrideWords, want, (unsigned)rank, 403, false);
                    }
                    __syncthreads();
                }
                break;
            case kOpDrain:
                put_drain();
                break;
            case kOpReducePut: {
                const void* src[kMaxRanks + 1];
                void* dst[kMaxRanks];
                const int ns = op->nsrc, nd = op->ndst;
                for (int k = 0; k < ns; ++k) src[k] = plan_buf(a, op->src[k]);
                for (int k = 0; k < nd; ++k) dst[k] = const_cast<void*>(plan_buf(a, op->dst[k]));
                for (unsigned long long i = op->first + threadIdx.x; i < op->end; i += op->step) {
                    u32x4 o = ld16(src[0], i);          // a single source is a plain copy
                    if (ns > 1) {
                        VecAcc<DT> acc;
                        acc.set(o);
                        for (int k = 1; k < ns; ++k) acc.add(ld16(src[k], i));
                        o = acc.pack();
                    }
                    for (int k = 0; k < nd; ++k) {
                        if (op->dst_wt & (1 << k)) st16_wt(dst[k], i, o);
                        else st16(dst[k], i, o);
                    }
                }
                break;
            }
            default:
                break;
        }
    }
}

}  // namespace msx
