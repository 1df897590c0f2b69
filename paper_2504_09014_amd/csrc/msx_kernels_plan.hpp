// Plan interpreter: ONE generic kernel that runs an AllReduce from an execution plan, the
// analogue of the paper's Executor (DSL section, "Executor": a single kernel interprets any
// plan, with the primitives inlined).  A plan is a list of operations per workgroup (per rank
// and channel), produced on the host by a small lowering step for a fixed size and rank count;
// buffers are named by kind and rank, so one plan serves any pointers of that shape.  The same
// algorithms exist as hand-written kernels; running both gives the interpreter's overhead.
//
// Operations: the MemoryChannel primitives (signal, wait, rank barrier), the fused reduce-then-put
// of the DSL's operation-fusion paragraph over HB vectors, the LL packet operations (put packets,
// reduce packets and pass the result on, copy packets out: what 1PA and 2PA over the LL protocol
// are made of, Collectives Library section), and the three operations of a read phase / write
// phase schedule over the whole chip (sum into registers, chip-wide barrier, put what is held).
#pragma once
#include "msx_device.hpp"
#include "msx_kernels_ll.hpp"

namespace msx {

enum PlanCode : int {
    kOpEnd = 0,
    kOpBarrier = 1,       // rank barrier on this channel; flags bit 0 release, bit 1 acquire
    kOpSignal = 2,        // signal `peer`; flags bit 0: release fence first
    kOpWait = 3,          // wait for `peer`; flags bit 1: acquire
    kOpReducePut = 4,     // for each vector of the range: sum the sources in list order, store to every destination
    kOpDrain = 5,         // every wave waits for its outstanding stores (before a fence-less signal)
    // LL protocol.  Packet q of the range lives at  aux3 + slot * aux + q * 16  of a rank's scratch half.
    kOpPutPacket = 6,     // packet aux2 * p + q of src[0] goes to slot `peer` of every rank p in dst_wt (bit mask)
    kOpReducePacket = 7,  // poll packet q of every slot but `peer` (my own), sum in rank order with packet aux2 + q
                          // of src[0] (mine), store to dst[0]; ranks in dst_wt get the sum as packet q of slot
                          // `peer`, one region (all ranks' slots) further on
    kOpCopyPacket = 8,    // poll packet q of every slot j but `peer` and store it as packet aux2 * j + q of dst[0]
    // read phase / write phase schedule (interpreter instantiated with HELD > 0)
    // They come as rounds of five: reduce-hold, barrier, put-held, drain, barrier.
    kOpReduceHold = 9,    // sum vector first + t + h * step (t = thread, h < aux tiles) of all sources into held[h]
    kOpGridBarrier = 10,  // every workgroup of the launch; flags bit 0: a write phase ends here (the pace is
                          // decided), bit 1: one begins (the pace is picked up)
    kOpPutHeld = 11       // store held[h] to vector first + t + h * step of every destination, paced
};

constexpr int kPlanDrainFirst = 4;    // flag of a barrier or a signal: wait for this workgroup's stores first

enum BufKind : int { kBufIn = 0, kBufOut = 1, kBufScratch = 2 };

struct PlanRef { short kind; short rank; };   // which buffer: kind of rank

struct alignas(16) PlanOp {
    int code;
    int peer;
    int flags;
    int nsrc, ndst;
    PlanRef src[kMaxRanks + 1];
    PlanRef dst[kMaxRanks];
    int dst_wt;                 // bit d: destination d is written through (visible to peers without a fence);
                                // packet operations: the ranks packets are sent to
    unsigned aux;               // packet operations: bytes per slot; held operations: tiles
    unsigned long long first;   // first vector (packet) this workgroup touches is first + threadIdx.x
    unsigned long long end;     // one past the last vector (packet) of the range
    unsigned long long step;    // distance between consecutive vectors (packets) of one thread
    unsigned aux2, aux3;        // packet operations: chunk stride / own offset in packets; byte offset of the region
};
static_assert(sizeof(PlanOp) == 128, "eight 16-byte vectors per operation");

struct PlanArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    void* scratch[kMaxRanks];
    const PlanOp* ops;          // workgroup b's list starts at ops + b * stride
    size_t nbytes;              // bytes per rank (the packet operations pad the last packet from it)
    unsigned stride;            // operations per workgroup, padding included
    int n;
    int head;                   // bit 0: every list begins with the same rank barrier (not in the lists: it runs
                                // while the list is on its way); bits 1, 2: its release / acquire flags
    int packets;                // the plan uses the LL protocol: take a flag and a scratch half for this call
    int pace;                   // held operations: hold the write phases to the common schedule
};

// Buffer table in LDS, [kind][rank]: indexed at run time without spilling the kernel arguments to
// private memory (a launch that needs private memory costs several microseconds more).
struct PlanBufs { const void* p[3][kMaxRanks]; };

// Whatever is read from an operation record or from the buffer table comes out of LDS: a per-lane value as far
// as the compiler can tell.  It is the same in every lane, and passing it through scalar registers says so
// (base-plus-offset addressing instead of 64-bit vector arithmetic and a register pair per load in flight;
// with per-lane strides the read phase of the held operations spilled a thousand registers).
__device__ __forceinline__ unsigned uniform(unsigned x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ int uniform(int x) { return (int)__builtin_amdgcn_readfirstlane((unsigned)x); }
__device__ __forceinline__ unsigned long long uniform(unsigned long long x)
{
    return ((unsigned long long)uniform((unsigned)(x >> 32)) << 32) | uniform((unsigned)x);
}
// The buffers an operation names, resolved to pointers: row [operation in the LDS window][source 0..8, destination
// 0..7].  Filled for the whole window at once, one (operation, buffer) pair per thread, so that an operation
// finds its pointers with independent LDS reads instead of a chain of two dependent ones per buffer.
constexpr int kPlanPtrs = kMaxRanks + 1 + kMaxRanks;
struct PlanPtrs { unsigned long long p[kPlanPtrs]; };
__device__ __forceinline__ const void* plan_src(const PlanPtrs& t, int k) { return (const void*)uniform(t.p[k]); }
__device__ __forceinline__ void* plan_dst(const PlanPtrs& t, int k) { return (void*)uniform(t.p[kMaxRanks + 1 + k]); }

// The data-moving operation, specialised on the list lengths so that the pointer tables stay in
// registers and all loads of one vector are issued together, and on whether every destination is written
// through (WT; otherwise each store asks its bit of dst_wt).  No load or store sits under a per-lane condition:
// such joins make the compiler wait for all memory operations in flight (see settle()).
template <int DT, int NS, int ND, bool WT>
__device__ __forceinline__ void plan_reduce_put_run(const PlanPtrs& a, const PlanOp* op)
{
    const void* src[NS];
    void* dst[ND];
#pragma unroll
    for (int k = 0; k < NS; ++k) src[k] = plan_src(a, k);
#pragma unroll
    for (int k = 0; k < ND; ++k) dst[k] = plan_dst(a, k);
    const int wt = uniform(op->dst_wt);
    const unsigned long long end = uniform(op->end), step = uniform(op->step);
    for (unsigned long long i = uniform(op->first) + threadIdx.x; i < end; i += step) {
        u32x4 v[NS];
#pragma unroll
        for (int k = 0; k < NS; ++k) v[k] = ld16(src[k], i);
        u32x4 o = v[0];                              // a single source is a plain copy
        if constexpr (NS > 1) {
            VecAcc<DT> acc;
            acc.set(v[0]);
#pragma unroll
            for (int k = 1; k < NS; ++k) acc.add(v[k]);
            o = acc.pack();
        }
        settle(o);
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            if (WT || (wt & (1 << k))) st16_wt(dst[k], i, o);
            else st16(dst[k], i, o);
        }
    }
}

// General form for list lengths without a specialisation: no tables, one vector at a time.
template <int DT>
__device__ __forceinline__ void plan_reduce_put_any(const PlanPtrs& a, const PlanOp* op)
{
    const int ns = uniform(op->nsrc), nd = uniform(op->ndst), wt = uniform(op->dst_wt);
    const unsigned long long end = uniform(op->end), step = uniform(op->step);
    for (unsigned long long i = uniform(op->first) + threadIdx.x; i < end; i += step) {
        u32x4 o = ld16(plan_src(a, 0), i);
        if (ns > 1) {
            VecAcc<DT> acc;
            acc.set(o);
            for (int k = 1; k < ns; ++k) acc.add(ld16((const void*)uniform(a.p[k]), i));
            o = acc.pack();
        }
        for (int k = 0; k < nd; ++k) {
            void* d = (void*)uniform(a.p[kMaxRanks + 1 + k]);
            if (wt & (1 << k)) st16_wt(d, i, o);
            else st16(d, i, o);
        }
    }
}

// ---- LL packet operations -------------------------------------------------------------------------
// What a packet operation needs beyond its record: the call's flag and scratch half, who I am.
struct PlanLl {
    CallTag tag;
    int n, rank;
    size_t nbytes;
};

// NR: rank count known at compile time (8), or 0 for "take it at run time".
template <int NR>
__device__ __forceinline__ void plan_put_packet(const PlanPtrs& bufs, const PlanOp* op, const DevCtx& c, const PlanLl& l)
{
    const int n_l = NR ? NR : per_lane(l.n), to = per_lane(op->dst_wt);   // per-lane copies for conditions (see per_lane)
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)((l.nbytes + 7) / 8);
    const void* src = plan_src(bufs, 0);
    const unsigned cs = uniform(op->aux2);
    const unsigned base = uniform(op->aux3 + l.tag.rot * c.ll_rot_stride + (unsigned)op->peer * op->aux);
    const unsigned end = uniform((unsigned)op->end), step = uniform((unsigned)op->step);
    for (unsigned q = uniform((unsigned)op->first) + threadIdx.x; q < end; q += step) {
        if (cs == 0) {                      // the same packet to everybody
            u32x2 w = load_words(src, q, l.nbytes);
            settle(w);                      // one wait for the load, none between the stores
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l && ((to >> p) & 1)) ll_store(rs, (unsigned)p * c.ll_rank_stride + base + q * 16u, w.x, w.y, l.tag.flag);
        } else {                            // packet q of chunk p to rank p: all loads first, then all stores
            u32x2 w[kMaxRanks];
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l && ((to >> p) & 1) && (unsigned)p * cs + q < P) w[p] = load_words(src, (size_t)p * cs + q, l.nbytes);
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p) settle(w[p]);
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l && ((to >> p) & 1) && (unsigned)p * cs + q < P)
                    ll_store(rs, (unsigned)p * c.ll_rank_stride + base + q * 16u, w[p].x, w[p].y, l.tag.flag);
        }
    }
}

template <int DT, int NR>
__device__ __forceinline__ void plan_reduce_packet(const PlanPtrs& bufs, const PlanOp* op, const DevCtx& c, const PlanLl& l)
{
    const int rank = l.rank;
    const int n_l = NR ? NR : per_lane(l.n), rank_l = per_lane(rank), to = per_lane(op->dst_wt);
    const CallTag tag = l.tag;
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)((l.nbytes + 7) / 8);
    const void* own_buf = plan_src(bufs, 0);
    void* out = plan_dst(bufs, 0);
    const unsigned slot_stride = uniform(op->aux), own_off = uniform(op->aux2);
    const unsigned region = uniform(op->aux3 + tag.rot * c.ll_rot_stride);
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + region;
    const unsigned next = region + (unsigned)(NR ? NR : l.n) * slot_stride + (unsigned)rank * slot_stride;
    const unsigned end = uniform((unsigned)op->end), step = uniform((unsigned)op->step);
    for (unsigned q = uniform((unsigned)op->first) + threadIdx.x; q < end; q += step) {
        const unsigned k = own_off + q;
        if (k >= P) break;
        const u32x2 own = load_words(own_buf, k, l.nbytes);
        u32x4 v[kMaxRanks];
        MSX_LL_POLL_ALL(v, my_off, slot_stride, q)
        WordAcc<DT> a0, a1;
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l) {
                const unsigned w0 = j == rank_l ? own.x : v[j].x;
                const unsigned w1 = j == rank_l ? own.y : v[j].z;
                if (j == 0) { a0.set(w0); a1.set(w1); } else { a0.add(w0); a1.add(w1); }
            }
        const u32x2 o = {a0.pack(), a1.pack()};
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && ((to >> p) & 1)) ll_store(rs, (unsigned)p * c.ll_rank_stride + next + q * 16u, o.x, o.y, tag.flag);
        store_words(out, k, l.nbytes, o);
    }
}

template <int NR>
__device__ __forceinline__ void plan_copy_packet(const PlanPtrs& bufs, const PlanOp* op, const DevCtx& c, const PlanLl& l)
{
    const int rank = l.rank;
    const int n_l = NR ? NR : per_lane(l.n), rank_l = per_lane(rank);
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)((l.nbytes + 7) / 8);
    void* out = plan_dst(bufs, 0);
    const unsigned slot_stride = uniform(op->aux), cs = uniform(op->aux2);
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + uniform(op->aux3 + l.tag.rot * c.ll_rot_stride);
    const unsigned end = uniform((unsigned)op->end), step = uniform((unsigned)op->step);
    for (unsigned q = uniform((unsigned)op->first) + threadIdx.x; q < end; q += step) {
        u32x4 v[kMaxRanks];
        bool ready = false;                 // only packets that exist were sent: the last chunks may be short
        for (unsigned spins = 0; !ready && spins <= c.spin_limit; ++spins) {
            poll_fence();
            ready = true;
#pragma unroll
            for (int j = 0; j < kMaxRanks; ++j)
                if (j < n_l && j != rank_l && (unsigned)j * cs + q < P) v[j] = ll_load(rs, my_off + (unsigned)j * slot_stride + q * 16u);
#pragma unroll
            for (int j = 0; j < kMaxRanks; ++j)
                if (j < n_l && j != rank_l && (unsigned)j * cs + q < P) ready = ready && ll_ready(v[j], l.tag.flag);
        }
        if (!ready) { report(c, kStatusTimeout, (unsigned)rank, 411u, l.tag.flag, 0u); break; }
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l && j != rank_l && (unsigned)j * cs + q < P)
                store_words(out, (size_t)j * cs + q, l.nbytes, u32x2{v[j].x, v[j].z});
    }
}

// ---- the read phase / write phase operations ------------------------------------------------------
// As in k_allreduce_hb_phased: every thread sums HELD vectors of its rank's chunk into registers, all
// workgroups meet, every thread puts its sums to all ranks, paced against the wall clock.  Eight sources
// and eight destinations (the schedule exists for 8 ranks); ALL = the workgroup has all HELD tiles, so the
// copy of the code without any condition runs and two groups of loads stay in flight.
template <int DT, int HELD, bool ALL>
__device__ __forceinline__ void plan_reduce_hold(const PlanPtrs& bufs, const PlanOp* op, u32x4 (&held)[HELD ? HELD : 1])
{
    if constexpr (HELD > 0) {
        constexpr int G = 2, HG = HELD / G;
        static_assert(HELD % (2 * G) == 0, "unrolled in pairs of groups");
        const void* src[kMaxRanks];
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j) src[j] = plan_src(bufs, j);
        const unsigned mine = uniform(op->aux);
        const int nq = (int)((mine + G - 1) / G);
        const size_t i0 = (size_t)uniform(op->first) + threadIdx.x, tstep = (size_t)uniform(op->step);
        u32x4 va[G][kMaxRanks], vb[G][kMaxRanks];
        auto issue = [&](int g, u32x4 (&v)[G][kMaxRanks]) {
#pragma unroll
            for (int i = 0; i < G; ++i)
                if (ALL || (unsigned)(g * G + i) < mine) {
#pragma unroll
                    for (int j = 0; j < kMaxRanks; ++j) v[i][j] = ld16(src[j], i0 + (size_t)(g * G + i) * tstep);
                }
        };
        auto reduce = [&](int g, u32x4 (&v)[G][kMaxRanks]) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                VecAcc<DT> acc;
                acc.set(v[i][0]);
#pragma unroll
                for (int j = 1; j < kMaxRanks; ++j) acc.add(v[i][j]);
                held[g * G + i] = acc.pack();
            }
        };
        if (ALL || 0 < nq) issue(0, va);
        static_for<HG / 2>([&](auto k) {
            constexpr int g = 2 * decltype(k)::value;
            if (ALL || g + 1 < nq) issue(g + 1, vb);
            if (ALL || g < nq) reduce(g, va);
            if (g + 2 < HG && (ALL || g + 2 < nq)) issue(g + 2, va);
            if (ALL || g + 1 < nq) reduce(g + 1, vb);
        });
    }
}

template <int HELD, bool ALL>
__device__ __forceinline__ void plan_put_held(const PlanPtrs& bufs, const PlanOp* op, const u32x4 (&held)[HELD ? HELD : 1],
                                              unsigned long long w0, unsigned pace)
{
    if constexpr (HELD > 0) {
        void* dst[kMaxRanks];
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j) dst[j] = plan_dst(bufs, j);
        const unsigned mine = uniform(op->aux);
        const size_t i0 = (size_t)uniform(op->first) + threadIdx.x, tstep = (size_t)uniform(op->step);
        static_for<HELD>([&](auto k) {
            constexpr int h = decltype(k)::value;
            if (ALL || (unsigned)h < mine) {
                wait_until(w0 + (unsigned long long)((unsigned)h * pace));
#pragma unroll
                for (int p = 0; p < kMaxRanks; ++p) st16_wt(dst[p], i0 + (size_t)h * tstep, held[h]);
            }
        });
    }
}

// HELD: sums a thread can hold between a kOpReduceHold and a kOpPutHeld (0: the plan has no such operations;
// 64 fills the register file, one workgroup per CU).  The instantiation with held sums runs the operations of
// the read phase / write phase schedule only (barriers, drain, the held pair, a plain reduce-put for ragged
// ends): whatever else sat in its loop would compete with the sums for registers.
// FAM picks the operation families an instantiation carries, by what a plan contains (the host looks): 0 the
// channel operations (barrier, signal, wait, drain, reduce-put), 1 the packet operations, 2 both (no lowering
// here mixes them, so 2 is not instantiated and the host refuses such a plan).  NR: the rank count the packet
// operations are compiled for (8, or 0 = any, read from the arguments), again so that a call carries one copy.  The code of
// the families a plan does not use is still in the way of the ones it does: a small message spends its time
// fetching instructions, and the two-family kernel took 0.4 us longer per call than the one-family kernels.
template <int DT, int HELD, int FAM = 0, int NR = 0>
__global__ __launch_bounds__(256) void k_plan_executor(PlanArgs a, DevCtx c)
{
    constexpr bool kChan = HELD == 0 && FAM != 1, kPkt = HELD == 0 && FAM != 0;
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    // The workgroup's list is fetched into LDS in one sweep, so stepping through it costs no memory round
    // trip per operation.  Its first 32 operations (one vector per thread) are requested first thing and
    // land while the prologue - call state, the barrier every list begins with - waits on its own round trips.
    constexpr unsigned kLdsOps = 64, kVecsPerOp = (unsigned)(sizeof(PlanOp) / 16);
    __shared__ PlanOp lds_ops[kLdsOps];
    __shared__ PlanPtrs lds_ptrs[kLdsOps];
    __shared__ PlanBufs bufs;
    const unsigned n_ops = a.stride < kLdsOps ? a.stride : kLdsOps;     // longer lists come in windows of kLdsOps
    const u32x4* g = (const u32x4*)(a.ops + (size_t)blockIdx.x * a.stride);
    // (no branch around the load - surplus threads fetch the last vector again - so that everything the
    // kernel asks of its arguments up to here is requested, and waited for, together)
    const unsigned early_vecs = n_ops * kVecsPerOp;
    const u32x4 early = g[threadIdx.x < early_vecs ? threadIdx.x : early_vecs - 1u];
    // Lane t of the first 24 keeps pointer t of the three tables, fetched with one vector load straight from
    // the kernel-argument segment (the explicit arguments start at its offset 0, and the tables are the first
    // members of the first argument).  Through scalar registers the 24 pointers were fetched, and waited for,
    // in several goes in front of the first barrier: 0.6 us.
    static_assert(offsetof(PlanArgs, in) == 0 && offsetof(PlanArgs, out) == sizeof(void*) * kMaxRanks &&
                  offsetof(PlanArgs, scratch) == 2 * sizeof(void*) * kMaxRanks, "table layout");
    const void* mine = nullptr;
    if (threadIdx.x < 3u * (unsigned)kMaxRanks)
        mine = ((const void* const MSX_GLOBAL*)__builtin_amdgcn_kernarg_segment_ptr())[threadIdx.x];
    PlanLl ll{CallTag{0u, 0u, 0u, 0u}, n, rank, a.nbytes};
    if constexpr (kPkt)
        if (a.packets) ll.tag = call_begin(c);
    if (rank == c.drop_rank) {
        if constexpr (kPkt)
            if (a.packets) call_end(c, ll.tag);
        return;
    }
    [[maybe_unused]] GridBar gb{0u, 0u, true};
    [[maybe_unused]] PaceCtl ctl{0u, 0u, 0u, 0u};
    [[maybe_unused]] unsigned pace = 0u, gen = 0u, key = 0u;
    [[maybe_unused]] bool wrote = false;
    if constexpr (HELD > 0) {
        gb = grid_barrier_begin(c);
        key = ((unsigned)a.nbytes ^ (unsigned)(a.nbytes >> 32)) * 2654435761u + gridDim.x * 64u + (unsigned)(DT * 8) + 48u + 1u;
        ctl = pace_load(c, key);
        pace = a.pace ? ctl.pace : 0u;
    }
    bool alive = true;
    if constexpr (kChan || HELD > 0)
        if (a.head & 1) alive = rank_barrier<true>(c, rank, n, chan, 400, (a.head & 2) != 0, (a.head & 4) != 0);
    // every buffer the `count` operations in the window name, looked up once (workgroup-collective)
    auto resolve = [&](unsigned count) {
        __syncthreads();
        for (unsigned t = threadIdx.x; t < count * (unsigned)kPlanPtrs; t += 256u) {
            const unsigned o = t / (unsigned)kPlanPtrs, k = t % (unsigned)kPlanPtrs;
            const PlanRef r = k <= (unsigned)kMaxRanks ? lds_ops[o].src[k] : lds_ops[o].dst[k - kMaxRanks - 1];
            const unsigned kind = (unsigned)r.kind < 3u ? (unsigned)r.kind : 0u;
            lds_ptrs[o].p[k] = (unsigned long long)bufs.p[kind][(unsigned)r.rank & (unsigned)(kMaxRanks - 1)];
        }
        __syncthreads();
    };
    {
        if (threadIdx.x < 3u * (unsigned)kMaxRanks) (&bufs.p[0][0])[threadIdx.x] = mine;
        u32x4* l = (u32x4*)lds_ops;
        if (threadIdx.x < n_ops * kVecsPerOp) l[threadIdx.x] = early;
        for (unsigned i = threadIdx.x + 256u; i < n_ops * kVecsPerOp; i += 256u) l[i] = g[i];
    }
    resolve(n_ops);
    // operation pc of my list, out of the window in LDS (a long list comes in windows of kLdsOps; workgroup-collective)
    auto at = [&](unsigned pc) -> const PlanOp* {
        if (pc != 0 && pc % kLdsOps == 0) {
            __syncthreads();
            const unsigned left = a.stride - pc, nv = (left < kLdsOps ? left : kLdsOps) * kVecsPerOp;
            for (unsigned i = threadIdx.x; i < nv; i += 256u) ((u32x4*)lds_ops)[i] = g[(size_t)pc * kVecsPerOp + i];
            resolve(nv / kVecsPerOp);
        }
        return &lds_ops[pc % kLdsOps];
    };
    for (unsigned pc = 0; alive && pc < a.stride; ++pc) {
        const PlanOp* op = at(pc);
        const int code = uniform(op->code);
        if (code == kOpEnd) break;
        switch (code) {
            case kOpBarrier:
                if (op->flags & kPlanDrainFirst) put_drain();
                if constexpr (kChan || HELD > 0)
                    alive = rank_barrier<true>(c, rank, n, chan, 400, (op->flags & 1) != 0, (op->flags & 2) != 0);
                break;
            case kOpSignal:
                if (op->flags & kPlanDrainFirst) put_drain();
                if constexpr (kChan) channel_signal(c, rank, op->peer, chan, 401, (op->flags & 1) != 0);
                break;
            case kOpWait:
                // a wait that runs out ends the list: what it guards must not be consumed
                if constexpr (kChan)
                    alive = channel_wait(c, rank, op->peer, chan, (op->flags & 2) ? 402 : 403, (op->flags & 2) != 0);
                break;
            case kOpDrain:
                put_drain();
                break;
            case kOpReducePut: {
                const int ns = op->nsrc, nd = op->ndst, wt = op->dst_wt;
                if constexpr (HELD > 0) {
                    plan_reduce_put_any<DT>(lds_ptrs[pc % kLdsOps], op);    // a chunk's ragged end only: less than one vector per thread
                } else if constexpr (kChan) {
                    if (ns == 8 && nd == 8 && wt == 0xff) plan_reduce_put_run<DT, 8, 8, true>(lds_ptrs[pc % kLdsOps], op);
                    else if (ns == 1 && nd == 1 && wt == 1) plan_reduce_put_run<DT, 1, 1, true>(lds_ptrs[pc % kLdsOps], op);
                    else if (ns == 2 && nd == 1 && wt == 1) plan_reduce_put_run<DT, 2, 1, true>(lds_ptrs[pc % kLdsOps], op);
                    else if (ns == 2 && nd == 2) plan_reduce_put_run<DT, 2, 2, false>(lds_ptrs[pc % kLdsOps], op);
                    else plan_reduce_put_any<DT>(lds_ptrs[pc % kLdsOps], op);
                }
                break;
            }
            case kOpPutPacket:
                if constexpr (kPkt) {
                    plan_put_packet<NR>(lds_ptrs[pc % kLdsOps], op, c, ll);
                }
                break;
            case kOpReducePacket:
                if constexpr (kPkt) {
                    plan_reduce_packet<DT, NR>(lds_ptrs[pc % kLdsOps], op, c, ll);
                }
                break;
            case kOpCopyPacket:
                if constexpr (kPkt) {
                    plan_copy_packet<NR>(lds_ptrs[pc % kLdsOps], op, c, ll);
                }
                break;
            case kOpReduceHold:
                // One round of the schedule: this operation and the four behind it (chip-wide barrier, put what
                // is held, drain, chip-wide barrier) run as one straight piece of code, so that the sums are
                // live inside this block only and not around the interpreter's loop (where the register
                // allocator moved them through private memory at every join).
                if constexpr (HELD > 0) {
                    if (pc + 4 >= a.stride) { alive = false; break; }
                    const unsigned tiles = uniform(op->aux);
                    // all = every one of the HELD tiles exists.  The whole round is instantiated once per case:
                    // where the two cases joined with the sums live (say, in front of a common barrier), the
                    // register allocator spilled hundreds of registers.
                    auto round = [&](auto all) {
                        constexpr bool ALL = decltype(all)::value;
                        u32x4 held[HELD];
                        plan_reduce_hold<DT, HELD, ALL>(lds_ptrs[pc % kLdsOps], op, held);
                        // the sums are final here: said explicitly, or the scheduler moves their last steps past
                        // the barrier's loop
                        static_for<HELD>([&](auto k) { settle(held[decltype(k)::value]); });
                        op = at(++pc);
                        bool ok = op->code == kOpGridBarrier;
                        grid_barrier(c, gb, ++gen, (unsigned)rank, 413);
                        if (a.pace && wrote)                // workgroup 0's decision after the previous write phase
                            pace = pace_clamp(__hip_atomic_load(c.gbar + kGridBarPaceWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                        op = at(++pc);
                        ok = ok && op->code == kOpPutHeld && op->aux == tiles;
                        const unsigned long long w0 = wall_clock64();
                        wrote = true;
                        if (ok) plan_put_held<HELD, ALL>(lds_ptrs[pc % kLdsOps], op, held, w0, pace);
                        op = at(++pc);
                        ok = ok && op->code == kOpDrain;
                        put_drain();
                        op = at(++pc);
                        ok = ok && op->code == kOpGridBarrier;
                        grid_barrier(c, gb, ++gen, (unsigned)rank, 414);
                        if (a.pace && blockIdx.x == 0) {
                            if (tiles >= (unsigned)HELD / 4) pace_update(ctl, wall_clock64() - w0, tiles);
                            if (threadIdx.x == 0) st32_wt(c.gbar + kGridBarPaceWord, ctl.pace);
                        }
                        if (!ok) {                          // not the sequence the lowering emits: refuse to go on
                            report(c, kStatusTimeout, (unsigned)rank, 415u, pc, (unsigned)op->code);
                            alive = false;
                        }
                    };
                    if (tiles == (unsigned)HELD) round(std::true_type{});
                    else round(std::false_type{});
                }
                break;
            default:
                break;
        }
    }
    if constexpr (HELD > 0) {
        if (a.pace && blockIdx.x == 0 && threadIdx.x == 0) pace_save(c, ctl, key);
        grid_barrier_end(c, gb, gen);
    }
    if constexpr (kPkt)
        if (a.packets) call_end(c, ll.tag);
}

}  // namespace msx
