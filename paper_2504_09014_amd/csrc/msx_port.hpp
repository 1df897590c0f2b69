// PortChannel, emulated inside one GPU (Primitive API section, "PortChannel", and its request
// queue figure): port-mapped I/O, where the GPU does not move the bytes itself but asks a port to.
// A GPU thread pushes put / signal / flush requests into a FIFO in host memory; a CPU proxy thread
// of the library pops them and drives the copy path of the runtime (hipMemcpyAsync, device to
// device) on a stream of its own.  A signal is a one-wave kernel enqueued behind the copies on that
// stream, so it is strictly ordered after the puts before it without the CPU waiting for anything,
// and it lands in the receiver's ordinary device-side semaphores: the receiving rank waits exactly as
// on a MemoryChannel.  A flush returns once the copies pushed before it have completed (the proxy
// records an event behind them and reports when it has fired).  As in the paper the FIFO and its tail
// live in memory both sides can reach and the head is written by the GPU only.  There is no second
// device here, so source and destination are buffers of two emulated ranks in the same HBM.  One FIFO
// per sending rank (a single producer each: the first thread of the rank's first workgroup), one
// proxy thread serving all of them.
#pragma once
#include "msx_device.hpp"
#include "msx_kernels_hb.hpp"

namespace msx {

constexpr unsigned kPortSlots = 64;
enum PortType : unsigned { kPortPut = 1, kPortSignal = 2, kPortFlush = 3 };

struct PortReq {
    unsigned long long src, dst, bytes;
    unsigned type;
    unsigned arg;       // signal: receiver | sender << 8 | semaphores (channels 0 .. k-1) << 16
};

struct PortFifo {
    PortReq req[kPortSlots];
    unsigned long long head;            // requests pushed so far                       (written by the GPU)
    unsigned long long tail;            // requests taken out of the queue              (written by the proxy)
    unsigned long long flushed;         // sequence number of the last flush that is complete (proxy)
    unsigned long long pad[5];
};

// In pinned, device-mapped host memory.
struct PortShared {
    PortFifo fifo[kMaxRanks];
};

__device__ __forceinline__ unsigned port_signal_arg(int recv, int send, int nsem)
{
    return (unsigned)recv | ((unsigned)send << 8) | ((unsigned)nsem << 16);
}

// One thread pushes one request; returns its sequence number (1-based), or 0 when the FIFO
// stayed full for the whole spin budget.
__device__ __forceinline__ unsigned long long port_push(const DevCtx& c, PortFifo* f, unsigned type,
                                                        const void* src, void* dst, size_t bytes, unsigned arg)
{
    const unsigned long long seq = __hip_atomic_load(&f->head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    bool room = false;
    for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
        const unsigned long long done = __hip_atomic_load(&f->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (seq - done < kPortSlots) { room = true; break; }
        __builtin_amdgcn_s_sleep(8);
    }
    if (!room) { report(c, kStatusTimeout, 0u, 500u, (unsigned)seq, 0u); return 0; }
    PortReq* r = &f->req[seq % kPortSlots];
    __hip_atomic_store(&r->src, (unsigned long long)src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&r->dst, (unsigned long long)dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&r->bytes, (unsigned long long)bytes, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&r->type, type, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(&r->arg, arg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    // the request (and whatever this thread wrote before, e.g. the source data) first, then the head
    __hip_atomic_store(&f->head, seq + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    return seq + 1;
}

__device__ __forceinline__ void port_put(const DevCtx& c, PortFifo* f, void* dst, const void* src, size_t bytes)
{
    port_push(c, f, kPortPut, src, dst, bytes, 0);
}
// signal(): the receiver's semaphores of channels 0 .. nsem-1 for this sender go up by one, after every put
// pushed before it has landed
__device__ __forceinline__ void port_signal(const DevCtx& c, PortFifo* f, int me, int peer, int nsem)
{
    port_push(c, f, kPortSignal, nullptr, nullptr, 0, port_signal_arg(peer, me, nsem));
}
// flush(): returns when every put pushed so far has been carried out (the source may be reused)
__device__ __forceinline__ bool port_flush(const DevCtx& c, PortFifo* f, unsigned rank)
{
    const unsigned long long seq = port_push(c, f, kPortFlush, nullptr, nullptr, 0, 0);
    if (seq == 0) return false;
    for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
        if (__hip_atomic_load(&f->flushed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= seq) return true;
        __builtin_amdgcn_s_sleep(8);
    }
    report(c, kStatusTimeout, rank, 501u, (unsigned)seq, 0u);
    return false;
}

// The kernel the proxy enqueues for a signal request: one semaphore per thread (one wave up to 64 channels).
__global__ __launch_bounds__(256) void k_port_signal(unsigned* sem, int recv, int send, int nsem)
{
    if ((int)threadIdx.x < nsem)
        __hip_atomic_fetch_add(sem + (size_t)sem_index(recv, send, (int)threadIdx.x) * kSemStrideWords, 1u,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Hand-off through the port: rank 0 (workgroup 0) asks the port to copy src -> staging, to signal
// rank 1 and to flush; rank 1 (workgroups 1 .. readers, its channels) waits for the signal, then copies
// staging -> dst with its own threads.
__global__ __launch_bounds__(256) void k_port_put_signal_wait(DevCtx c, PortShared* ps, const void* src, void* staging,
                                                               void* dst, size_t nbytes, int readers)
{
    if (blockIdx.x == 0) {
        if (c.drop_rank == 0) return;
        if (threadIdx.x == 0) {
            port_put(c, &ps->fifo[0], staging, src, nbytes);
            port_signal(c, &ps->fifo[0], 0, 1, readers);
            port_flush(c, &ps->fifo[0], 0u);
        }
        return;
    }
    if (c.drop_rank == 1) return;
    const int chan = (int)blockIdx.x - 1;
    if (!channel_wait(c, 1, 0, chan, 502)) return;       // acquires: the copy's bytes are read from memory
    const size_t nvec = (nbytes + 15) / 16;
    const size_t lo = (nvec * (size_t)chan / (size_t)readers) * 16;
    size_t hi = (nvec * (size_t)(chan + 1) / (size_t)readers) * 16;
    if (hi > nbytes) hi = nbytes;
    if (hi > lo) hb_put((char*)dst + lo, (const char*)staging + lo, hi - lo, threadIdx.x, blockDim.x);
}

// ---- two-phase ring over the PortChannel, copies overlapped with the reduction ----------------------
// Collectives Library section (2PR: the ring may run over the PortChannel inside a node too, its copies
// overlapped with the reduction) and the overlapped ring reduce-scatter example of the DSL section.
// Every chunk is split in two halves.  In a reduce-scatter step a rank asks the port to put the first
// half of the chunk it passes on, reduces - with its threads, meanwhile - the second half of that chunk
// (which arrived at the end of the step before), waits for the first half of the next chunk, asks for the
// second half to be put, reduces the first half that has just arrived, waits for the second, flushes.
// The all-gather phase forwards each half as soon as it is there.  Chunk k is summed in the order k, k+1,
// ..., k-1 (mod n) and the partial sum travels in the element type, exactly as in k_allreduce_ring: the
// halves change WHEN an element is added, not in which order or with which rounding, so the results are
// those of the plain ring bit for bit.
// Partial sums are staged in the rank's own output (written through, so that the copy that reads them
// next finds them in memory); `scratch` receives the partials of the previous rank.  The rank's first
// workgroup talks to the port (its first thread pushes); all workgroups reduce, each its share of a half, and
// count the halves they are done with on the semaphores of the diagonal (rank, rank, channel), which is how
// the first workgroup knows that a half is complete before it asks for it to be put.
template <int DT>
__global__ __launch_bounds__(256) void k_allreduce_ring_port(RingArgs a, PortShared* ps, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    const int next = rank + 1 == n ? 0 : rank + 1;
    const int prev = rank == 0 ? n - 1 : rank - 1;
    const size_t cv = a.chunk_vecs, mid = cv / 2;
    const bool op = chan == 0;                       // this workgroup talks to the port
    PortFifo* const fifo = &ps->fifo[rank];
    // my "this half is reduced" counter: the diagonal semaphore (rank, rank) of my channel
    unsigned* const done_sem = c.sem + (size_t)sem_index(rank, rank, chan) * kSemStrideWords;

    if (!rank_barrier<true>(c, rank, n, chan, 80, false, false)) return;   // everybody is done with the previous call's scratch

    auto half_lo = [&](int h) { return h == 0 ? (size_t)0 : mid; };
    auto half_hi = [&](int h) { return h == 0 ? mid : cv; };
    // my share of half h of chunk j: partial received from the previous rank + my own values -> my output
    auto reduce = [&](int j, int h) {
        const size_t h0 = half_lo(h), len = half_hi(h) - h0;
        const size_t lo = h0 + len * (size_t)chan / (size_t)a.chans, hi = h0 + len * (size_t)(chan + 1) / (size_t)a.chans;
        for (size_t i = lo + threadIdx.x; i < hi; i += 2 * (size_t)blockDim.x) {       // two vectors per thread in flight
            const size_t idx = (size_t)j * cv + i, idx1 = idx + blockDim.x;
            const bool two = i + blockDim.x < hi;
            const u32x4 p0 = ld16(a.scratch[rank], idx), m0 = ld16(a.in[rank], idx);
            u32x4 p1 = p0, m1 = m0;
            if (two) { p1 = ld16(a.scratch[rank], idx1); m1 = ld16(a.in[rank], idx1); }
            VecAcc<DT> a0, a1;
            a0.set(p0); a0.add(m0);
            a1.set(p1); a1.add(m1);
            u32x4 o0 = a0.pack(), o1 = a1.pack();
            settle(o0); settle(o1);
            st16_wt(a.out[rank], idx, o0);
            if (two) st16_wt(a.out[rank], idx1, o1);
        }
        put_drain();
        __syncthreads();                             // every wave's stores have landed
        if (threadIdx.x == 0) sem_signal(done_sem, false);
    };
    // the first workgroup: every workgroup of the rank is done with the half reduced last.  One counter per
    // workgroup, one waiting thread each: a sum over the workgroups would let one that is a half ahead stand
    // in for one that is behind.
    auto all_reduced = [&]() -> bool {
        __shared__ unsigned failed;
        if (threadIdx.x == 0) failed = 0u;
        __syncthreads();
        if ((int)threadIdx.x < a.chans) {
            const unsigned idx = sem_index(rank, rank, (int)threadIdx.x);
            const unsigned want = c.expected[idx] + 1u;
            c.expected[idx] = want;
            if (!sem_spin(c, c.sem + (size_t)idx * kSemStrideWords, want, (unsigned)rank, 81, false)) failed = 1u;
        }
        __syncthreads();
        return failed == 0u;
    };
    // ask the port to copy half h of chunk j and to signal the next rank (nsem of its channels)
    auto put = [&](const void* from, void* to, int j, int h, int nsem) {
        if (threadIdx.x == 0) {
            const size_t off = ((size_t)j * cv + half_lo(h)) * 16, len = (half_hi(h) - half_lo(h)) * 16;
            port_put(c, fifo, (char*)to + off, (const char*)from + off, len);
            port_signal(c, fifo, rank, next, nsem);
        }
    };

    // reduce-scatter: n-1 steps; in step s chunk rank-s goes out and chunk rank-1-s comes in
    for (int s = 0; s + 1 < n; ++s) {
        int cs = rank - s; if (cs < 0) cs += n;
        int cr = rank - 1 - s; if (cr < 0) cr += n;
        const void* from = s == 0 ? a.in[rank] : (const void*)a.out[rank];
        if (op) {
            if (s > 0 && !all_reduced()) return;     // first half of the chunk to pass on: reduced in the step before
            put(from, a.scratch[next], cs, 0, a.chans);
        }
        if (s > 0) reduce(cs, 1);                    // its second half, while the port copies the first
        if (!channel_wait(c, rank, prev, chan, 82)) return;      // the first half of the incoming chunk is here
        if (op) {
            if (s > 0 && !all_reduced()) return;
            put(from, a.scratch[next], cs, 1, a.chans);
        }
        reduce(cr, 0);                               // while the port copies the second half
        if (!channel_wait(c, rank, prev, chan, 83)) return;      // the second half is here
        if (op && threadIdx.x == 0) port_flush(c, fifo, (unsigned)rank);
    }
    const int fin = next;                            // the chunk that ends its trip here: rank+1
    if (op && !all_reduced()) return;
    reduce(fin, 1);
    if (!op) return;                                 // the all-gather only forwards: the first workgroup does it alone
    if (!all_reduced()) return;

    // all-gather: finished chunks go round, each half forwarded as soon as it is here
    put(a.out[rank], a.out[next], fin, 0, 1);
    put(a.out[rank], a.out[next], fin, 1, 1);
    for (int t = 1; t < n; ++t) {
        int j = rank + 1 - t; if (j < 0) j += n;
        if (!channel_wait(c, rank, prev, 0, 84)) return;
        if (t + 1 < n) put(a.out[rank], a.out[next], j, 0, 1);
        if (!channel_wait(c, rank, prev, 0, 85)) return;
        if (t + 1 < n) put(a.out[rank], a.out[next], j, 1, 1);
    }
    if (threadIdx.x == 0) port_flush(c, fifo, (unsigned)rank);
}

// requests one rank pushes in one call of k_allreduce_ring_port (the host tells the proxy how many to expect)
__host__ __device__ inline unsigned ring_port_requests(int n)
{
    return n < 2 ? 0u : (unsigned)(4 * (n - 1)) * 2u + (unsigned)(n - 1) + 1u;   // puts + signals, a flush per step, a last one
}

}  // namespace msx
