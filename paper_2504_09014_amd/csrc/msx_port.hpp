// PortChannel, emulated inside one GPU (Primitive API section, "PortChannel", and its request
// queue figure): port-mapped I/O, where the GPU does not move the bytes itself but asks a port to.
// A GPU thread pushes put / signal / flush requests into a FIFO in host memory; a CPU proxy thread
// of the library pops them and drives the copy engine path of the runtime (hipMemcpyAsync, device
// to device) on a stream of its own, bumps the receiver's semaphore once the copies before a
// signal have completed, and advances the tail on flush.  As in the paper the FIFO and its tail
// live in memory both sides can reach, the semaphore is polled by the waiting GPU thread, and
// flush returns once the tail has passed the request.  There is no second device here, so source
// and destination are buffers of two emulated ranks in the same HBM.
#pragma once
#include "msx_device.hpp"

namespace msx {

constexpr unsigned kPortSlots = 64;
enum PortType : unsigned { kPortPut = 1, kPortSignal = 2, kPortFlush = 3 };

struct PortReq {
    unsigned long long src, dst, bytes;
    unsigned type;
    unsigned arg;       // signal: semaphore index
};

// In pinned, device-mapped host memory.
struct PortFifo {
    PortReq req[kPortSlots];
    unsigned long long head;            // requests pushed so far   (written by the GPU)
    unsigned long long tail;            // requests flushed through (written by the proxy)
    unsigned sem[kMaxRanks * kMaxRanks];   // [recv][send], incremented by the proxy
};

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
__device__ __forceinline__ void port_signal(const DevCtx& c, PortFifo* f, int me, int peer)
{
    port_push(c, f, kPortSignal, nullptr, nullptr, 0, (unsigned)(peer * kMaxRanks + me));
}
// flush(): returns when everything pushed so far has been carried out (the source may be reused)
__device__ __forceinline__ bool port_flush(const DevCtx& c, PortFifo* f)
{
    const unsigned long long seq = port_push(c, f, kPortFlush, nullptr, nullptr, 0, 0);
    if (seq == 0) return false;
    for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
        if (__hip_atomic_load(&f->tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= seq) return true;
        __builtin_amdgcn_s_sleep(8);
    }
    report(c, kStatusTimeout, 0u, 501u, (unsigned)seq, 0u);
    return false;
}
// wait(): one thread polls the semaphore the proxy increments until it has reached `want`
__device__ __forceinline__ bool port_wait(const DevCtx& c, PortFifo* f, unsigned want, int me, int peer)
{
    const unsigned idx = (unsigned)(me * kMaxRanks + peer);
    unsigned seen = 0;
    bool ok = false;
    for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
        seen = __hip_atomic_load(&f->sem[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if ((int)(seen - want) >= 0) { ok = true; break; }
        __builtin_amdgcn_s_sleep(8);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
    if (!ok) report(c, kStatusTimeout, (unsigned)me, 502u, want, seen);
    return ok;
}

// Hand-off through the port: rank 0 (workgroup 0) asks the port to copy src -> staging, to signal
// rank 1 and to flush; rank 1 (workgroups 1 .. readers) waits for the signal, then copies
// staging -> dst with its own threads.  state = {expected value of the (1 <- 0) semaphore,
// readers finished, go word}: every reader takes the expected value when it starts and the last reader
// to finish advances it, so the launch can be replayed.
__global__ __launch_bounds__(256) void k_port_put_signal_wait(DevCtx c, PortFifo* f, unsigned* state,
                                                               const void* src, void* staging, void* dst,
                                                               size_t nbytes, int readers)
{
    if (blockIdx.x == 0) {
        if (c.drop_rank == 0) return;
        if (threadIdx.x == 0) {
            port_put(c, f, staging, src, nbytes);
            port_signal(c, f, 0, 1);
            port_flush(c, f);
        }
        return;
    }
    if (c.drop_rank == 1) return;
    const int chan = (int)blockIdx.x - 1;
    const unsigned want = state[0] + 1u;
    if (threadIdx.x == 0) {
        if (chan == 0) {
            // only one thread of the rank polls the semaphore in host memory; it then releases the
            // rank's other workgroups through a word in device memory
            port_wait(c, f, want, 1, 0);
            __hip_atomic_store(state + 2, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            unsigned seen = 0;
            bool ok = false;
            for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
                seen = __hip_atomic_load(state + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((int)(seen - want) >= 0) { ok = true; break; }
                __builtin_amdgcn_s_sleep(8);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (!ok) report(c, kStatusTimeout, 1u, 503u, want, seen);
        }
    }
    __syncthreads();
    const size_t nvec = (nbytes + 15) / 16;
    const size_t lo = (nvec * (size_t)chan / (size_t)readers) * 16;
    size_t hi = (nvec * (size_t)(chan + 1) / (size_t)readers) * 16;
    if (hi > nbytes) hi = nbytes;
    if (hi > lo) hb_put((char*)dst + lo, (const char*)staging + lo, hi - lo, threadIdx.x, blockDim.x);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned done = __hip_atomic_fetch_add(state + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == (unsigned)readers - 1u) {
            __hip_atomic_store(state + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(state + 0, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace msx
