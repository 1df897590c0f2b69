// One-primitive kernels: each exercises a single MemoryChannel primitive pair between two
// emulated ranks, for the tests and for the hop-latency figures (the analogue of the
// paper's primitive-versus-best-achievable table).
#pragma once
#include "msx_device.hpp"

namespace msx {

// signal / wait ping-pong between two workgroups of a wider launch; the other workgroups
// leave at once.  block_a plays rank 0, block_b rank 1, on channel 0.
__global__ __launch_bounds__(64) void k_pingpong(DevCtx c, int iters, int block_a, int block_b,
                                                 double ns_per_tick, double* ns_out)
{
    const int b = (int)blockIdx.x;
    if (b != block_a && b != block_b) return;
    const int me = b == block_a ? 0 : 1;
    const int peer = 1 - me;
    long long t0 = 0;
    if (me == 0) {
        t0 = wall_clock64();
        for (int i = 0; i < iters; ++i) {
            channel_signal(c, me, peer, 0, 300);
            channel_wait(c, me, peer, 0, 301);
        }
        if (threadIdx.x == 0) *ns_out = (double)(wall_clock64() - t0) * ns_per_tick / (double)(iters > 0 ? iters : 1);
    } else {
        for (int i = 0; i < iters; ++i) {
            channel_wait(c, me, peer, 0, 302);
            channel_signal(c, me, peer, 0, 303);
        }
    }
}

// `rounds` rank barriers on every channel; fences bit 0 = release, bit 1 = acquire
__global__ __launch_bounds__(256) void k_barrier_rounds(DevCtx c, int n, int rounds, int fences)
{
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    for (int r = 0; r < rounds; ++r) rank_barrier(c, rank, n, chan, 310, (fences & 1) != 0, (fences & 2) != 0);
}

// channel-0 semaphore values, [n recv][n send]
__global__ void k_sem_snapshot(DevCtx c, int n, unsigned* out)
{
    const int i = (int)threadIdx.x;
    if (i < n * n) {
        const int recv = i / n, send = i % n;
        out[i] = __hip_atomic_load(c.sem + (size_t)sem_index(recv, send, 0) * kSemStrideWords,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// HB hand-off: rank 0 put + signal, rank 1 wait + read.  Each channel moves its own
// contiguous share, so the per-channel semaphore covers exactly the data its reader needs.
__global__ __launch_bounds__(256) void k_put_signal_wait(DevCtx c, const void* src, void* staging, void* dst,
                                                          size_t nbytes, int chans)
{
    const int rank = (int)(blockIdx.x & 1u);
    const int chan = (int)(blockIdx.x >> 1);
    if (rank == c.drop_rank) return;
    const size_t nvec = (nbytes + 15) / 16;                       // share boundaries in 16-byte steps
    const size_t lo = (nvec * (size_t)chan / (size_t)chans) * 16;
    size_t hi = (nvec * (size_t)(chan + 1) / (size_t)chans) * 16;
    if (hi > nbytes) hi = nbytes;
    const size_t len = hi > lo ? hi - lo : 0;
    if (rank == 0) {
        hb_put((char*)staging + lo, (const char*)src + lo, len, threadIdx.x, blockDim.x);
        channel_signal(c, 0, 1, chan, 320);
    } else {
        channel_wait(c, 1, 0, chan, 321);
        hb_put((char*)dst + lo, (const char*)staging + lo, len, threadIdx.x, blockDim.x);
    }
}

// ---- plain streams: what this GPU's memory sustains for one-directional and 1:1 traffic ------------------
// MODE 0: read nvec 16-byte vectors (their XOR goes to sink[0] only if it is all ones in every lane, which
// keeps the loads alive without a store per thread), 1: write nvec vectors, 2: copy.  Streaming accesses,
// grid-stride, U vectors in flight per thread (8 when only reading): the yardstick the bandwidth kernels are
// held against.
template <int MODE>
__global__ __launch_bounds__(256) void k_stream(const u32x4* src, u32x4* dst, size_t nvec, unsigned* sink)
{
    constexpr int U = MODE == 0 ? 8 : 4;
    const size_t T = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const u32x4 fill = {(unsigned)i, 1u, 2u, 3u};
    for (; i + (U - 1) * T < nvec; i += U * T) {
        if constexpr (MODE == 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) __builtin_nontemporal_store(fill, dst + i + u * T);
        } else {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * T);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (MODE == 0) acc ^= v[u];
                else __builtin_nontemporal_store(v[u], dst + i + u * T);
            }
        }
    }
    for (; i < nvec; i += T) {
        if constexpr (MODE == 1) __builtin_nontemporal_store(fill, dst + i);
        else {
            const u32x4 v = __builtin_nontemporal_load(src + i);
            if constexpr (MODE == 0) acc ^= v;
            else __builtin_nontemporal_store(v, dst + i);
        }
    }
    if constexpr (MODE == 0)
        if ((acc.x & acc.y & acc.z & acc.w) == 0xffffffffu && sink) sink[0] = 1u;
}

// LL encode into caller memory (byte image check against the CPU encoder)
__global__ __launch_bounds__(256) void k_ll_encode(const void* src, size_t nbytes, unsigned flag, u32x4* packets)
{
    const size_t P = (nbytes + 7) / 8;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < P; k += (size_t)gridDim.x * blockDim.x) {
        const size_t off = k * 8;
        unsigned w[2] = {0, 0};
        for (int b = 0; b < 8; ++b)
            if (off + (size_t)b < nbytes) w[b >> 2] |= (unsigned)((const unsigned char*)src)[off + b] << (8 * (b & 3));
        packets[k] = u32x4{w[0], flag, w[1], flag};
    }
}

// LL hand-off through the library scratch: rank 0 writes packets into rank 1's slot 0,
// rank 1 polls each packet and writes the payload out.
__global__ __launch_bounds__(256) void k_ll_roundtrip(DevCtx c, const void* src, void* dst, size_t nbytes,
                                                       int chans)
{
    const int rank = (int)(blockIdx.x & 1u);
    const int chan = (int)(blockIdx.x >> 1);
    const CallTag tag = call_begin(c);
    const unsigned flag = tag.flag, rot = tag.rot;
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)((nbytes + 7) / 8);
    const unsigned RT = (unsigned)chans * blockDim.x;
    const unsigned rt = (unsigned)chan * blockDim.x + threadIdx.x;
    const unsigned base = 1u * c.ll_rank_stride + rot * c.ll_rot_stride;
    for (unsigned k = rt; k < P; k += RT) {
        const size_t off = (size_t)k * 8;
        if (rank == 0) {
            chaos_delay(c, 330);
            unsigned w[2] = {0, 0};
            for (int b = 0; b < 8; ++b)
                if (off + (size_t)b < nbytes) w[b >> 2] |= (unsigned)((const unsigned char*)src)[off + b] << (8 * (b & 3));
            ll_store(rs, base + k * 16u, w[0], w[1], flag);
        } else {
            u32x4 v = {0, 0, 0, 0};
            bool ready = false;
            for (unsigned spins = 0; !ready && spins <= c.spin_limit; ++spins) {
                poll_fence();
                v = ll_load(rs, base + k * 16u);
                ready = ll_ready(v, flag);
            }
            if (!ready) report(c, kStatusTimeout, 1u, 331u, flag, v.y);
            const unsigned w[2] = {v.x, v.z};
            for (int b = 0; b < 8; ++b)
                if (off + (size_t)b < nbytes) ((unsigned char*)dst)[off + b] = (unsigned char)(w[b >> 2] >> (8 * (b & 3)));
        }
    }
    call_end(c, tag);
}

}  // namespace msx
