// LL-protocol AllReduce kernels: one-phase all-pairs (1PA) and two-phase all-pairs (2PA)
// over 16-byte packets {w0, flag, w1, flag} in each receiver's scratch.  Collectives
// Library section (1PA, 2PA with rotating buffers) and MemoryChannel LL protocol.
//
// No semaphore and no fence is used here: a packet is complete when both flags match.
// A thread always works on the same packet index in every phase, so no workgroup barrier
// is needed either.  The scratch has two rotating halves (picked by the call counter) so a
// rank may start the next call while a slow peer still reads the previous call's packets.
// The flag and the half come from device memory (call_begin / call_end), so a launch can be
// captured in a HIP graph and replayed.
#pragma once
#include "msx_device.hpp"

namespace msx {

struct LlArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    const void* res[kMaxRanks];
    size_t nbytes;      // payload bytes per rank
    int n;
    int chans;
    int has_res;
    int res_shared;
};

// payload words of packet k (bytes [8k, 8k+8)), zero padded past nbytes; nbytes is even
__device__ __forceinline__ u32x2 load_words(const void* base, size_t k, size_t nbytes)
{
    const size_t off = k * 8;
    const MSX_GLOBAL char* b = (const MSX_GLOBAL char*)base;
    if (off + 8 <= nbytes) return *(const MSX_GLOBAL u32x2*)(b + off);
    unsigned h[4] = {0, 0, 0, 0};
    for (int i = 0; i < 4; ++i)
        if (off + 2 * i + 2 <= nbytes) h[i] = *(const MSX_GLOBAL unsigned short*)(b + off + 2 * i);
    return u32x2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
}

__device__ __forceinline__ void store_words(void* base, size_t k, size_t nbytes, u32x2 w)
{
    const size_t off = k * 8;
    MSX_GLOBAL char* b = (MSX_GLOBAL char*)base;
    if (off + 8 <= nbytes) { *(MSX_GLOBAL u32x2*)(b + off) = w; return; }
    const unsigned h[4] = {w.x & 0xffffu, w.x >> 16, w.y & 0xffffu, w.y >> 16};
    for (int i = 0; i < 4; ++i)
        if (off + 2 * i + 2 <= nbytes) *(MSX_GLOBAL unsigned short*)(b + off + 2 * i) = (unsigned short)h[i];
}

// Poll packet `pos` of slots j != me (j < n_l) of my scratch until all carry the flag.  Used inside the
// loop over a thread's packets: when the spin budget runs out the thread reports it and leaves that loop.
#define MSX_LL_POLL_ALL(v, base_off, slot_stride, pos)                                        \
    {                                                                                         \
        bool ready = false;                                                                   \
        for (unsigned spins = 0; !ready && spins <= c.spin_limit; ++spins) {                  \
            poll_fence();                                                                     \
            _Pragma("unroll") for (int j = 0; j < kMaxRanks; ++j)                             \
                if (j < n_l && j != rank_l) v[j] = ll_load(rs, (base_off) + (unsigned)j * (slot_stride) + (unsigned)(pos) * 16u); \
            unsigned miss = 0u;              /* any bit set: some packet lacks a flag */       \
            _Pragma("unroll") for (int j = 0; j < kMaxRanks; ++j)                             \
                if (j < n_l && j != rank_l) miss |= (v[j].y ^ tag.flag) | (v[j].w ^ tag.flag);    \
            ready = miss == 0u;                                                               \
        }                                                                                     \
        if (!ready) {                                                                         \
            unsigned late = 0u, seen = 0u;   /* the last slot still without the flag */         \
            _Pragma("unroll") for (int j = 0; j < kMaxRanks; ++j)                             \
                if (j < n_l && j != rank_l && !ll_ready(v[j], tag.flag)) { late = (unsigned)j; seen = v[j].y; } \
            report(c, kStatusTimeout, (unsigned)rank, 100u, tag.flag, seen, late);            \
            break;                           /* nothing is built from packets that never came */ \
        }                                                                                     \
    }

// ---- 1PA: every rank sends ALL its data to every peer, then reduces everything itself --------
template <int DT, int NR>
__global__ __launch_bounds__(1024) void k_allreduce_1pa_ll(LlArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n), rank_l = per_lane(rank);   // per-lane copies for conditions (see per_lane)
    const unsigned P = (unsigned)((a.nbytes + 7) / 8);          // packets per rank
    const unsigned RT = (unsigned)a.chans * blockDim.x;
    const unsigned rt = (unsigned)chan * blockDim.x + threadIdx.x;
    // the payload of my first packet is requested before the call state, so both arrive together
    u32x2 first = {0u, 0u};
    if (rt < P) first = load_words(a.in[rank], rt, a.nbytes);
    const CallTag tag = call_begin(c);
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned slot_stride = P * 16u;
    const unsigned rot_off = tag.rot * c.ll_rot_stride;
    chaos_delay(c, 70);

    // send: my packet k goes to slot `rank` of every peer, all peers before any wait
    for (unsigned k = rt; k < P; k += RT) {
        u32x2 w = k == rt ? first : load_words(a.in[rank], k, a.nbytes);
        settle(w);
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l)
                ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + (unsigned)rank * slot_stride + k * 16u,
                         w.x, w.y, tag.flag);
    }
    // receive + reduce in rank order 0..n-1 (identical bits on every rank)
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + rot_off;
    for (unsigned k = rt; k < P; k += RT) {
        const u32x2 own = k == rt ? first : load_words(a.in[rank], k, a.nbytes);
        u32x2 r = {0u, 0u};
        if (a.has_res) r = load_words(a.res[rank], k, a.nbytes);     // in flight during the poll
        u32x4 v[kMaxRanks];
        MSX_LL_POLL_ALL(v, my_off, slot_stride, k)
        WordAcc<DT> a0, a1;
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l) {
                const unsigned w0 = j == rank_l ? own.x : v[j].x;
                const unsigned w1 = j == rank_l ? own.y : v[j].z;
                if (j == 0) { a0.set(w0); a1.set(w1); } else { a0.add(w0); a1.add(w1); }
            }
        if (a.has_res) { a0.add(r.x); a1.add(r.y); }
        store_words(a.out[rank], k, a.nbytes, u32x2{a0.pack(), a1.pack()});
    }
    call_end(c, tag);
}

// ---- 2PA: reduce-scatter over packets, then all-gather over packets ----------------------------
// Packets are split into n chunks of cp = ceil(P/n); rank r owns chunk r.
//   scratch of rank p, phase 1: slot j (source rank) at (j*cp + q)*16
//                      phase 2: n*cp*16 + (j*cp + q)*16
template <int DT, int NR>
__global__ __launch_bounds__(1024) void k_allreduce_2pa_ll(LlArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n), rank_l = per_lane(rank);   // per-lane copies for conditions (see per_lane)
    const CallTag tag = call_begin(c);
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)((a.nbytes + 7) / 8);
    const unsigned cp = (P + (unsigned)n - 1) / (unsigned)n;
    const unsigned RT = (unsigned)a.chans * blockDim.x;
    const unsigned rt = (unsigned)chan * blockDim.x + threadIdx.x;
    const unsigned slot_stride = cp * 16u;
    const unsigned rot_off = tag.rot * c.ll_rot_stride;
    const unsigned ph2 = (unsigned)n * slot_stride;
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + rot_off;
    chaos_delay(c, 80);

    // phase 1 send: packet q of chunk p goes to slot `rank` of rank p.  All loads first, then
    // all stores, so the n-1 input reads overlap instead of queueing behind each other.
    for (unsigned q = rt; q < cp; q += RT) {
        u32x2 w[kMaxRanks];
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l && (unsigned)p * cp + q < P) w[p] = load_words(a.in[rank], (size_t)p * cp + q, a.nbytes);
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p) settle(w[p]);      // one wait for all the loads, none between the stores
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l && (unsigned)p * cp + q < P)
                ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + (unsigned)rank * slot_stride + q * 16u,
                         w[p].x, w[p].y, tag.flag);
    }
    // phase 1 receive + reduce my chunk, phase 2 send the result to every peer
    for (unsigned q = rt; q < cp; q += RT) {
        const unsigned k = (unsigned)rank * cp + q;
        if (k >= P) break;
        const u32x2 own = load_words(a.in[rank], k, a.nbytes);
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
        if (!a.has_res || a.res_shared) {
            if (a.has_res) {
                const u32x2 r = load_words(a.res[0], k, a.nbytes);
                a0.add(r.x); a1.add(r.y);
            }
            const u32x2 o = {a0.pack(), a1.pack()};
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l && p != rank_l)
                    ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + ph2 + (unsigned)rank * slot_stride + q * 16u,
                             o.x, o.y, tag.flag);
            store_words(a.out[rank], k, a.nbytes, o);
        } else {
            // every destination adds its own residual before the single rounding
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l) {
                    const u32x2 r = load_words(a.res[p], k, a.nbytes);
                    WordAcc<DT> t0 = a0, t1 = a1;
                    t0.add(r.x); t1.add(r.y);
                    const u32x2 o = {t0.pack(), t1.pack()};
                    if (p != rank_l)
                        ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + ph2 + (unsigned)rank * slot_stride + q * 16u,
                                 o.x, o.y, tag.flag);
                    else
                        store_words(a.out[rank], k, a.nbytes, o);
                }
        }
    }
    // phase 2 receive: the other chunks, reduced by their owners
    for (unsigned q = rt; q < cp; q += RT) {
        u32x4 v[kMaxRanks];
        // only slots whose packet exists were sent: the last chunks may be short or empty
        bool ready = false;
        for (unsigned spins = 0; !ready && spins <= c.spin_limit; ++spins) {
            poll_fence();
            ready = true;
#pragma unroll
            for (int j = 0; j < kMaxRanks; ++j)
                if (j < n_l && j != rank_l && (unsigned)j * cp + q < P)
                    v[j] = ll_load(rs, my_off + ph2 + (unsigned)j * slot_stride + q * 16u);
#pragma unroll
            for (int j = 0; j < kMaxRanks; ++j)
                if (j < n_l && j != rank_l && (unsigned)j * cp + q < P) ready = ready && ll_ready(v[j], tag.flag);
        }
        if (!ready) { report(c, kStatusTimeout, (unsigned)rank, 101u, tag.flag, 0u); break; }
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l && j != rank_l && (unsigned)j * cp + q < P)
                store_words(a.out[rank], (size_t)j * cp + q, a.nbytes, u32x2{v[j].x, v[j].z});
    }
    call_end(c, tag);
}

// ---- AllGather and ReduceScatter over LL packets (small messages) -------------------------------
// The two halves of 2PA on their own: the paper evaluates AllGather as a collective of its
// own and says its algorithms mirror the AllReduce ones.  nbytes = bytes per block, a
// multiple of 8 (the host sends other sizes down the HB path).
struct LlCollArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    size_t nbytes;
    int n;
    int chans;
};

// AllGather: rank r's block travels as packets to slot r of every peer's scratch; every rank
// decodes the n-1 foreign slots into its output and copies its own block directly.
template <int NR>
__global__ __launch_bounds__(1024) void k_allgather_ll(LlCollArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n), rank_l = per_lane(rank);   // per-lane copies for conditions (see per_lane)
    const CallTag tag = call_begin(c);
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)(a.nbytes / 8);
    const unsigned RT = (unsigned)a.chans * blockDim.x;
    const unsigned rt = (unsigned)chan * blockDim.x + threadIdx.x;
    const unsigned slot_stride = P * 16u;
    const unsigned rot_off = tag.rot * c.ll_rot_stride;
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + rot_off;
    char* const mine = (char*)a.out[rank] + (size_t)rank * a.nbytes;
    chaos_delay(c, 90);
    for (unsigned k = rt; k < P; k += RT) {
        u32x2 w = load_words(a.in[rank], k, a.nbytes);
        settle(w);
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l)
                ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + (unsigned)rank * slot_stride + k * 16u,
                         w.x, w.y, tag.flag);
        if ((const void*)mine != a.in[rank]) store_words(mine, k, a.nbytes, w);
    }
    for (unsigned k = rt; k < P; k += RT) {
        u32x4 v[kMaxRanks];
        MSX_LL_POLL_ALL(v, my_off, slot_stride, k)
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l && j != rank_l)
                store_words((char*)a.out[rank] + (size_t)j * a.nbytes, k, a.nbytes, u32x2{v[j].x, v[j].z});
    }
    call_end(c, tag);
}

// ReduceScatter: rank r sends block p of its input to slot r of rank p; rank r sums the n-1
// received copies of block r with its own, in rank order, into out[r].
template <int DT, int NR>
__global__ __launch_bounds__(1024) void k_reducescatter_ll(LlCollArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n), rank_l = per_lane(rank);   // per-lane copies for conditions (see per_lane)
    const CallTag tag = call_begin(c);
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned P = (unsigned)(a.nbytes / 8);
    const unsigned RT = (unsigned)a.chans * blockDim.x;
    const unsigned rt = (unsigned)chan * blockDim.x + threadIdx.x;
    const unsigned slot_stride = P * 16u;
    const unsigned rot_off = tag.rot * c.ll_rot_stride;
    const unsigned my_off = (unsigned)rank * c.ll_rank_stride + rot_off;
    chaos_delay(c, 95);
    for (unsigned k = rt; k < P; k += RT) {
        u32x2 w[kMaxRanks];
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l) w[p] = load_words((const char*)a.in[rank] + (size_t)p * a.nbytes, k, a.nbytes);
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p) settle(w[p]);
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != rank_l)
                ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + (unsigned)rank * slot_stride + k * 16u,
                         w[p].x, w[p].y, tag.flag);
    }
    for (unsigned k = rt; k < P; k += RT) {
        const u32x2 own = load_words((const char*)a.in[rank] + (size_t)rank * a.nbytes, k, a.nbytes);
        u32x4 v[kMaxRanks];
        MSX_LL_POLL_ALL(v, my_off, slot_stride, k)
        WordAcc<DT> a0, a1;
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j)
            if (j < n_l) {
                const unsigned w0 = j == rank_l ? own.x : v[j].x;
                const unsigned w1 = j == rank_l ? own.y : v[j].z;
                if (j == 0) { a0.set(w0); a1.set(w1); } else { a0.add(w0); a1.add(w1); }
            }
        store_words(a.out[rank], k, a.nbytes, u32x2{a0.pack(), a1.pack()});
    }
    call_end(c, tag);
}

}  // namespace msx
