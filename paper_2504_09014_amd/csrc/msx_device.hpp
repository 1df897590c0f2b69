// Device-side MemoryChannel primitives for ranks emulated inside one gfx950 GPU.
//
// A "rank" is the set of workgroups b of a launch with b % nranks == rank; workgroup
// b / nranks of a rank is its "channel".  Workgroups are dealt round-robin to the 8 XCDs,
// so with 8 ranks every rank lives on its own XCD and its own L2; anything another rank
// must see therefore has to be made visible at device (agent) scope.
//
//   signal / wait / rank barrier : MemoryChannel "Synchronization" paragraph
//   HB put (16-byte copies)      : MemoryChannel "Data Transfer" paragraph
//   LL packet store / poll       : MemoryChannel "Protocols" paragraph, item (ii)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

namespace msx {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxRanks = 8;
constexpr int kMaxChannels = 256;
constexpr int kSemStrideWords = 32;  // one semaphore per 128-byte line

// status.code values written by the device
constexpr unsigned kStatusOk = 0;
constexpr unsigned kStatusTimeout = 1;
constexpr unsigned kStatusCapacity = 2;
constexpr unsigned kStatusBadIndex = 3;

// Everything a kernel needs from the per-device context; passed by value.
struct DevCtx {
    unsigned* sem;        // [kMaxRanks recv][kMaxRanks send][kMaxChannels] x kSemStrideWords
    unsigned* expected;   // [kMaxRanks recv][kMaxRanks send][kMaxChannels] value the next wait needs
    unsigned* status;     // 8 words: code, rank, site, expected, seen, block
    unsigned* latch;      // host memory the device can write (or null): set to the code of a timeout, so that the
                          // host sees it at its next call without waiting for the device
    unsigned* call_state; // {last LL flag handed out, LL calls so far, workgroups finished this call}
    unsigned* gbar;       // chip-wide barrier: 8 counters, one per 128-byte line, then the 8 values they held when the last call ended
    void* ll;             // LL scratch, ll_bytes long: [rank][rotation][...]
    unsigned ll_bytes;
    unsigned ll_rank_stride;
    unsigned ll_rot_stride;
    unsigned spin_limit;
    int drop_rank;        // failure-path tests: this rank's workgroups leave at once (-1: none)
    unsigned chaos;       // 0, or a seed for pseudo-random delays before signalling
};

__device__ __forceinline__ unsigned sem_index(int recv, int send, int chan)
{
    return (unsigned)((recv * kMaxRanks + send) * kMaxChannels + chan);
}

__device__ __forceinline__ void report(const DevCtx& c, unsigned code, unsigned rank, unsigned site,
                                       unsigned expected, unsigned seen, unsigned extra = 0u)
{
    if (atomicCAS(c.status, 0u, code) == 0u) {
        c.status[1] = rank;
        c.status[2] = site;
        c.status[3] = expected;
        c.status[4] = seen;
        c.status[5] = blockIdx.x;
        c.status[6] = extra;
        if (code == kStatusTimeout && c.latch)
            __hip_atomic_store(c.latch, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Pseudo-random pause (tests only): makes workgroups arrive at their signals in scrambled order.
__device__ __forceinline__ void chaos_delay(const DevCtx& c, unsigned site)
{
    if (c.chaos == 0) return;
    unsigned h = (c.chaos * 2654435761u) ^ (blockIdx.x * 40503u + site * 9176u + 0x9e3779b9u);
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    unsigned n = h & 1023u;
    for (unsigned i = 0; i < n; ++i) __builtin_amdgcn_s_sleep(8);
}

// ---- wave-uniform values in conditions ----------------------------------------------------
// A copy of a wave-uniform integer (the rank, the rank count) that the compiler must treat as a
// per-lane value.  Conditions such as `j != rank` or `j < n` inside the unrolled per-peer loops
// are formed from these copies, so they take the ordinary divergent-branch lowering.  Formed from
// the uniform originals they are kept as 64-bit lane masks across loops, and this compiler
// re-derives such a mask with vector compares wherever it needs the negation, also inside a
// loop whose lanes leave at different iterations.  That mask has bits only for the lanes still
// active there; a later loop running with other lanes reads it as false (seen as an LL poll loop
// that, once lane 0 had left, started waiting on the rank's own, never written, packet slot).
__device__ __forceinline__ int per_lane(int x)
{
    asm("" : "+v"(x));
    return x;
}

// ---- semaphores ---------------------------------------------------------------------

// signal(): make every earlier store of this workgroup visible device-wide, then bump the
// receiver's counter.  Call from ONE thread, after a workgroup barrier if other threads
// of the workgroup produced the data.  release = false skips the fence: for a signal that
// publishes no data of this launch ("I have arrived", "I am done reading").
__device__ __forceinline__ void sem_signal(unsigned* sem, bool release = true)
{
    if (release) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(sem, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The spinning half of wait(): one thread polls until the counter has reached `expected`
// (signed distance, so the 32-bit counter may wrap), then acquires.  Returns false and
// records the timeout when the spin budget runs out.
__device__ __forceinline__ bool sem_spin(const DevCtx& c, unsigned* sem, unsigned expected,
                                         unsigned rank, unsigned site, bool acquire = true)
{
    unsigned seen = 0;
    bool ok = false;
    for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
        seen = __hip_atomic_load(sem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((int)(seen - expected) >= 0) { ok = true; break; }
        __builtin_amdgcn_s_sleep(1);
    }
    if (acquire) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    if (!ok) report(c, kStatusTimeout, rank, site, expected, seen);
    return ok;
}

// One-directional hand-off helpers for a (sender rank -> receiver rank) channel.
// Both are workgroup-collective: every thread of the workgroup must call them.
// release = false is for puts made with write-through stores and drained by every wave
// (st16_wt + put_drain): they are already visible device-wide when the workgroup barrier ends.
__device__ __forceinline__ void channel_signal(const DevCtx& c, int me, int peer, int chan, unsigned site,
                                               bool release = true)
{
    __syncthreads();   // all threads' puts are issued and complete before the release below
    if (threadIdx.x == 0) {
        chaos_delay(c, site);
        sem_signal(c.sem + (size_t)sem_index(peer, me, chan) * kSemStrideWords, release);
    }
}

// Returns false (in every thread) when the wait ran out of its spin budget: what the peer was to deliver is
// not there, and the caller must not go on to consume it (nor wait again in this launch: the result word in
// LDS is rewritten by the next wait without a barrier in between).
__device__ __forceinline__ bool channel_wait(const DevCtx& c, int me, int peer, int chan, unsigned site,
                                             bool acquire = true)
{
    __shared__ unsigned wait_failed;
    if (threadIdx.x == 0) {
        unsigned idx = sem_index(me, peer, chan);
        unsigned want = c.expected[idx] + 1u;
        c.expected[idx] = want;
        wait_failed = sem_spin(c, c.sem + (size_t)idx * kSemStrideWords, want, (unsigned)me, site, acquire) ? 0u : 1u;
    }
    __syncthreads();   // the first thread waited for everybody
    return wait_failed == 0u;
}

// Barrier among all ranks on one channel: signal every peer, then wait for every peer.
// Threads 0..n-2 each serve one peer so the n-1 hops overlap.  Workgroup-collective.
//   release: this workgroup wrote data the peers (or their next kernel) will read
//   acquire: this workgroup is about to read data the peers wrote
// A device-scope release writes the whole L2 of this XCD back and an acquire invalidates it,
// and those operations queue up per XCD, so each barrier asks only for what it needs.
// CHECKED: the result tells every thread whether all peers arrived in time (through a word in LDS: one store
// and one load more); the unchecked form is for barriers with nothing behind them that depends on the peers.
template <bool CHECKED = false>
__device__ __forceinline__ bool rank_barrier(const DevCtx& c, int me, int n, int chan, unsigned site,
                                             bool release = true, bool acquire = true)
{
    __shared__ unsigned barrier_failed;
    if (CHECKED && threadIdx.x == 0) barrier_failed = 0u;   // only ever re-armed by a thread that saw it clear
    __syncthreads();
    const int t = (int)threadIdx.x;
    if (t < n - 1) {
        int peer = me + 1 + t;
        if (peer >= n) peer -= n;
        chaos_delay(c, site + (unsigned)t);
        sem_signal(c.sem + (size_t)sem_index(peer, me, chan) * kSemStrideWords, release);
        unsigned idx = sem_index(me, peer, chan);
        unsigned want = c.expected[idx] + 1u;
        c.expected[idx] = want;
        const bool ok = sem_spin(c, c.sem + (size_t)idx * kSemStrideWords, want, (unsigned)me, site, acquire);
        if (CHECKED && !ok) barrier_failed = 1u;
    }
    __syncthreads();
    return CHECKED ? barrier_failed == 0u : true;
}

// ---- barrier over every workgroup of a co-resident launch -----------------------------------------
// Eight counters (workgroup b adds to counter b % 8, so the arrivals of one barrier queue up on eight
// lines instead of one); the first wave of every workgroup polls all eight with one 8-lane load.  The
// counters only grow: a call reads, when it starts, the values they had when the last call ended (kept
// beside them), and workgroup 0 leaves the new values behind when it has passed its last barrier (every
// workgroup has read the old ones by then).  Signed distances, so the counters may wrap.
// Measured on MI355X with 256 workgroups: about 2 us from the last arrival to the release (one counter
// and one polling thread: 5 us).
struct GridBar { unsigned base, per_gen; bool ok; };   // lanes 0..7 of the first wave hold counter x's values

constexpr int kGridBarBaseWord = 8 * kSemStrideWords;
constexpr int kGridBarPaceWord = kGridBarBaseWord + kSemStrideWords;     // a word of its own line: the write-phase schedule
constexpr unsigned kPaceSlots = 31;    // remembered shapes: word 0 of the first line is the running launch's pace, 4 words per slot behind it
constexpr size_t kGridBarBytes = (size_t)(kGridBarPaceWord + 4 + 4 * kPaceSlots) * 4;

// Workgroup-collective; first thing (before any arrival of this call can have happened: an arrival
// needs this workgroup's own).
__device__ __forceinline__ GridBar grid_barrier_begin(const DevCtx& c)
{
    GridBar g{0u, 0u, true};
    if (threadIdx.x < 8) {
        g.base = c.gbar[kGridBarBaseWord + threadIdx.x];
        g.per_gen = (gridDim.x + 7u - threadIdx.x) / 8u;      // workgroups b with b % 8 == x
    }
    return g;
}

// gen = 1, 2, ... counts this call's barriers; every workgroup of the launch takes part in each.
// No fence: data the workgroups exchange is written through and drained before the call.
__device__ __forceinline__ void grid_barrier(const DevCtx& c, GridBar& g, unsigned gen, unsigned rank, unsigned site)
{
    __syncthreads();
    if (threadIdx.x < 64) {
        if (threadIdx.x == 0) {
            chaos_delay(c, site + gen);
            __hip_atomic_fetch_add(c.gbar + (blockIdx.x & 7u) * kSemStrideWords, 1u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        const unsigned want = g.base + gen * g.per_gen;
        unsigned seen = want;
        if (g.ok) {                                              // after one timeout the call no longer waits
            bool done = false;
            for (unsigned spins = 0; spins <= c.spin_limit; ++spins) {
                if (threadIdx.x < 8)
                    seen = __hip_atomic_load(c.gbar + threadIdx.x * kSemStrideWords, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
                if (__all((int)(seen - want) >= 0)) { done = true; break; }
                __builtin_amdgcn_s_sleep(1);
            }
            if (!done) {
                g.ok = false;
                if ((int)(seen - want) < 0) report(c, kStatusTimeout, rank, site, want, seen, threadIdx.x);
            }
        }
    }
    __syncthreads();
}

// Workgroup-collective; after the call's last barrier (gens = how many there were).
__device__ __forceinline__ void grid_barrier_end(const DevCtx& c, const GridBar& g, unsigned gens)
{
    if (blockIdx.x == 0 && threadIdx.x < 8) c.gbar[kGridBarBaseWord + threadIdx.x] = g.base + gens * g.per_gen;
}

// ---- pacing against the wall clock ------------------------------------------------------------------
// Holds the wave until the 100 MHz wall clock has reached `target`.  Written as one assembly block: a C++
// loop (or even a branch around this call) between the loads and sums of a long unrolled sequence made
// the register allocator spill a thousand registers.  The clock always advances, so the loop ends; callers
// keep targets within a millisecond of the present.
__device__ __forceinline__ void wait_until(unsigned long long target)
{
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)target);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(target >> 32));
    asm volatile(
        "1:\n\t"
        "s_memrealtime s[90:91]\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "s_sub_u32 s90, s90, %0\n\t"
        "s_subb_u32 s91, s91, %1\n\t"
        "s_cmp_lt_i32 s91, 0\n\t"        // now - target < 0: not yet
        "s_cbranch_scc0 2f\n\t"
        "s_sleep 1\n\t"
        "s_branch 1b\n"
        "2:\n\t"
        :
        : "s"(lo), "s"(hi)
        : "s90", "s91", "scc");
}

// ---- the schedule of paced write phases (phased kernels) -----------------------------------------
// A write phase of H tiles is held to `pace` wall-clock ticks per tile (wait_until), so that all dies finish
// it together; the controller looks for the tightest schedule the memory system still meets.  Workgroup 0
// decides after every full write phase, from how long the phase took, and leaves the new pace in the barrier's
// memory; everybody picks it up behind the next barrier, so the whole launch follows one schedule.
//   first full phase (unpaced): pace = 29/32 of what it took per tile
//   schedule met (done within 1/16 + 3 us of it): remember it, and tighten by 1/13 unless frozen
//   schedule missed (too tight: nobody is held back any more and the slow dies are late again): back to the
//   last one that was met, and stop tightening; missed three times in a row: learn again from scratch; missed
//   before any was met: loosen by 1/16
//   frozen and met 256 times in a row: tighten once more (conditions may have changed since the miss that froze
//   it - another launch beside it, a colder chip - and a schedule that is merely met is never found too loose
//   otherwise); a miss sends it straight back to the last good one
// The state outlives the call (beside the barrier counters, 31 slots tagged with the shape of the launch), so
// a call of a shape seen before starts from the schedule that one ended with.
struct PaceCtl { unsigned pace, good, frozen, misses, age; };
constexpr unsigned kPaceRetryAfter = 256;

// no schedule is slower than this many ticks per tile (15 us; a phase of 64 tiles then lasts a millisecond):
// whatever the words in memory say, a wave never waits longer
constexpr unsigned kMaxPace = 1500;
__host__ __device__ __forceinline__ unsigned pace_clamp(unsigned pace) { return pace > kMaxPace ? 0u : pace; }

// word 0 of the first line: the pace of the launch that is running; behind it kPaceSlots remembered shapes,
// direct-mapped (a bench run alone meets a dozen shapes; with seven slots they kept evicting each other)
__device__ __forceinline__ PaceCtl pace_load(const DevCtx& c, unsigned key)
{
    const unsigned* w = c.gbar + kGridBarPaceWord + 4u + ((key >> 7) % kPaceSlots) * 4u;
    PaceCtl p{0u, 0u, 0u, 0u, 0u};
    if (w[1] == key) { p.pace = pace_clamp(w[0]); p.good = pace_clamp(w[2]); p.frozen = w[3] & 1u; p.misses = (w[3] >> 8) & 3u; p.age = (w[3] >> 16) & 0x1ffu; }
    return p;
}

// workgroup 0, one thread, after the call's last barrier
__device__ __forceinline__ void pace_save(const DevCtx& c, const PaceCtl& p, unsigned key)
{
    unsigned* w = c.gbar + kGridBarPaceWord + 4u + ((key >> 7) % kPaceSlots) * 4u;
    w[0] = p.pace; w[1] = key; w[2] = p.good; w[3] = (p.frozen & 1u) | (p.misses << 8) | (p.age << 16);
}

__host__ __device__ __forceinline__ void pace_update(PaceCtl& p, unsigned long long took, unsigned tiles)
{
    if (took >= 100000ull) return;                                  // a millisecond: something else is going on
    const unsigned t = (unsigned)took;
    const unsigned fresh = pace_clamp(t * 29u / (32u * tiles));
    if (p.pace == 0) {
        p.pace = fresh;
    } else {
        const unsigned sched = p.pace * tiles;
        if (t <= sched + sched / 16u + 300u) {
            p.good = p.pace;
            p.misses = 0;
            if (!p.frozen) { p.pace = p.pace * 12u / 13u; p.age = 0; }
            else if (++p.age >= kPaceRetryAfter) { p.age = 0; p.frozen = 0; }
        } else if (!p.good) {
            // no schedule has been met yet: this one is too tight, try a looser one (never looser than what the
            // unpaced phase just took, which is met by definition and ends the search)
            const unsigned looser = p.pace + p.pace / 16u + 1u, unpaced = t / tiles + 1u;
            p.pace = pace_clamp(looser < unpaced ? looser : unpaced);
        } else if (++p.misses >= 3u) {
            p = PaceCtl{fresh, 0u, 0u, 0u, 0u};
        } else {
            p.pace = p.good;
            p.frozen = 1u;
        }
    }
}

// ---- per-call flag and scratch rotation for the LL protocol -----------------------------------
// The flag of a call and the scratch half it uses come from device memory, not from kernel
// arguments, so a captured launch can be replayed: every workgroup reads the state when it
// starts and then counts itself in; the workgroup that finds all others counted advances the
// state when it ends (every workgroup has read it by then).  Counting in at the start keeps the
// counter's round trip off the end of the kernel, where nothing else is left to hide it.
struct CallTag { unsigned flag; unsigned rot; unsigned arrivals; unsigned calls; };

// Workgroup-collective; every workgroup of the launch calls it exactly once, first thing.
__device__ __forceinline__ CallTag call_begin(const DevCtx& c)
{
    const unsigned e = c.call_state[0], k = c.call_state[1];
    asm volatile("" ::"s"(e), "s"(k));   // both values have arrived before the barrier below
    __syncthreads();                     // ... in every wave of this workgroup
    unsigned arrivals = 0u;
    if (threadIdx.x == 0)
        arrivals = __hip_atomic_fetch_add(c.call_state + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned f = e + 1u;
    if (f == 0u) f = 1u;            // 0 is what untouched scratch holds
    return CallTag{f, k & 1u, arrivals, k};
}

// Every workgroup calls it exactly once, at its end (any path).
__device__ __forceinline__ void call_end(const DevCtx& c, CallTag tag)
{
    if (threadIdx.x == 0 && tag.arrivals == gridDim.x - 1u) {
        __hip_atomic_store(c.call_state + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(c.call_state + 0, tag.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(c.call_state + 1, tag.calls + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- HB protocol: cooperative 16-byte copy ---------------------------------------------

// put(): threads tid of tids copy nbytes from src to dst (both 16-byte aligned when
// nbytes >= 16; a tail shorter than 16 bytes is moved bytewise by the first threads).
__device__ __forceinline__ void hb_put(void* dst, const void* src, size_t nbytes, size_t tid, size_t tids)
{
    const u32x4* s = (const u32x4*)src;
    u32x4* d = (u32x4*)dst;
    const size_t nvec = nbytes >> 4;
    size_t i = tid;
    for (; i + 3 * tids < nvec; i += 4 * tids) {
        u32x4 a = __builtin_nontemporal_load(s + i);
        u32x4 b = __builtin_nontemporal_load(s + i + tids);
        u32x4 e = __builtin_nontemporal_load(s + i + 2 * tids);
        u32x4 f = __builtin_nontemporal_load(s + i + 3 * tids);
        __builtin_nontemporal_store(a, d + i);
        __builtin_nontemporal_store(b, d + i + tids);
        __builtin_nontemporal_store(e, d + i + 2 * tids);
        __builtin_nontemporal_store(f, d + i + 3 * tids);
    }
    for (; i < nvec; i += tids) __builtin_nontemporal_store(__builtin_nontemporal_load(s + i), d + i);
    const size_t done = nvec << 4;
    for (size_t b = done + tid; b < nbytes; b += tids)
        ((unsigned char*)dst)[b] = ((const unsigned char*)src)[b];
}

// ---- LL protocol: 16-byte packets = two 8-byte units {data, flag} -------------------------

// The LL scratch is addressed through one buffer descriptor: accesses carry the device
// (agent) scope bit so that a packet store goes straight to memory the other XCDs see and
// a poll never reads a stale line; out-of-range offsets are dropped by the hardware
// range check instead of faulting.
constexpr int kAuxAgentScope = 1 << 4;      // "sc1" on this target

__device__ __forceinline__ __amdgpu_buffer_rsrc_t ll_resource(const DevCtx& c)
{
    return __builtin_amdgcn_make_buffer_rsrc(c.ll, 0, (int)c.ll_bytes, 0x00020000);
}

__device__ __forceinline__ void ll_store(__amdgpu_buffer_rsrc_t r, unsigned byte_off, unsigned w0,
                                         unsigned w1, unsigned flag)
{
    u32x4 p = {w0, flag, w1, flag};
    __builtin_amdgcn_raw_buffer_store_b128(p, r, (int)byte_off, 0, kAuxAgentScope);
}

__device__ __forceinline__ u32x4 ll_load(__amdgpu_buffer_rsrc_t r, unsigned byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kAuxAgentScope);
}

__device__ __forceinline__ bool ll_ready(u32x4 p, unsigned flag)
{
    return p.y == flag && p.w == flag;   // both units of the packet must carry the flag
}

// Keeps the compiler from hoisting a poll out of its retry loop.
__device__ __forceinline__ void poll_fence() { asm volatile("" ::: "memory"); }

// ---- element arithmetic -------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even, NaN kept quiet
__device__ __forceinline__ unsigned bf16_round(float f)
{
    unsigned u = __float_as_uint(f);
    unsigned r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    unsigned q = (u >> 16) | 0x40u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? q : r;
}

// Four fp32 -> four OCP E4M3 codes in one word (a in bits 0-7).  E4M3: 1-4-3, bias 7, largest finite 448 =
// 0x7E, no infinity; round to nearest even, magnitudes from 448 up (and infinities) saturate to 0x7E, NaN ->
// 0x7F.  Done by the conversion instruction of the matrix-core data types (denormals kept).  It is fed
// values clamped to +-448, so that what it does on overflow never matters (infinities saturate like the rest);
// the clamp does not keep NaNs, so those are patched in afterwards as 0x7F.
__device__ __forceinline__ unsigned e4m3_quad(float a, float b, float c, float d)
{
    const float ca = __builtin_amdgcn_fmed3f(a, 448.0f, -448.0f), cb = __builtin_amdgcn_fmed3f(b, 448.0f, -448.0f);
    const float cc = __builtin_amdgcn_fmed3f(c, 448.0f, -448.0f), cd = __builtin_amdgcn_fmed3f(d, 448.0f, -448.0f);
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(cc, cd, w, true);
    unsigned u = (unsigned)w;
    if (a != a) u = (u & 0xffffff00u) | 0x0000007fu;
    if (b != b) u = (u & 0xffff00ffu) | 0x00007f00u;
    if (c != c) u = (u & 0xff00ffffu) | 0x007f0000u;
    if (d != d) u = (u & 0x00ffffffu) | 0x7f000000u;
    return u;
}

// Accumulator for the elements held in one 32-bit word: 1 x fp32 or 2 x bf16.
template <int DT> struct WordAcc;
template <> struct WordAcc<0> {   // fp32
    float a;
    __device__ __forceinline__ void set(unsigned w) { a = __uint_as_float(w); }
    __device__ __forceinline__ void add(unsigned w) { a += __uint_as_float(w); }
    __device__ __forceinline__ unsigned pack() const { return __float_as_uint(a); }
};
template <> struct WordAcc<1> {   // bf16 pair
    float lo, hi;
    __device__ __forceinline__ void set(unsigned w) { lo = bf16_lo(w); hi = bf16_hi(w); }
    __device__ __forceinline__ void add(unsigned w) { lo += bf16_lo(w); hi += bf16_hi(w); }
    __device__ __forceinline__ unsigned pack() const { return bf16_round(lo) | (bf16_round(hi) << 16); }
};

template <int DT> struct VecAcc {
    WordAcc<DT> w[4];
    __device__ __forceinline__ void set(u32x4 v) { w[0].set(v.x); w[1].set(v.y); w[2].set(v.z); w[3].set(v.w); }
    __device__ __forceinline__ void add(u32x4 v) { w[0].add(v.x); w[1].add(v.y); w[2].add(v.z); w[3].add(v.w); }
    __device__ __forceinline__ u32x4 pack() const { return u32x4{w[0].pack(), w[1].pack(), w[2].pack(), w[3].pack()}; }
};

// Rank buffers are device memory.  Saying so in the pointer type keeps every access a global one also where
// the pointer reaches the kernel through a table in LDS (the plan interpreter), where the compiler could not
// tell and would fall back to flat accesses.
#define MSX_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ u32x4 ld16(const void* base, size_t vec_index)
{
    return __builtin_nontemporal_load((const MSX_GLOBAL u32x4*)base + vec_index);
}
// the same load without the streaming hint: the line may stay in the caches
__device__ __forceinline__ u32x4 ld16_keep(const void* base, size_t vec_index)
{
    return *((const MSX_GLOBAL u32x4*)base + vec_index);
}
__device__ __forceinline__ void st16(void* base, size_t vec_index, u32x4 v)
{
    __builtin_nontemporal_store(v, (MSX_GLOBAL u32x4*)base + vec_index);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order: a loop whose index is a constant
// in every iteration whatever the optimiser's unrolling limits are
template <int... I, class F>
__device__ __forceinline__ void static_for_each(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f)
{
    static_for_each(std::make_integer_sequence<int, N>{}, f);
}

// Marks a loaded vector as consumed.  The write-through stores below are inline assembly, whose memory
// counter the compiler cannot see: when a conditional store is the first use of a loaded register, the
// compiler waits for "all outstanding memory operations" in front of it, which also drains the stores issued
// so far, and a sequence of conditional stores to N peers then runs one round trip at a time (measured: a
// small AllGather 4.8 us instead of 3.3 us).  Settling the vector once, before the stores, leaves no load
// pending at any of them.
__device__ __forceinline__ void settle(u32x4& v) { asm volatile("" : "+v"(v)); }
// The same for the payload of an LL packet.  The packet stores are builtins, which the compiler does count,
// but it cannot carry the count across the per-peer conditions either: without this every peer's store sat
// behind a wait for ALL earlier memory operations, the previous peer's store included (seven store round trips
// one after the other in the first phase of 2PA).
__device__ __forceinline__ void settle(u32x2& v) { asm volatile("" : "+v"(v)); }

// First 16-byte vector of rank r's chunk when V vectors are split over n ranks: the even split rounded down
// to a whole 128-byte line (8 vectors), so that no two ranks write into the same line and every wave's accesses
// start on a line (with 7 ranks the unaligned split cost 20 % of the bandwidth).  chunk_begin(V, n, n) = V.
__host__ __device__ __forceinline__ size_t chunk_begin(size_t V, int r, int n)
{
    if (r >= n) return V;
    const size_t b = V * (size_t)r / (size_t)n;
    return V >= (size_t)64 * (size_t)n ? (b & ~(size_t)7) : b;     // tiny inputs keep the exact split
}

// ---- write-through put ---------------------------------------------------------------------------
// A device-scope release fence writes the whole L2 of the XCD back, and those write-backs queue
// up per XCD (measured: about 0.16 us per workgroup and barrier, 40 us for 256 workgroups per
// rank).  The bulk data of a put therefore goes out with DEVICE-SCOPE, write-through, streaming
// 16-byte stores: such a store is performed at the point all XCDs share before it is counted
// as complete, so once every wave of the workgroup has drained its store counter
// (put_drain, then the workgroup barrier inside the signal) the data is visible device-wide
// and the semaphore increment needs no L2 write-back in front of it.  Same HBM bandwidth as
// ordinary streaming stores (measured).  The two wait states after the store cover the
// "wide store data overwritten by the next VALU instruction" hazard, which the compiler
// cannot see inside inline assembly.
__device__ __forceinline__ void st16_wt(void* base, size_t vec_index, u32x4 v)
{
    u32x4* p = (u32x4*)base + vec_index;
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// the same write-through store without the streaming hint: the memory-side cache may keep the line, which
// pays while everything a call writes fits into it (measured: 6.7 instead of 5.6 TB/s at 32 MiB per rank)
__device__ __forceinline__ void st16_wt_keep(void* base, size_t vec_index, u32x4 v)
{
    u32x4* p = (u32x4*)base + vec_index;
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// the same with the address as a wave-uniform base (scalar registers) plus a 32-bit byte offset per lane: one
// vector register of address instead of two, where registers are what a kernel runs out of
__device__ __forceinline__ void st16_wt_keep_at(const void* uniform_base, unsigned byte_off, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, %2 sc1\n\ts_nop 1" : : "v"(byte_off), "v"(v), "s"(uniform_base) : "memory");
}
__device__ __forceinline__ void st8_wt(void* addr, u32x2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void st32_wt(void* addr, unsigned v)
{
    asm volatile("global_store_dword %0, %1, off sc1" : : "v"(addr), "v"(v) : "memory");
}
// every store this wave has issued (write-through ones included) is complete
__device__ __forceinline__ void put_drain() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }

}  // namespace msx
