// Host side of libmsx: per-device context, options, argument checks, algorithm choice and
// launches behind the C ABI declared in include/msx.h.  Every launch is sized so that all
// of its workgroups are resident at once (ranks wait on each other inside one kernel).
#include "../../include/msx.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <functional>
#include <memory>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <thread>

#include "msx_device.hpp"
#include "msx_kernels_hb.hpp"
#include "msx_phased.hpp"
#include "msx_kernels_ll.hpp"
#include "msx_kernels_moe.hpp"
#include "msx_kernels_plan.hpp"
#include "msx_plan.hpp"
#include "msx_combine.hpp"
#include "msx_kernels_generic.hpp"
#include "msx_port.hpp"
#include "msx_kernels_prim.hpp"

using namespace msx;

namespace {

struct Options {
    int algo = MSX_ALGO_AUTO;
    // Automatic choice, from the per-size sweep on MI355X: inside one chip a peer's buffer is as
    // close as the rank's own, so the fused HB kernel (two flag hops, 16 S bytes) beats the packet
    // protocols from 4 KiB up; 1PA-LL ties with it below.  2PA-LL is reachable by request only.
    size_t ll_1pa_max = 2u << 10;
    size_t ll_2pa_max = 0;
    size_t ll_max_bytes = 4u << 20;
    int hb_blocks = 0, ll_blocks = 0, threads = 0;
    int hb_unroll = 0;        // 0 = by size
    int cache_mode = -1;      // -1 = by footprint, else 0 | 1 | 2 (see choose_cache_mode)
    // fused HB AllReduce: from this many bytes per rank on, the launch alternates between chip-wide read and
    // write phases (k_allreduce_hb_phased).  -1 = automatic: 8 ranks from 40 MiB, the AllReduce of 3 to 7 ranks
    // from 64 or 128 MiB (see use_phased), never otherwise
    long long hb_phased_min = -1;
    size_t a2a_blocks_min = (size_t)4 << 20;   // all-to-all: block after block from blocks of this many bytes
    int hb_barriers = 1;
    int hb_pace = 1;          // phased kernels: pace the write phase (see k_allreduce_hb_phased)
    int peer_outer = 0;
    int barrier_fences = 3;   // msx_prim_barrier only: bit 0 release, bit 1 acquire
    int coll_algo = 0;        // allgather / reducescatter: 0 auto, 1 LL packets, 2 HB
    size_t coll_ll_max = 0;   // auto: LL up to this many bytes per block (0: never; HB wins on one chip)
    unsigned spin_limit = 1u << 20;
    int drop_rank = -1;
    unsigned chaos = 0;
};

// PortChannel emulation: the FIFOs in pinned host memory and the CPU proxy thread that serves them.
struct Port {
    PortShared* shared = nullptr;      // host address (pinned, mapped)
    PortShared* shared_dev = nullptr;  // the same memory as the device sees it
    unsigned* sem = nullptr;           // the context's device-side semaphores (signals land there)
    hipStream_t stream = nullptr;      // the proxy's own stream (default priority)
    std::vector<hipEvent_t> events;    // for flush requests, reused in turn
    std::thread thread;
    std::mutex mu;
    std::condition_variable cv;
    unsigned long long announced = 0;  // requests launched kernels will push in total
    unsigned long long consumed = 0;   // requests served so far
    bool stop = false;
    std::atomic<int> hip_error{0};     // first HIP error the proxy ran into (it stops signalling then)
    int device = 0;
};

// Where a token dispatch leaves the slots of its tokens for the combine that follows.
struct Ctx;
struct MoePlan {
    Ctx* owner = nullptr;
    void* slots = nullptr;         // u16 [kMaxRanks][T][8]
    size_t slots_bytes = 0;
    unsigned* base = nullptr;      // u32 [kMaxRanks][8]
    int T = -1, n = 0;             // shape of the routing the last dispatch through this plan left behind
    bool fixed_size = false;       // created by msx_moe_plan_create: never regrown inside a dispatch
};

struct Ctx {
    int device = -1;
    DevCtx d{};
    int cus = 0;
    double ns_per_tick = 10.0;
    MoePlan moe;                   // the built-in routing plan (grown on demand)
    unsigned* latch = nullptr;     // pinned host word the kernels set on a timeout (d.latch is its device address)
    int max_blocks = 0;            // workgroups one launch of this context may take (0: all the GPU can hold)
    void* ring = nullptr;          // ring AllReduce: per-rank receive scratch, grown on demand
    size_t ring_bytes = 0;
    struct Plan { int algo, n, chans, held; size_t nbytes; PlanOp* ops; unsigned stride; int head; };
    std::vector<Plan> plans;       // lowered execution plans, kept on the device
    Port* port = nullptr;          // created on the first port-channel call
    unsigned* snap = nullptr;  // small device scratch for snapshots
    size_t ll_limit = 0;       // ll_max_bytes this context was sized for
    bool fixed = false;        // its device memory is the file-scope array below: nothing to free, nothing may grow
    std::map<std::pair<const void*, int>, int> occ;   // (kernel, threads) -> resident blocks per CU
};

std::mutex g_mu;
Options g_opt;
unsigned g_status_detail = 0;   // seventh status word of the last reported event (which peer was late)
Ctx* g_ctx[64] = {};
thread_local int t_hip_err = 0;
thread_local int t_grid = 0, t_block = 0, t_algo = 0;

int hip_fail(hipError_t e)
{
    t_hip_err = (int)e;
    return MSX_ERR_HIP;
}
#define HIPCHK(x)                                    \
    do {                                             \
        hipError_t e_ = (x);                         \
        if (e_ != hipSuccess) return hip_fail(e_);   \
    } while (0)

size_t elem_size(int dtype) { return (dtype == MSX_F32 || dtype == MSX_I32) ? 4 : 2; }
bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// The proxy: pops requests of every rank's FIFO in order.  put -> a device-to-device copy on the proxy's stream;
// signal -> a one-wave kernel behind it on the same stream (ordered after the copies, nothing waits on the CPU);
// flush -> an event behind what has been enqueued, polled until it has fired.  After a HIP error nothing more is
// copied or signalled: the waiting ranks run into their timeouts, and msx_status names the error.
void port_proxy(Port* p)
{
    (void)hipSetDevice(p->device);
    unsigned long long taken[kMaxRanks] = {};
    for (int r = 0; r < kMaxRanks; ++r) taken[r] = p->shared->fifo[r].tail;
    struct Pending { int rank; unsigned long long seq; hipEvent_t ev; };
    std::vector<Pending> pending;
    size_t next_event = 0;
    auto fail = [&](hipError_t e) {
        int none = 0;
        p->hip_error.compare_exchange_strong(none, (int)e);
    };
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(p->mu);
            p->cv.wait(lk, [&] { return p->stop || p->consumed < p->announced || !pending.empty(); });
            if (p->stop) break;
        }
        auto idle_since = std::chrono::steady_clock::now();
        for (;;) {
            {
                std::lock_guard<std::mutex> lk(p->mu);
                if (p->stop || (p->consumed >= p->announced && pending.empty())) break;
            }
            bool progress = false;
            for (int r = 0; r < kMaxRanks; ++r) {
                PortFifo* f = &p->shared->fifo[r];
                while (__atomic_load_n(&f->head, __ATOMIC_ACQUIRE) > taken[r]) {
                    const PortReq q = f->req[taken[r] % kPortSlots];
                    const unsigned long long seq = ++taken[r];
                    const bool ok = p->hip_error.load() == 0;
                    if (q.type == kPortPut) {
                        if (ok && q.bytes) {
                            hipError_t e = hipMemcpyAsync((void*)q.dst, (const void*)q.src, (size_t)q.bytes,
                                                          hipMemcpyDeviceToDevice, p->stream);
                            if (e != hipSuccess) fail(e);
                        }
                    } else if (q.type == kPortSignal) {
                        const int recv = (int)(q.arg & 0xffu), send = (int)((q.arg >> 8) & 0xffu), nsem = (int)(q.arg >> 16);
                        if (ok && recv < kMaxRanks && send < kMaxRanks && nsem >= 1 && nsem <= kMaxChannels) {
                            hipLaunchKernelGGL(k_port_signal, dim3(1), dim3(nsem <= 64 ? 64 : 256), 0, p->stream, p->sem, recv, send, nsem);
                            hipError_t e = hipGetLastError();
                            if (e != hipSuccess) fail(e);
                        }
                    } else if (q.type == kPortFlush) {
                        hipEvent_t ev = p->events[next_event++ % p->events.size()];
                        hipError_t e = ok ? hipEventRecord(ev, p->stream) : hipErrorUnknown;
                        if (e == hipSuccess) pending.push_back(Pending{r, seq, ev});
                        else if (ok) fail(e);
                    }
                    __atomic_store_n(&f->tail, seq, __ATOMIC_RELEASE);
                    std::lock_guard<std::mutex> lk(p->mu);
                    ++p->consumed;
                    progress = true;
                }
            }
            for (size_t k = 0; k < pending.size();) {
                const hipError_t e = hipEventQuery(pending[k].ev);
                if (e == hipErrorNotReady) { ++k; continue; }
                if (e == hipSuccess) __atomic_store_n(&p->shared->fifo[pending[k].rank].flushed, pending[k].seq, __ATOMIC_RELEASE);
                else fail(e);
                pending.erase(pending.begin() + (long)k);
                progress = true;
            }
            if (progress) {
                idle_since = std::chrono::steady_clock::now();
            } else if (std::chrono::steady_clock::now() - idle_since > std::chrono::seconds(3)) {
                std::lock_guard<std::mutex> lk(p->mu);   // the kernels never pushed what they announced: forget the rest
                p->announced = p->consumed;
                pending.clear();
            } else {
                std::this_thread::yield();
            }
        }
    }
}

void destroy_port(Port* p)
{
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->stop = true;
    }
    p->cv.notify_all();
    if (p->thread.joinable()) p->thread.join();
    if (p->stream) { (void)hipStreamSynchronize(p->stream); (void)hipStreamDestroy(p->stream); }
    for (hipEvent_t e : p->events) (void)hipEventDestroy(e);
    if (p->shared) (void)hipHostFree(p->shared);
    delete p;
}

int get_port(Ctx* c, Port** out)
{
    if (c->port) { *out = c->port; return MSX_OK; }
    Port* p = new Port();
    p->device = c->device;
    p->sem = c->d.sem;
    bool ok = hipHostMalloc((void**)&p->shared, sizeof(PortShared), hipHostMallocMapped) == hipSuccess;
    if (ok) memset(p->shared, 0, sizeof(PortShared));
    ok = ok && hipHostGetDevicePointer((void**)&p->shared_dev, p->shared, 0) == hipSuccess &&
         hipStreamCreateWithFlags(&p->stream, hipStreamNonBlocking) == hipSuccess;
    for (int k = 0; ok && k < 64; ++k) {
        hipEvent_t e;
        ok = hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
        if (ok) p->events.push_back(e);
    }
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        for (hipEvent_t e : p->events) (void)hipEventDestroy(e);
        if (p->stream) (void)hipStreamDestroy(p->stream);
        if (p->shared) (void)hipHostFree(p->shared);
        delete p;
        return MSX_ERR_NOMEM;
    }
    p->thread = std::thread(port_proxy, p);
    c->port = p;
    *out = p;
    return MSX_OK;
}

// tell the proxy that a launch is about to push `requests` requests
void port_announce(Port* p, unsigned long long requests)
{
    {
        std::lock_guard<std::mutex> pl(p->mu);
        p->announced += requests;
    }
    p->cv.notify_all();
}

std::vector<Ctx*> g_made;         // contexts made by msx_ctx_create, any device
std::vector<MoePlan*> g_plans;    // routing plans made by msx_moe_plan_create

int destroy_ctx(Ctx* c)
{
    if (!c) return MSX_OK;
    (void)hipDeviceSynchronize();
    destroy_port(c->port);
    for (size_t i = 0; i < g_plans.size();) {        // plans die with their context
        if (g_plans[i]->owner != c) { ++i; continue; }
        if (g_plans[i]->slots) (void)hipFree(g_plans[i]->slots);
        if (g_plans[i]->base) (void)hipFree(g_plans[i]->base);
        delete g_plans[i];
        g_plans.erase(g_plans.begin() + (long)i);
    }
    if (c->latch) (void)hipHostFree(c->latch);
    if (c->d.sem) (void)hipFree(c->d.sem);
    if (c->d.expected) (void)hipFree(c->d.expected);
    if (c->d.status) (void)hipFree(c->d.status);
    if (c->d.call_state) (void)hipFree(c->d.call_state);
    if (c->d.gbar) (void)hipFree(c->d.gbar);
    if (c->d.ll) (void)hipFree(c->d.ll);
    if (c->moe.slots) (void)hipFree(c->moe.slots);
    if (c->ring) (void)hipFree(c->ring);
    for (auto& p : c->plans) (void)hipFree(p.ops);
    if (c->moe.base) (void)hipFree(c->moe.base);
    if (c->snap) (void)hipFree(c->snap);
    delete c;
    return MSX_OK;
}

// A new context on the current device (blocks: allocates and clears its device memory).  ll_max = largest
// per-rank message its LL scratch is sized for.  Caller holds g_mu.
int make_ctx(size_t ll_max, Ctx** out)
{
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MSX_ERR_ARG;
    Ctx* c = new Ctx();
    c->moe.owner = c;
    c->device = dev;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) { delete c; return hip_fail(e); }
    c->cus = prop.multiProcessorCount;
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
        c->ns_per_tick = 1.0e6 / (double)khz;

    const size_t sem_bytes = (size_t)kMaxRanks * kMaxRanks * kMaxChannels * kSemStrideWords * 4;
    const size_t exp_bytes = (size_t)kMaxRanks * kMaxRanks * kMaxChannels * 4;
    // one rotation half holds either 1PA's n slots of P packets (P <= ll_max/4/8) or 2PA's
    // 2 phases x n slots of ceil(P/n) packets (P <= ll_max/8): both at most 4*ll_max (+ slack)
    if (ll_max < 4096) ll_max = 4096;
    if (ll_max > (16u << 20)) ll_max = 16u << 20;
    const size_t rot = 4 * ll_max + 4096;
    const size_t rank_stride = 2 * rot;
    const size_t ll_bytes = rank_stride * kMaxRanks;
    c->ll_limit = ll_max;

    bool ok = hipMalloc((void**)&c->d.sem, sem_bytes) == hipSuccess &&
              hipMalloc((void**)&c->d.expected, exp_bytes) == hipSuccess &&
              hipMalloc((void**)&c->d.status, 64) == hipSuccess &&
              hipMalloc((void**)&c->d.call_state, 64) == hipSuccess &&
              hipMalloc((void**)&c->d.gbar, kGridBarBytes) == hipSuccess &&
              hipMalloc((void**)&c->d.ll, ll_bytes) == hipSuccess &&
              hipMalloc((void**)&c->moe.base, 64 * 4) == hipSuccess &&
              hipMalloc((void**)&c->snap, 4096) == hipSuccess &&
              hipHostMalloc((void**)&c->latch, 64, hipHostMallocMapped) == hipSuccess;
    if (ok) {
        *c->latch = 0u;
        ok = hipHostGetDevicePointer((void**)&c->d.latch, c->latch, 0) == hipSuccess;
    }
    ok = ok && hipMemset(c->d.sem, 0, sem_bytes) == hipSuccess &&
         hipMemset(c->d.expected, 0, exp_bytes) == hipSuccess &&
         hipMemset(c->d.status, 0, 64) == hipSuccess &&
         hipMemset(c->d.call_state, 0, 64) == hipSuccess &&
         hipMemset(c->d.gbar, 0, kGridBarBytes) == hipSuccess &&
         hipMemset(c->d.ll, 0, ll_bytes) == hipSuccess &&
         hipMemset(c->moe.base, 0, 64 * 4) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (!ok) { destroy_ctx(c); t_hip_err = (int)hipErrorOutOfMemory; return MSX_ERR_NOMEM; }
    c->d.ll_bytes = (unsigned)ll_bytes;
    c->d.ll_rank_stride = (unsigned)rank_stride;
    c->d.ll_rot_stride = (unsigned)rot;
    *out = c;
    return MSX_OK;
}

thread_local Ctx* t_use = nullptr;      // msx_ctx_use: the context this thread's calls run on (null: the default one)

bool known_ctx(const Ctx* c)
{
    for (const Ctx* k : g_made)
        if (k == c) return true;
    return false;
}

// The default context of the current device, created on first use.  Caller holds g_mu.
int default_ctx(Ctx** out)
{
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MSX_ERR_ARG;
    if (!g_ctx[dev]) {
        int rc = make_ctx(g_opt.ll_max_bytes, &g_ctx[dev]);
        if (rc) return rc;
    }
    *out = g_ctx[dev];
    return MSX_OK;
}

// A timeout a kernel of this context has run into and nobody has read yet (msx_status / msx_last_status read
// and clear it, a reset clears it): until then the context launches nothing more.
int latched(const Ctx* c)
{
    return c->latch && __atomic_load_n(c->latch, __ATOMIC_RELAXED) != 0u ? MSX_ERR_TIMEOUT : MSX_OK;
}

// The context this thread's next call runs on: the one chosen with msx_ctx_use, else the device's default.
// launching = the caller is about to enqueue kernels (refused while a timeout is latched).  Caller holds g_mu.
int get_ctx(Ctx** out, bool launching = true)
{
    Ctx* c = t_use;
    if (c) {
        int dev = -1;
        HIPCHK(hipGetDevice(&dev));
        if (!known_ctx(c) || c->device != dev) return MSX_ERR_ARG;
    } else {
        int rc = default_ctx(&c);
        if (rc) return rc;
    }
    if (launching) {
        int rc = latched(c);
        if (rc) return rc;
    }
    *out = c;
    return MSX_OK;
}

// ---- the context that lives in a file-scope device array ---------------------------------------
// For callers that must not allocate (msx_allreduce_ex_static): semaphores, expected values, status,
// call state, the chip-wide barrier's counters and a small LL scratch, carved out of one array that
// every GPU the library runs on holds until the process ends.  In host code the array's name only
// stands for the symbol; its address on a device comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticLlMax = (size_t)64 << 10;                       // LL algorithms: bytes per rank
constexpr size_t kStaticMaxBytes = (size_t)16 << 20;                    // any algorithm: bytes per rank
constexpr size_t kStaticSemBytes = (size_t)kMaxRanks * kMaxRanks * kMaxChannels * kSemStrideWords * 4;
constexpr size_t kStaticExpBytes = (size_t)kMaxRanks * kMaxRanks * kMaxChannels * 4;
constexpr size_t kStaticRot = 4 * kStaticLlMax + 4096;
constexpr size_t kStaticLlBytes = 2 * kStaticRot * kMaxRanks;
constexpr size_t kStaticOffExp = kStaticSemBytes;
constexpr size_t kStaticOffStatus = kStaticOffExp + kStaticExpBytes;
constexpr size_t kStaticOffCall = kStaticOffStatus + 256;
constexpr size_t kStaticOffGbar = kStaticOffCall + 256;
constexpr size_t kStaticOffLl = kStaticOffGbar + ((kGridBarBytes + 255) / 256) * 256;
constexpr size_t kStaticBytes = kStaticOffLl + kStaticLlBytes;          // about 6.2 MiB
static_assert(kStaticBytes % 16 == 0, "cleared in 16-byte vectors");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

__global__ __launch_bounds__(256) void k_clear(u32x4* p, size_t nvec)
{
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

Ctx* g_static[64] = {};

// The current device's fixed context; set up on first use (msx_init does it).  Caller holds g_mu.  Set-up
// clears the array with a kernel on the null stream and waits for it, so it cannot happen while `stream` is
// being captured: such a caller has to run msx_init first.
int get_static_ctx(hipStream_t stream, Ctx** out)
{
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MSX_ERR_ARG;
    if (g_static[dev]) { *out = g_static[dev]; return MSX_OK; }
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (stream && hipStreamIsCapturing(stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
        return MSX_ERR_UNSUPPORTED;
    unsigned char* ptr = nullptr;
    HIPCHK(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return MSX_ERR_HIP;
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, dev));
    hipLaunchKernelGGL(k_clear, dim3(256), dim3(256), 0, nullptr, (u32x4*)ptr, kStaticBytes / 16);
    HIPCHK(hipGetLastError());
    HIPCHK(hipDeviceSynchronize());
    Ctx* c = new Ctx();
    c->device = dev;
    c->fixed = true;
    c->cus = prop.multiProcessorCount;
    c->d.sem = (unsigned*)ptr;
    c->d.expected = (unsigned*)(ptr + kStaticOffExp);
    c->d.status = (unsigned*)(ptr + kStaticOffStatus);
    c->d.call_state = (unsigned*)(ptr + kStaticOffCall);
    c->d.gbar = (unsigned*)(ptr + kStaticOffGbar);
    c->d.ll = ptr + kStaticOffLl;
    c->d.ll_bytes = (unsigned)kStaticLlBytes;
    c->d.ll_rank_stride = (unsigned)(2 * kStaticRot);
    c->d.ll_rot_stride = (unsigned)kStaticRot;
    c->ll_limit = kStaticLlMax;
    g_static[dev] = c;
    *out = c;
    return MSX_OK;
}

// kernel-argument copy of the device context with the current test hooks applied
DevCtx dev_ctx(const Ctx* c)
{
    DevCtx d = c->d;
    d.spin_limit = g_opt.spin_limit;
    d.drop_rank = g_opt.drop_rank;
    d.chaos = g_opt.chaos;
    return d;
}

// how many workgroups of `threads` threads of kernel k can be resident on the whole GPU
int resident_blocks(Ctx* c, const void* k, int threads, int* out)
{
    auto key = std::make_pair(k, threads);
    auto it = c->occ.find(key);
    int per_cu = 0;
    if (it == c->occ.end()) {
        HIPCHK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, threads, 0));
        c->occ[key] = per_cu;
    } else {
        per_cu = it->second;
    }
    *out = per_cu * c->cus;
    if (c->max_blocks > 0 && *out > c->max_blocks) *out = c->max_blocks;
    return MSX_OK;
}

// channels (workgroups per rank) for `work` items per rank handled `per_thread` at a time
// A cap on workgroups per rank that was found with 8 ranks, as a total over the chip shared out over n ranks.
int per_rank_cap(int total, int n) { return std::min(kMaxChannels, std::max(1, total / std::max(1, n))); }

int pick_channels(Ctx* c, const void* k, int threads, int n, size_t work, size_t per_thread, int want,
                  int cap, int* chans)
{
    int resident = 0;
    int rc = resident_blocks(c, k, threads, &resident);
    if (rc) return rc;
    int limit = resident / n;
    if (limit > kMaxChannels) limit = kMaxChannels;
    if (limit < 1) return MSX_ERR_UNSUPPORTED;
    int ch = want;
    if (ch <= 0) {
        const size_t per_block = (size_t)threads * per_thread;
        size_t need = (work + per_block - 1) / per_block;
        if (need < 1) need = 1;
        ch = need > (size_t)cap ? cap : (int)need;
    }
    if (ch > limit) ch = limit;
    *chans = ch;
    return MSX_OK;
}

int check_common(int dtype, int op, int nranks)
{
    if (dtype != MSX_F32 && dtype != MSX_BF16 && dtype != MSX_F16 && dtype != MSX_I32) return MSX_ERR_ARG;
    if (op != MSX_SUM && op != MSX_MAX && op != MSX_MIN) return MSX_ERR_UNSUPPORTED;
    if (nranks < 1 || nranks > kMaxRanks) return MSX_ERR_ARG;
    return MSX_OK;
}

int check_table(const void* const* t, int n)
{
    if (!t) return MSX_ERR_ARG;
    for (int i = 0; i < n; ++i)
        if (!t[i] || !aligned16(t[i])) return MSX_ERR_ARG;
    return MSX_OK;
}

void note_launch(int grid, int block, int algo) { t_grid = grid; t_block = block; t_algo = algo; }

// A prepared call: everything a collective does on the host (checks, algorithm and launch shape, argument
// blocks, scratch) done once; running it only enqueues the kernels.  Scratch a prepared call needs beyond the
// context's fixed parts (ring scratch, a lowered plan) belongs to it and is freed with it.
constexpr unsigned kPreparedMagic = 0x6d737850u;
struct Prepared {
    unsigned magic = kPreparedMagic;
    Ctx* ctx = nullptr;
    std::vector<std::function<hipError_t(hipStream_t)>> steps;
    std::vector<void*> owned;      // device allocations of this call
    int grid = 0, block = 0, algo = 0;
};
std::vector<Prepared*> g_prepared;
thread_local Prepared* t_record = nullptr;   // set while a msx_prepare_* call runs the ordinary host path

template <typename K, typename... A>
int launch(K k, int grid, int block, hipStream_t s, A... args)
{
    if (grid <= 0 || block <= 0) return MSX_ERR_ARG;
    if (t_record) {
        t_record->steps.push_back([=](hipStream_t st) {
            hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3((unsigned)block), 0, st, args...);
            return hipGetLastError();
        });
        return MSX_OK;
    }
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3((unsigned)block), 0, s, args...);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return MSX_OK;
}

// ---- AllReduce ------------------------------------------------------------------------------

typedef void (*HbKernel)(HbArgs, DevCtx);
typedef void (*LlKernel)(LlArgs, DevCtx);

HbKernel hb_fused_kernel(int dt, int u, int n, int res, int cache)
{
#define MSX_N(DT, U, RES) (n == 8 ? (HbKernel)k_allreduce_hb_fused<DT, U, 8, RES> : (HbKernel)k_allreduce_hb_fused<DT, U, 0, RES>)
#define MSX_R(DT, U) (res == 0 ? MSX_N(DT, U, 0) : res == 1 ? MSX_N(DT, U, 1) : MSX_N(DT, U, 2))
    // cache-keeping forms: 8 ranks, the unrolls the automatic choice uses
#define MSX_C(DT, U, RES) (cache == 1 ? (HbKernel)k_allreduce_hb_fused<DT, U, 8, RES, 1> : (HbKernel)k_allreduce_hb_fused<DT, U, 8, RES, 2>)
#define MSX_CR(DT, U) (res == 0 ? MSX_C(DT, U, 0) : res == 1 ? MSX_C(DT, U, 1) : MSX_C(DT, U, 2))
    if (cache != 0 && n == 8 && (u == 1 || u == 2)) {
        if (dt == MSX_F32) return u == 2 ? MSX_CR(0, 2) : MSX_CR(0, 1);
        return u == 2 ? MSX_CR(1, 2) : MSX_CR(1, 1);
    }
    if (dt == MSX_F32) return u >= 4 ? MSX_R(0, 4) : u == 2 ? MSX_R(0, 2) : MSX_R(0, 1);
    return u >= 4 ? MSX_R(1, 4) : u == 2 ? MSX_R(1, 2) : MSX_R(1, 1);
#undef MSX_CR
#undef MSX_C
#undef MSX_R
#undef MSX_N
}
// does a fused HB AllReduce of nbytes per rank run in chip-wide phases?  (res_mode 2, one residual per
// destination, would need loads in the write phase)
// The automatic choice starts at 40 MiB per rank (rows, for the reduce-scatter and the all-gather) with 8 ranks;
// measured against the free-running kernels, TB/s: AllReduce 32 MiB 5.3 / 5.6-5.9, 40 MiB 5.6 / 4.9, 48 MiB
// 5.9 / 5.0, 64 MiB 6.0-6.2 / 5.2; AllGather 32 MiB 5.2 / 5.5, 40 MiB 5.3 / 4.75, 64 MiB 6.0 / 4.5;
// ReduceScatter 32 MiB 4.3 / 4.35, 40 MiB 4.7 / 4.6, 64 MiB 5.55 / 4.9.
// Other rank counts (AllReduce without a residual only: the kernels with the rank count as a template argument),
// phased / free-running TB/s at 64 MiB and 256 MiB per rank: 3 ranks 4.55 / 4.8 and 5.75 / 5.25; 4 ranks 5.0 / 4.6
// and 6.15 / 5.1 (1 GiB 5.7 / 5.25); 5 ranks 5.3 / 4.8 and 6.2 / 4.9; 6 ranks 5.3 / 4.75 and 5.75 / 5.05; 7 ranks
// 5.4 / 4.8 and 6.1 / 4.95.  So: 4 to 7 ranks from 64 MiB, 3 ranks from 128 MiB.  Two ranks: 4.0 / 3.7, 5.4 / 5.25,
// 5.2 / 5.6 (1 GiB) - no clear gain, left to the free-running kernel.
// AllGather with other rank counts (its phased kernel takes the rank count at run time), phased / free-running
// TB/s by row size: 4 ranks 64 MiB 5.55 / 5.4, 128 MiB 6.0 / 4.6, 256 MiB 6.2 / 4.8, 1 GiB 5.6 / 5.1; 6 ranks 64 MiB
// 4.8 / 4.4, 128 MiB 5.7 / 4.7, 256 MiB 5.9 / 4.8; 3, 5, 7 ranks at 256 MiB 5.3 / 4.8, 5.7 / 4.7, 5.6 / 4.7; 2 ranks
// 128 MiB 4.95 / 5.7, 256 MiB 5.6 / 5.25, 1 GiB 5.35 / 5.25.  So: 3 to 7 ranks from 128 MiB rows, 2 ranks from 256 MiB.
// The ReduceScatter of other rank counts stays free-running (5.6 against 5.2 TB/s at 4 ranks, 4.1 / 3.8 at 2).
enum PhasedKind { kPhasedOther = 0, kPhasedAllReduce = 1, kPhasedAllGather = 2 };
bool use_phased(size_t nbytes, int n, int res_mode, int kind = kPhasedOther)
{
    if (n < 2 || res_mode == 2 || g_opt.hb_unroll != 0) return false;
    if (g_opt.hb_phased_min >= 0) return nbytes >= (size_t)g_opt.hb_phased_min;
    if (n == 8) return nbytes >= ((size_t)40 << 20);
    if (kind == kPhasedAllGather) return nbytes >= ((size_t)(n == 2 ? 256 : 128) << 20);
    if (kind != kPhasedAllReduce || res_mode != 0 || n < 3) return false;
    return nbytes >= ((size_t)(n == 3 ? 128 : 64) << 20);
}
HbKernel hb_2phase_kernel(int dt, int u, int n)
{
#define MSX_ROW(DT, U) (n == 8 ? (HbKernel)k_allreduce_hb_2phase<DT, U, 8> : (HbKernel)k_allreduce_hb_2phase<DT, U, 0>)
    if (dt == MSX_F32) return u >= 2 ? MSX_ROW(0, 2) : MSX_ROW(0, 1);
    return u >= 2 ? MSX_ROW(1, 2) : MSX_ROW(1, 1);
#undef MSX_ROW
}
LlKernel ll_1pa_kernel(int dt, int n)
{
    if (dt == MSX_F32) return n == 8 ? (LlKernel)k_allreduce_1pa_ll<0, 8> : (LlKernel)k_allreduce_1pa_ll<0, 0>;
    return n == 8 ? (LlKernel)k_allreduce_1pa_ll<1, 8> : (LlKernel)k_allreduce_1pa_ll<1, 0>;
}
LlKernel ll_2pa_kernel(int dt, int n)
{
    if (dt == MSX_F32) return n == 8 ? (LlKernel)k_allreduce_2pa_ll<0, 8> : (LlKernel)k_allreduce_2pa_ll<0, 0>;
    return n == 8 ? (LlKernel)k_allreduce_2pa_ll<1, 8> : (LlKernel)k_allreduce_2pa_ll<1, 0>;
}

int ll_block_threads(size_t work)
{
    if (g_opt.threads > 0) {
        int t = (g_opt.threads + 63) / 64 * 64;
        return t > 1024 ? 1024 : t;
    }
    size_t t = (work + 63) / 64 * 64;
    if (t < 64) t = 64;
    if (t > 512) t = 512;
    return (int)t;
}


// ---- host-side choices (pure functions of sizes and options; no device needed) -------------------------

// which algorithm the automatic choice runs for nbytes per rank; ll_limit = what the LL scratch holds
int choose_algo(size_t nbytes, int n, size_t ll_limit)
{
    if (n == 1) return MSX_ALGO_2PA_HB;
    if (nbytes <= g_opt.ll_1pa_max && nbytes <= ll_limit / 4) return MSX_ALGO_1PA_LL;
    if (nbytes <= g_opt.ll_2pa_max && nbytes <= ll_limit) return MSX_ALGO_2PA_LL;
    return MSX_ALGO_2PA_HB;
}

// launch shape of the HB AllReduce kernels: unroll and wanted workgroups per rank (before the
// co-residency clamp).  Small messages: every thread issues all its loads at once, one pass;
// large ones: many plain workgroups.
void choose_hb_shape(size_t nbytes, int n, int threads, int* unroll, int* want)
{
    const size_t per_rank = (nbytes / 16 + (size_t)n - 1) / (size_t)n;
    int U = g_opt.hb_unroll, w = g_opt.hb_blocks;
    // up to 2 MiB per rank: one vector per thread in a single pass (more, smaller workgroups: 4.2-4.6 us
    // instead of 5.0-5.2 us at 64-512 KiB); up to 4 MiB: two vectors per thread
    if (U == 0) U = per_rank <= 16384 ? 1 : per_rank <= 32768 ? 2 : 1;
    if (w == 0) {
        if (per_rank <= 32768) w = (int)((per_rank + (size_t)threads * U - 1) / ((size_t)threads * U));
        else if (per_rank <= 262144) w = 32;   // up to 4 MiB of chunk per rank
        else {                                 // about 1024 workgroups in all, whatever the rank count
            w = 1024 / n;
            if (w > kMaxChannels) w = kMaxChannels;
        }
        if (w < 1) w = 1;
    }
    *unroll = U;
    *want = w;
}

// Cache hints of the fused HB AllReduce by footprint (inputs + outputs of all ranks), from a sweep: up to
// 64 MiB everything may stay cached, up to 512 MiB (the outputs then just fill the 256 MiB memory-side cache)
// the stores may, beyond that both stream.
int choose_cache_mode(size_t nbytes, int n, int res_mode)
{
    if (g_opt.cache_mode >= 0) return g_opt.cache_mode;
    const size_t footprint = (2 * (size_t)n + (res_mode == 0 ? 0 : res_mode == 1 ? 1 : (size_t)n)) * nbytes;
    if (footprint <= ((size_t)64 << 20)) return 2;
    if (footprint <= ((size_t)512 << 20)) return 1;
    return 0;
}

// ---- lowering of an AllReduce to an execution plan (the host half of the Executor analogue) ------------

PlanOp plan_op(int code, int peer = 0, int flags = 0)
{
    PlanOp o{};
    o.code = code;
    o.peer = peer;
    o.flags = flags;
    return o;
}

PlanOp plan_reduce_put(std::vector<PlanRef> src, std::vector<PlanRef> dst, int dst_wt, size_t first, size_t end,
                       size_t step)
{
    PlanOp o{};
    o.code = kOpReducePut;
    o.nsrc = (int)src.size();
    o.ndst = (int)dst.size();
    for (size_t k = 0; k < src.size(); ++k) o.src[k] = src[k];
    for (size_t k = 0; k < dst.size(); ++k) o.dst[k] = dst[k];
    o.dst_wt = dst_wt;
    o.first = first;
    o.end = end;
    o.step = step;
    return o;
}

// Ring scratch of `need` bytes: the context's own (grown on demand, which waits for the device), or, for a
// prepared call, an allocation that call owns.
int ring_scratch(Ctx* c, size_t need, void** out)
{
    if (t_record) {
        void* p = nullptr;
        if (hipMalloc(&p, need) != hipSuccess) return MSX_ERR_NOMEM;
        t_record->owned.push_back(p);
        *out = p;
        return MSX_OK;
    }
    if (need > c->ring_bytes) {
        HIPCHK(hipDeviceSynchronize());
        if (c->ring) { HIPCHK(hipFree(c->ring)); c->ring = nullptr; c->ring_bytes = 0; }
        if (hipMalloc(&c->ring, need) != hipSuccess) return MSX_ERR_NOMEM;
        c->ring_bytes = need;
    }
    *out = c->ring;
    return MSX_OK;
}

constexpr size_t kPlanCacheMax = 16;     // lowered plans a context keeps; the oldest goes first

bool plan_algo(int algo)
{
    return algo == MSX_ALGO_PLAN_2PA_HB || algo == MSX_ALGO_PLAN_2PR_HB || algo == MSX_ALGO_PLAN_1PA_LL ||
           algo == MSX_ALGO_PLAN_2PA_LL;
}

// Same steps as the hand-written kernels, written as data: k_allreduce_hb_fused (held == 0) or
// k_allreduce_hb_phased (held = sums a thread holds per phase), k_allreduce_ring, k_allreduce_1pa_ll,
// k_allreduce_2pa_ll.  nbytes = bytes per rank; the HB plans need whole 16-byte vectors split evenly.
void lower_allreduce(int algo, int n, int chans, size_t nbytes, int threads, int held, std::vector<PlanOp>* ops,
                     std::vector<unsigned>* start)
{
    start->assign((size_t)n * chans, 0);   // one more entry (the total) is appended at the end
    const size_t nvec = nbytes / 16, cv = nvec / (size_t)n;
    const size_t P = (nbytes + 7) / 8, cp = (P + (size_t)n - 1) / (size_t)n;     // LL: packets per rank / per chunk
    for (int b = 0; b < n * chans; ++b) {
        const int rank = b % n, chan = b / n;
        (*start)[b] = (unsigned)ops->size();
        const short r = (short)rank;
        const int peers = ((1 << n) - 1) & ~(1 << rank);
        if (algo == MSX_ALGO_PLAN_1PA_LL || algo == MSX_ALGO_PLAN_2PA_LL) {
            const bool one = algo == MSX_ALGO_PLAN_1PA_LL;
            const size_t range = one ? P : cp;
            auto packet_op = [&](int code, int to, unsigned chunk_stride, unsigned region) {
                PlanOp o = plan_op(code, rank);
                o.nsrc = o.ndst = 1;
                o.src[0] = PlanRef{kBufIn, r};
                o.dst[0] = PlanRef{kBufOut, r};
                o.dst_wt = to;
                o.aux = (unsigned)(range * 16);
                o.aux2 = chunk_stride;
                o.aux3 = region;
                o.first = (size_t)chan * threads;
                o.end = range;
                o.step = (size_t)chans * threads;
                return o;
            };
            ops->push_back(packet_op(kOpPutPacket, peers, one ? 0u : (unsigned)cp, 0u));
            ops->push_back(packet_op(kOpReducePacket, one ? 0 : peers, one ? 0u : (unsigned)(rank * cp), 0u));
            if (!one) ops->push_back(packet_op(kOpCopyPacket, 0, (unsigned)cp, (unsigned)((size_t)n * cp * 16)));
        } else if (algo == MSX_ALGO_PLAN_2PA_HB) {
            std::vector<PlanRef> src, dst;
            for (short j = 0; j < n; ++j) { src.push_back({kBufIn, j}); dst.push_back({kBufOut, j}); }
            ops->push_back(plan_op(kOpBarrier));
            if (held == 0) {
                ops->push_back(plan_reduce_put(src, dst, (1 << n) - 1, (size_t)rank * cv + (size_t)chan * threads,
                                               (size_t)(rank + 1) * cv, (size_t)chans * threads));
            } else {
                // rounds of a chip-wide read phase and a chip-wide write phase; tiles of `threads` vectors dealt
                // out one by one over the rank's workgroups; every workgroup takes part in every barrier
                const size_t tiles = cv / (size_t)threads, per_round = (size_t)chans * held;
                const size_t rounds = (tiles + per_round - 1) / per_round;
                for (size_t round = 0; round < rounds; ++round) {
                    const size_t first = round * per_round + (size_t)chan;
                    const size_t left = first >= tiles ? 0 : (tiles - first + (size_t)chans - 1) / (size_t)chans;
                    const unsigned mine = (unsigned)(left < (size_t)held ? left : (size_t)held);
                    PlanOp rd = plan_reduce_put(src, dst, (1 << n) - 1, (size_t)rank * cv + first * threads, 0,
                                                (size_t)chans * threads);
                    rd.code = kOpReduceHold;
                    rd.aux = mine;
                    PlanOp wr = rd;
                    wr.code = kOpPutHeld;
                    ops->push_back(rd);
                    ops->push_back(plan_op(kOpGridBarrier, 0, 2));
                    ops->push_back(wr);
                    ops->push_back(plan_op(kOpDrain));
                    ops->push_back(plan_op(kOpGridBarrier, 0, 1));
                }
                if (chan == 0 && tiles * threads < cv)      // what is left behind the chunk's last whole tile
                    ops->push_back(plan_reduce_put(src, dst, (1 << n) - 1, (size_t)rank * cv + tiles * threads,
                                                   (size_t)(rank + 1) * cv, (size_t)threads));
            }
            ops->push_back(plan_op(kOpDrain));
            ops->push_back(plan_op(kOpBarrier));
        } else {
            const short next = (short)((rank + 1) % n), prev = (short)((rank + n - 1) % n);
            const size_t lo = cv * (size_t)chan / (size_t)chans, hi = cv * (size_t)(chan + 1) / (size_t)chans;
            auto range = [&](int chunk, std::vector<PlanRef> s, std::vector<PlanRef> d, int wt) {
                return plan_reduce_put(s, d, wt, (size_t)chunk * cv + lo, (size_t)chunk * cv + hi, (size_t)threads);
            };
            ops->push_back(plan_op(kOpBarrier));
            ops->push_back(range(rank, {{kBufIn, r}}, {{kBufScratch, next}}, 1));
            ops->push_back(plan_op(kOpDrain));
            ops->push_back(plan_op(kOpSignal, next));
            for (int s = 0; s + 1 < n; ++s) {
                const int j = (rank - 1 - s + 2 * n) % n;
                ops->push_back(plan_op(kOpWait, prev, 2));
                if (s + 2 == n) ops->push_back(range(j, {{kBufScratch, r}, {kBufIn, r}}, {{kBufOut, r}, {kBufOut, next}}, 2));
                else ops->push_back(range(j, {{kBufScratch, r}, {kBufIn, r}}, {{kBufScratch, next}}, 1));
                ops->push_back(plan_op(kOpDrain));
                ops->push_back(plan_op(kOpSignal, next));
            }
            for (int s = 0; s + 1 < n; ++s) {
                const int j = (rank - s + n) % n;
                ops->push_back(plan_op(kOpWait, prev, 2));
                if (s + 2 < n) {
                    ops->push_back(range(j, {{kBufOut, r}}, {{kBufOut, next}}, 1));
                    ops->push_back(plan_op(kOpDrain));
                    ops->push_back(plan_op(kOpSignal, next));
                }
            }
        }
        ops->push_back(plan_op(kOpEnd));
    }
    start->push_back((unsigned)ops->size());
}

// The lists as the interpreter reads them: every workgroup's at a fixed stride, padded with end marks; a rank
// barrier that every list begins with is taken out (the kernel runs it while the list is on its way) and
// described by *head (bit 0: there is one; bits 1, 2: its flags); a drain right in front of a barrier or a
// signal becomes a flag of that operation (kPlanDrainFirst): one step of the interpreter less per hand-off.
void pack_plan(const std::vector<PlanOp>& ops, const std::vector<unsigned>& start, std::vector<PlanOp>* packed,
               unsigned* stride, int* head)
{
    const size_t lists = start.size() - 1;
    bool common = lists > 0;
    for (size_t b = 0; b < lists && common; ++b) {
        const PlanOp& o = ops[start[b]];
        common = start[b + 1] - start[b] > 1 && o.code == kOpBarrier && o.flags == ops[start[0]].flags;
    }
    *head = common ? 1 | (ops[start[0]].flags << 1) : 0;
    const unsigned skip = common ? 1u : 0u;
    std::vector<std::vector<PlanOp>> fused(lists);
    unsigned longest = 1;
    for (size_t b = 0; b < lists; ++b) {
        for (unsigned k = start[b] + skip; k < start[b + 1]; ++k) {
            PlanOp o = ops[k];
            if (o.code == kOpDrain && k + 1 < start[b + 1] && (ops[k + 1].code == kOpBarrier || ops[k + 1].code == kOpSignal)) {
                o = ops[++k];
                o.flags |= kPlanDrainFirst;
            }
            fused[b].push_back(o);
        }
        longest = std::max(longest, (unsigned)fused[b].size());
    }
    *stride = longest;
    packed->assign(lists * longest, plan_op(kOpEnd));
    for (size_t b = 0; b < lists; ++b)
        for (size_t k = 0; k < fused[b].size(); ++k) (*packed)[b * longest + k] = fused[b][k];
}

int plan_allreduce(Ctx* c, const void* const* send, void* const* recv, size_t nbytes, int dtype, int n, int algo,
                   hipStream_t stream)
{
    const bool ring = algo == MSX_ALGO_PLAN_2PR_HB;
    const bool packets = algo == MSX_ALGO_PLAN_1PA_LL || algo == MSX_ALGO_PLAN_2PA_LL;
    const int threads = 256;
    int chans = 1, rc, held = 0;
    // one instantiation per operation family (channel operations / packet operations)
    const void* kp = packets ? (n == 8 ? (dtype == MSX_F32 ? (const void*)k_plan_executor<0, 0, 1, 8> : (const void*)k_plan_executor<1, 0, 1, 8>)
                                       : (dtype == MSX_F32 ? (const void*)k_plan_executor<0, 0, 1, 0> : (const void*)k_plan_executor<1, 0, 1, 0>))
                             : (dtype == MSX_F32 ? (const void*)k_plan_executor<0, 0, 0> : (const void*)k_plan_executor<1, 0, 0>);
    if (packets) {
        if (nbytes % 2) return MSX_ERR_UNSUPPORTED;
        const size_t P = (nbytes + 7) / 8, cp = (P + (size_t)n - 1) / (size_t)n;
        const size_t need = algo == MSX_ALGO_PLAN_1PA_LL ? (size_t)n * P * 16 : 2 * (size_t)n * cp * 16;
        if (need > c->d.ll_rot_stride) return MSX_ERR_NOMEM;
        const size_t work = algo == MSX_ALGO_PLAN_1PA_LL ? P : cp;
        if ((rc = pick_channels(c, kp, threads, n, work, 1, g_opt.ll_blocks, 64, &chans))) return rc;
    } else {
        if (nbytes % (16 * (size_t)n)) return MSX_ERR_UNSUPPORTED;
        const size_t per_rank = nbytes / 16 / (size_t)n;
        int want = g_opt.hb_blocks, unroll_unused = 1;
        if (!ring) choose_hb_shape(nbytes, n, threads, &unroll_unused, &want);   // same shape as the hand kernel
        size_t per_thread = 4;
        int cap = ring ? 64 : kMaxChannels;
        if (!ring && n == 8 && use_phased(nbytes, n, 0)) {
            // very large messages: the read phase / write phase schedule, one workgroup per CU
            held = kPhasedHeld;
            kp = plan_executor_held(dtype == MSX_F32);
            want = g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels;
            per_thread = (size_t)held;
        }
        if ((rc = pick_channels(c, kp, threads, n, per_rank, per_thread, want, cap, &chans))) return rc;
    }
    void* ring_mem = nullptr;
    if (ring && (rc = ring_scratch(c, nbytes * (size_t)n, &ring_mem))) return rc;
    Ctx::Plan found{algo, n, chans, held, nbytes, nullptr, 0u, 0};
    if (!t_record)
        for (const auto& p : c->plans)
            if (p.algo == algo && p.n == n && p.chans == chans && p.held == held && p.nbytes == nbytes) found = p;
    if (!found.ops) {
        std::vector<PlanOp> ops, packed;
        std::vector<unsigned> start;
        lower_allreduce(algo, n, chans, nbytes, threads, held, &ops, &start);
        pack_plan(ops, start, &packed, &found.stride, &found.head);
        for (const PlanOp& o : packed) {                 // the kernel chosen above carries one family only
            const bool pkt_op = o.code == kOpPutPacket || o.code == kOpReducePacket || o.code == kOpCopyPacket;
            const bool chan_op = o.code == kOpBarrier || o.code == kOpSignal || o.code == kOpWait || o.code == kOpReducePut ||
                                 o.code == kOpDrain;
            if ((packets && (chan_op || (found.head & 1))) || (!packets && pkt_op)) return MSX_ERR_UNSUPPORTED;
        }
        if (hipMalloc((void**)&found.ops, packed.size() * sizeof(PlanOp)) != hipSuccess) return MSX_ERR_NOMEM;
        if (t_record) {                                  // a prepared call keeps its plan for itself
            t_record->owned.push_back(found.ops);
        } else {
            if (c->plans.size() >= kPlanCacheMax) {      // a launch in flight may still be reading the oldest one
                HIPCHK(hipDeviceSynchronize());
                (void)hipFree(c->plans.front().ops);
                c->plans.erase(c->plans.begin());
            }
            c->plans.push_back(found);
        }
        HIPCHK(hipMemcpy(found.ops, packed.data(), packed.size() * sizeof(PlanOp), hipMemcpyHostToDevice));
    }
    PlanArgs a{};
    for (int i = 0; i < n; ++i) {
        a.in[i] = send[i];
        a.out[i] = recv[i];
        a.scratch[i] = ring ? (void*)((char*)ring_mem + (size_t)i * nbytes) : nullptr;
    }
    a.ops = found.ops;
    a.nbytes = nbytes;
    a.stride = found.stride;
    a.n = n;
    a.head = found.head;
    a.packets = packets ? 1 : 0;
    a.pace = g_opt.hb_pace;
    note_launch(n * chans, threads, algo);
    typedef void (*K)(PlanArgs, DevCtx);
    return launch((K)kp, n * chans, threads, stream, a, dev_ctx(c));
}

typedef void (*GenericKernel)(HbArgs, DevCtx, int, int);

GenericKernel generic_kernel(int dtype, int op)
{
#define MSX_G(DT) (op == MSX_SUM ? (GenericKernel)k_reduce_generic<DT, 0> : op == MSX_MAX ? (GenericKernel)k_reduce_generic<DT, 1> : (GenericKernel)k_reduce_generic<DT, 2>)
    return dtype == MSX_F32 ? MSX_G(0) : dtype == MSX_BF16 ? MSX_G(1) : dtype == MSX_F16 ? MSX_G(2) : MSX_G(3);
#undef MSX_G
}

// fp16 and max / min: the generic HB kernel.  mode 0 AllReduce (count = elements per rank),
// mode 1 ReduceScatter (count = elements per block).
int reduce_generic(Ctx* c, const void* const* in, void* const* out, size_t count, int dtype, int op, int n,
                   int mode, int vec, hipStream_t stream)
{
    GenericKernel k = generic_kernel(dtype, op);
    const size_t vecs = count * elem_size(dtype) / 16;
    const size_t per_rank = mode == 0 ? (vecs + (size_t)n - 1) / (size_t)n
                            : mode == 2 ? (count + (size_t)n - 1) / (size_t)n : (vec ? vecs : count);
    int chans = 1, rc;
    if ((rc = pick_channels(c, (const void*)k, 256, n, per_rank, 1, g_opt.hb_blocks, per_rank_cap(1024, n), &chans))) return rc;
    HbArgs a{};
    for (int i = 0; i < n; ++i) {
        a.in[i] = in[i];
        a.out[i] = out[i];
    }
    a.count = count;
    a.n = n;
    a.chans = chans;
    a.barriers = g_opt.hb_barriers;
    note_launch(n * chans, 256, MSX_ALGO_2PA_HB);
    return launch(k, n * chans, 256, stream, a, dev_ctx(c), mode, vec);
}

int allreduce_impl(const void* const* send, void* const* recv, const void* const* residual, size_t count,
                   int dtype, int op, int nranks, int algo, hipStream_t stream, bool fixed_ctx = false)
{
    int rc = check_common(dtype, op, nranks);
    if (rc) return rc;
    if (algo < MSX_ALGO_AUTO || algo > MSX_ALGO_2PR_PORT) return MSX_ERR_ARG;
    if ((rc = check_table(send, nranks))) return rc;
    if ((rc = check_table((const void* const*)recv, nranks))) return rc;
    if (residual && (rc = check_table(residual, nranks))) return rc;
    if (count == 0) return MSX_OK;
    const size_t nbytes = count * elem_size(dtype);

    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    if (fixed_ctx) {
        // nothing below may allocate: the ring's and the interpreter's scratch grow on demand, so they are out
        if (nbytes > kStaticMaxBytes) return MSX_ERR_NOMEM;
        if (algo == MSX_ALGO_2PR_HB || algo == MSX_ALGO_2PR_PORT || plan_algo(algo)) return MSX_ERR_UNSUPPORTED;
        if ((rc = get_static_ctx(stream, &c))) return rc;
    } else if ((rc = get_ctx(&c))) return rc;
    const int n = nranks;

    bool res_shared = residual != nullptr;
    if (residual)
        for (int i = 1; i < n; ++i) res_shared = res_shared && residual[i] == residual[0];

    if (dtype == MSX_F16 || dtype == MSX_I32 || op != MSX_SUM) {
        // outside the tuned paths: only the fused all-pairs HB form exists
        if (residual) return MSX_ERR_UNSUPPORTED;
        if (algo == MSX_ALGO_AUTO && !fixed_ctx) algo = g_opt.algo;
        if (algo != MSX_ALGO_AUTO && algo != MSX_ALGO_2PA_HB) return MSX_ERR_UNSUPPORTED;
        return reduce_generic(c, send, recv, count, dtype, op, n, 0, 1, stream);
    }

    if (algo == MSX_ALGO_AUTO && !fixed_ctx) algo = g_opt.algo;
    if (algo == MSX_ALGO_AUTO) algo = choose_algo(nbytes, n, c->ll_limit);

    if (algo == MSX_ALGO_1PA_LL || algo == MSX_ALGO_2PA_LL) {
        const size_t P = (nbytes + 7) / 8;
        const size_t cp = (P + (size_t)n - 1) / (size_t)n;
        const size_t need = algo == MSX_ALGO_1PA_LL ? (size_t)n * P * 16 : 2 * (size_t)n * cp * 16;
        if (need > c->d.ll_rot_stride) return MSX_ERR_NOMEM;
        const size_t work = algo == MSX_ALGO_1PA_LL ? P : cp;
        LlKernel k = algo == MSX_ALGO_1PA_LL ? ll_1pa_kernel(dtype, n) : ll_2pa_kernel(dtype, n);
        const int threads = ll_block_threads(work);
        int chans = 1;
        if ((rc = pick_channels(c, (const void*)k, threads, n, work, 1, g_opt.ll_blocks, 32, &chans))) return rc;
        LlArgs a{};
        for (int i = 0; i < n; ++i) {
            a.in[i] = send[i];
            a.out[i] = recv[i];
            a.res[i] = residual ? residual[i] : nullptr;
        }
        a.nbytes = nbytes;
        a.n = n;
        a.chans = chans;
        a.has_res = residual ? 1 : 0;
        a.res_shared = res_shared ? 1 : 0;
        note_launch(n * chans, threads, algo);
        return launch(k, n * chans, threads, stream, a, dev_ctx(c));
    }

    if (plan_algo(algo) && n > 1) {
        if (residual) return MSX_ERR_UNSUPPORTED;
        return plan_allreduce(c, send, recv, nbytes, dtype, n, algo, stream);
    }
    if (plan_algo(algo)) algo = MSX_ALGO_2PA_HB;
    if ((algo == MSX_ALGO_2PR_HB || algo == MSX_ALGO_2PR_PORT) && n == 1) algo = MSX_ALGO_2PA_HB;
    if (algo == MSX_ALGO_2PR_PORT) {
        // two-phase ring whose copies go through the port (FIFO, CPU proxy, runtime copies), overlapped with the
        // reduction: n equal chunks of whole 16-byte vectors, no residual.  The proxy is told of every launch,
        // so this is neither a call to prepare nor one to capture.
        if (residual) return MSX_ERR_UNSUPPORTED;
        if (nbytes % (16 * (size_t)n)) return MSX_ERR_UNSUPPORTED;
        if (t_record) return MSX_ERR_UNSUPPORTED;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (stream && hipStreamIsCapturing(stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
            return MSX_ERR_UNSUPPORTED;
        Port* port = nullptr;
        if ((rc = get_port(c, &port))) return rc;
        void* ring_mem = nullptr;
        if ((rc = ring_scratch(c, nbytes * (size_t)n, &ring_mem))) return rc;
        const void* kp = dtype == MSX_F32 ? (const void*)k_allreduce_ring_port<0> : (const void*)k_allreduce_ring_port<1>;
        RingArgs a{};
        for (int i = 0; i < n; ++i) {
            a.in[i] = send[i];
            a.out[i] = recv[i];
            a.scratch[i] = (char*)ring_mem + (size_t)i * nbytes;
        }
        a.chunk_vecs = nbytes / 16 / (size_t)n;
        a.n = n;
        int chans = 1;
        // the reductions want workgroups, the copy kernels of the port want the rest of the chip
        if ((rc = pick_channels(c, kp, 256, n, a.chunk_vecs / 2 + 1, 8, g_opt.hb_blocks, 32, &chans))) return rc;
        a.chans = chans;
        const int pushing = g_opt.drop_rank >= 0 && g_opt.drop_rank < n ? n - 1 : n;
        port_announce(port, (unsigned long long)pushing * ring_port_requests(n));
        note_launch(n * chans, 256, algo);
        typedef void (*K)(RingArgs, PortShared*, DevCtx);
        return launch((K)kp, n * chans, 256, stream, a, port->shared_dev, dev_ctx(c));
    }
    if (algo == MSX_ALGO_2PR_HB) {
        // two-phase ring: n equal chunks of whole 16-byte vectors, no residual
        if (residual) return MSX_ERR_UNSUPPORTED;
        if (nbytes % (16 * (size_t)n)) return MSX_ERR_UNSUPPORTED;
        void* ring_mem = nullptr;
        if ((rc = ring_scratch(c, nbytes * (size_t)n, &ring_mem))) return rc;
        const void* kp = dtype == MSX_F32 ? (const void*)k_allreduce_ring<0> : (const void*)k_allreduce_ring<1>;
        RingArgs a{};
        for (int i = 0; i < n; ++i) {
            a.in[i] = send[i];
            a.out[i] = recv[i];
            a.scratch[i] = (char*)ring_mem + (size_t)i * nbytes;
        }
        a.chunk_vecs = nbytes / 16 / (size_t)n;
        a.n = n;
        int chans = 1;
        if ((rc = pick_channels(c, kp, 256, n, a.chunk_vecs, 4, g_opt.hb_blocks, 64, &chans))) return rc;
        a.chans = chans;
        note_launch(n * chans, 256, algo);
        typedef void (*K)(RingArgs, DevCtx);
        return launch((K)kp, n * chans, 256, stream, a, dev_ctx(c));
    }

    // HB protocol.  Launch shape by size (from a sweep on MI355X): small messages want every
    // thread to issue all its loads at once (more unrolling, one pass); large ones want many
    // plain workgroups.  Options override.
    if (algo == MSX_ALGO_2PA_HB_2PHASE && residual && !res_shared) return MSX_ERR_UNSUPPORTED;
    const int threads = 256;
    const size_t vecs = nbytes / 16;
    const size_t per_rank = (vecs + (size_t)n - 1) / (size_t)n;
    int U = 1, want = 1;
    choose_hb_shape(nbytes, n, threads, &U, &want);
    if (algo == MSX_ALGO_2PA_HB_2PHASE && U > 2) U = 2;
    const int res_mode = !residual ? 0 : res_shared ? 1 : 2;
    HbKernel k = algo == MSX_ALGO_2PA_HB ? hb_fused_kernel(dtype, U, n, res_mode, choose_cache_mode(nbytes, n, res_mode))
                                         : hb_2phase_kernel(dtype, U, n);
    // very large messages: the same sums in chip-wide read and write phases, one workgroup per CU (as many
    // as are resident; an explicit hb_blocks_per_rank still counts)
    if (algo == MSX_ALGO_2PA_HB && use_phased(nbytes, n, res_mode, kPhasedAllReduce)) {
        k = phased_reduce_kernel(dtype == MSX_F32, n, res_mode, 0);
        U = kPhasedHeld;
        want = g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels;
    }
    int chans = 1;
    if ((rc = pick_channels(c, (const void*)k, threads, n, per_rank, (size_t)U, want, kMaxChannels, &chans)))
        return rc;
    HbArgs a{};
    for (int i = 0; i < n; ++i) {
        a.in[i] = send[i];
        a.out[i] = recv[i];
        a.res[i] = residual ? residual[i] : nullptr;
    }
    a.count = count;
    a.n = n;
    a.chans = chans;
    a.has_res = residual ? 1 : 0;
    a.res_shared = res_shared ? 1 : 0;
    a.barriers = g_opt.hb_barriers;
    a.peer_outer = g_opt.peer_outer;
    a.pace = g_opt.hb_pace;
    note_launch(n * chans, threads, algo);
    return launch(k, n * chans, threads, stream, a, dev_ctx(c));
}


// AllGather / ReduceScatter over LL packets.  nbytes = bytes per block (multiple of 8).
int ll_coll(bool gather, const void* const* in, void* const* out, size_t nbytes, int dtype, int nranks,
            hipStream_t stream)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    const int n = nranks;
    const size_t P = nbytes / 8;
    if ((size_t)n * P * 16 > c->d.ll_rot_stride) return MSX_ERR_NOMEM;
    const void* kp;
    if (gather) kp = n == 8 ? (const void*)k_allgather_ll<8> : (const void*)k_allgather_ll<0>;
    else if (dtype == MSX_F32) kp = n == 8 ? (const void*)k_reducescatter_ll<0, 8> : (const void*)k_reducescatter_ll<0, 0>;
    else kp = n == 8 ? (const void*)k_reducescatter_ll<1, 8> : (const void*)k_reducescatter_ll<1, 0>;
    const int threads = ll_block_threads(P);
    int chans = 1;
    if ((rc = pick_channels(c, kp, threads, n, P, 1, g_opt.ll_blocks, 32, &chans))) return rc;
    LlCollArgs a{};
    for (int i = 0; i < n; ++i) {
        a.in[i] = in[i];
        a.out[i] = out[i];
    }
    a.nbytes = nbytes;
    a.n = n;
    a.chans = chans;
    note_launch(n * chans, threads, gather ? MSX_ALGO_1PA_LL : MSX_ALGO_2PA_LL);
    typedef void (*K)(LlCollArgs, DevCtx);
    return launch((K)kp, n * chans, threads, stream, a, dev_ctx(c));
}

// 1: use the LL kernels, 0: use the HB kernels, < 0: LL was demanded but cannot serve this request
int use_ll_coll(size_t nbytes, bool aligned8)
{
    const bool can = aligned8 && nbytes % 8 == 0;
    if (g_opt.coll_algo == 1) return can ? 1 : MSX_ERR_UNSUPPORTED;
    if (g_opt.coll_algo == 2 || !can) return 0;
    return nbytes <= g_opt.coll_ll_max ? 1 : 0;
}

// ---- the other HB collectives: a.count semantics differ per kernel -----------------------------

enum HbOther { kRS, kAG, kA2A, kA2AInplace };

// AllGather kernel by vectors in flight per thread: a write-only stream to 8 destinations gains about 5 %
// from 8 (measured), short blocks stay at 2
const void* ag_kernel(size_t vectors_per_rank, int keep)
{
    int u = g_opt.hb_unroll;
    if (u == 0) u = vectors_per_rank >= (size_t)8 * 128 * 256 ? 8 : 2;
    switch (u) {
        case 1: return (const void*)k_allgather_hb<1>;
        case 4: return (const void*)k_allgather_hb<4>;
        case 8: return keep ? (const void*)k_allgather_hb<8, 1> : (const void*)k_allgather_hb<8>;
        default: return keep ? (const void*)k_allgather_hb<2, 1> : (const void*)k_allgather_hb<2>;
    }
}

int hb_other(HbOther which, const void* const* in, void* const* out, size_t count_or_bytes, int dtype,
             int nranks, int vec, size_t work_units, hipStream_t stream)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    const int n = nranks, threads = 256;
    const void* kp = nullptr;
    // everything the call writes (n x n blocks) fits the memory-side cache: let the stores stay there
    const size_t block_bytes = which == kRS ? 0 : count_or_bytes;
    const int keep = g_opt.cache_mode >= 0 ? (g_opt.cache_mode != 0)
                                           : (block_bytes * (size_t)n * (size_t)n <= ((size_t)256 << 20));
    switch (which) {
        case kRS: kp = dtype == MSX_F32 ? (const void*)k_reducescatter_hb<0, 2> : (const void*)k_reducescatter_hb<1, 2>; break;
        case kAG: kp = ag_kernel(work_units, keep); break;
        case kA2A: kp = keep ? (const void*)k_alltoall_hb<1> : (const void*)k_alltoall_hb<0>; break;
        case kA2AInplace: kp = (const void*)k_alltoall_inplace; break;
    }
    // large blocks, 8 ranks: chip-wide read and write phases, one workgroup per CU (see k_allreduce_hb_phased)
    const size_t row_bytes = (which == kRS ? count_or_bytes * elem_size(dtype) : count_or_bytes) * (size_t)n;
    if ((which == kRS || which == kAG) && vec && use_phased(row_bytes, n, 0, which == kAG ? kPhasedAllGather : kPhasedOther)) {
        HbKernel pk = which == kRS ? phased_reduce_kernel(dtype == MSX_F32, n, 0, 1) : phased_allgather_kernel(n);
        int pch = 1;
        if ((rc = pick_channels(c, (const void*)pk, threads, n, work_units, kPhasedHeld,
                                g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels, kMaxChannels, &pch)))
            return rc;
        HbArgs pa{};
        for (int i = 0; i < n; ++i) {
            pa.in[i] = in[i];
            pa.out[i] = out[i];
        }
        pa.count = count_or_bytes;
        pa.n = n;
        pa.chans = pch;
        pa.barriers = g_opt.hb_barriers;
        pa.pace = g_opt.hb_pace;
        note_launch(n * pch, threads, MSX_ALGO_2PA_HB);
        return launch(pk, n * pch, threads, stream, pa, dev_ctx(c));
    }
    // workgroups per rank, from sweeps: one vector per thread in a single pass while that fits (small and
    // mid sizes are latency bound: 64 KiB rows 4.8 -> 4.2 us reduce-scatter, 7.9 -> 5.4 us all-gather); for
    // large inputs the read-heavy reduce-scatter runs best with few workgroups per rank (32; 64 up to
    // 64 MiB blocks), the write-heavy copies with many
    // (the sweeps were run with 8 ranks; what counts is the total over the chip, so fewer ranks get more each:
    // with the per-rank figures of 8 ranks a 2-rank reduce-scatter ran on 64 workgroups, at 1.2 TB/s)
    const int total = which == kRS ? (work_units <= ((size_t)4 << 20) ? 512 : 256) : 1024;
    const int cap = per_rank_cap(total, n);
    int chans = 1;
    if ((rc = pick_channels(c, kp, threads, n, work_units, 1, g_opt.hb_blocks, cap, &chans))) return rc;
    HbArgs a{};
    for (int i = 0; i < n; ++i) {
        a.in[i] = in ? in[i] : nullptr;
        a.out[i] = out[i];
    }
    a.count = count_or_bytes;
    a.n = n;
    a.chans = chans;
    a.barriers = g_opt.hb_barriers;
    // all-to-all of large blocks: block after block, the ranks in step (see k_alltoall_hb); "peer_outer" 1 / 2
    // force that order for any size (1: without the rank barrier between the blocks)
    if (which == kA2A) a.peer_outer = g_opt.peer_outer ? g_opt.peer_outer : (count_or_bytes >= g_opt.a2a_blocks_min ? 2 : 0);
    note_launch(n * chans, threads, MSX_ALGO_2PA_HB);
    const DevCtx d = dev_ctx(c);
    switch (which) {
        case kRS:
            if (dtype == MSX_F32) return launch(k_reducescatter_hb<0, 2>, n * chans, threads, stream, a, d, vec);
            return launch(k_reducescatter_hb<1, 2>, n * chans, threads, stream, a, d, vec);
        case kAG: {
            typedef void (*K)(HbArgs, DevCtx, int);
            return launch((K)kp, n * chans, threads, stream, a, d, vec);
        }
        case kA2A: {
            typedef void (*K)(HbArgs, DevCtx, int);
            return launch((K)kp, n * chans, threads, stream, a, d, vec);
        }
        case kA2AInplace: return launch(k_alltoall_inplace, n * chans, threads, stream, a, d, vec);
    }
    return MSX_ERR_ARG;
}

// ceil(2^32 / per_rank), with which the plan kernel turns e / per_rank into a multiplication (exact while
// e * per_rank < 2^32: n_experts below 65536), or 0 = divide
unsigned owner_magic(int n_experts, int per_rank)
{
    return (n_experts < 65536 && per_rank > 1) ? (unsigned)((0x100000000ull + (unsigned)per_rank - 1u) / (unsigned)per_rank) : 0u;
}

// The routing plan a dispatch / combine works on: the handle's, or the context's built-in one.  A prepared
// call needs a plan of fixed size (the built-in one may be regrown, and moved, by a later dispatch).
int moe_plan_of(Ctx* c, void* handle, MoePlan** out)
{
    if (!handle) {
        if (t_record) return MSX_ERR_ARG;
        *out = &c->moe;
        return MSX_OK;
    }
    for (MoePlan* p : g_plans)
        if (p == handle) {
            if (p->owner != c) return MSX_ERR_ARG;
            *out = p;
            return MSX_OK;
        }
    return MSX_ERR_ARG;
}

// Token dispatch; recv_scales != nullptr selects the fused FP8 quantisation (tokens are bf16 then).
int moe_dispatch_impl(const void* const* tokens, const int32_t* const* topk_idx, int T, int H, int K, int n_experts,
                      int dtype, int nranks, void* const* recv_tokens, float* const* recv_scales,
                      int32_t* const* recv_src_token, int32_t* recv_counts, size_t recv_capacity_tokens,
                      void* plan_handle, hipStream_t s)
{
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if ((rc = check_table(tokens, nranks))) return rc;
    if ((rc = check_table((const void* const*)topk_idx, nranks))) return rc;
    if ((rc = check_table((const void* const*)recv_tokens, nranks))) return rc;
    if (!recv_counts) return MSX_ERR_ARG;
    if (recv_src_token)
        for (int r = 0; r < nranks; ++r)
            if (!recv_src_token[r]) return MSX_ERR_ARG;
    if (recv_scales)
        for (int r = 0; r < nranks; ++r)
            if (!recv_scales[r] || ((uintptr_t)recv_scales[r] & 3u)) return MSX_ERR_ARG;
    if (T < 0 || H <= 0 || K <= 0 || K > 32 || n_experts <= 0 || n_experts % nranks) return MSX_ERR_ARG;
    if (T > 65534) return MSX_ERR_UNSUPPORTED;
    const size_t row_bytes = (size_t)H * elem_size(dtype);
    if (row_bytes % 16) return MSX_ERR_ARG;
    if (recv_capacity_tokens > 0xffffffffull) recv_capacity_tokens = 0xffffffffull;

    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    if ((rc = get_ctx(&c))) return rc;
    const int n = nranks;
    MoePlan* plan = nullptr;
    if ((rc = moe_plan_of(c, plan_handle, &plan))) return rc;
    const size_t need = (size_t)kMaxRanks * (size_t)(T > 0 ? T : 1) * 16;
    if (need > plan->slots_bytes) {
        if (plan->fixed_size) return MSX_ERR_NOMEM;      // made for fewer tokens per rank
        if (plan->slots) { HIPCHK(hipDeviceSynchronize()); HIPCHK(hipFree(plan->slots)); plan->slots = nullptr; plan->slots_bytes = 0; }
        HIPCHK(hipMalloc(&plan->slots, need));
        plan->slots_bytes = need;
    }
    MoeArgs a{};
    for (int i = 0; i < n; ++i) {
        a.tokens[i] = tokens[i];
        a.topk[i] = topk_idx[i];
        a.recv[i] = recv_tokens[i];
        a.recv_src[i] = recv_src_token ? recv_src_token[i] : nullptr;
    }
    a.recv_counts = recv_counts;
    a.slots = (unsigned short*)plan->slots;
    a.base = plan->base;
    a.T = T;
    a.K = K;
    a.n = n;
    a.per_rank = n_experts / n;
    a.n_experts = n_experts;
    // e / per_rank = high word of e * ceil(2^32 / per_rank), exact while e * per_rank < 2^32
    a.per_rank_magic = owner_magic(n_experts, a.per_rank);
    a.row_vecs = (unsigned)(row_bytes / 16);
    a.cap = (unsigned)recv_capacity_tokens;
    a.has_src = recv_src_token ? 1 : 0;
    const DevCtx d = dev_ctx(c);

    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_moe_plan, kPlanThreads, &resident))) return rc;
    if (resident < n) return MSX_ERR_UNSUPPORTED;
    a.chans = 1;
    if ((rc = launch(k_moe_plan, n, kPlanThreads, s, a, d))) return rc;

    int chans = 1;
    // one wave per token row, 4 waves per workgroup, a few rows per wave
    if ((rc = pick_channels(c, (const void*)k_moe_pack, 256, n, (size_t)T * 64, 4, g_opt.hb_blocks, per_rank_cap(1024, n), &chans)))
        return rc;
    a.chans = chans;
    plan->T = T;
    plan->n = n;
    // many rows of whole multiples of 64 vectors (bf16 / fp32 pack only): chip-wide read and write phases, one
    // workgroup per CU.  Automatic for 8 ranks from 32 MiB of tokens per rank; an explicit hb_phased_min_bytes
    // counts for every rank count.
    const size_t token_bytes = (size_t)T * row_bytes;
    if (!recv_scales && a.row_vecs % 64u == 0 && (unsigned long long)T * a.row_vecs < (1ull << 32) &&
        (g_opt.hb_phased_min < 0 ? n == 8 && token_bytes >= ((size_t)32 << 20)
                                 : token_bytes >= (size_t)g_opt.hb_phased_min)) {
        auto kd = k_moe_pack_dealt<kPhasedHeld>;
        int dch = 1;
        if ((rc = pick_channels(c, (const void*)kd, 256, n, (size_t)T * a.row_vecs, (size_t)kPhasedHeld,
                                g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels, kMaxChannels, &dch)))
            return rc;
        a.chans = dch;
        note_launch(n * dch, 256, MSX_ALGO_2PA_HB);
        return launch(kd, n * dch, 256, s, a, d, g_opt.hb_pace);
    }
    note_launch(n * chans, 256, MSX_ALGO_2PA_HB);
    if (recv_scales) {
        MoeFp8Args f{};
        for (int i = 0; i < n; ++i) f.recv_scales[i] = recv_scales[i];
        f.groups = (unsigned)(H / 128);
        return launch(k_moe_pack_fp8, n * chans, 256, s, a, f, d);
    }
    return launch(k_moe_pack, n * chans, 256, s, a, d);
}



bool parse_u64(const char* s, unsigned long long* v)
{
    if (!s || !*s) return false;
    char* end = nullptr;
    unsigned long long x = strtoull(s, &end, 10);
    if (*end) return false;
    *v = x;
    return true;
}

}  // namespace

// =============================================================================================
// C ABI
// =============================================================================================

extern "C" {

int msx_allreduce_ex(const void* const* send, void* const* recv, const void* const* residual, size_t count,
                     int dtype, int op, int nranks, int algo, void* stream)
{
    return allreduce_impl(send, recv, residual, count, dtype, op, nranks, algo, (hipStream_t)stream);
}

int msx_allreduce_ex_static(const void* const* send, void* const* recv, const void* const* residual, size_t count,
                            int dtype, int op, int nranks, int algo, void* stream)
{
    return allreduce_impl(send, recv, residual, count, dtype, op, nranks, algo, (hipStream_t)stream, true);
}

int msx_allreduce(void* buf, size_t count, int dtype, int op, int nranks, void* stream)
{
    int rc = check_common(dtype, op, nranks);
    if (rc) return rc;
    if (count == 0) return MSX_OK;
    if (!buf || !aligned16(buf)) return MSX_ERR_ARG;
    const size_t row = count * elem_size(dtype);
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    for (int r = 0; r < nranks; ++r) in[r] = out[r] = (char*)buf + (size_t)r * row;
    if (nranks > 1 && (row & 15u)) {
        // rows that do not start on 16-byte boundaries: the element-by-element kernel
        std::lock_guard<std::mutex> lk(g_mu);
        Ctx* c = nullptr;
        if ((rc = get_ctx(&c))) return rc;
        return reduce_generic(c, in, out, count, dtype, op, nranks, 2, 0, (hipStream_t)stream);
    }
    return allreduce_impl(in, out, nullptr, count, dtype, op, nranks, MSX_ALGO_AUTO, (hipStream_t)stream);
}

int msx_reducescatter_ex(const void* const* send, void* const* recv, size_t count, int dtype, int op, int nranks,
                         void* stream)
{
    int rc = check_common(dtype, op, nranks);
    if (rc) return rc;
    if ((rc = check_table(send, nranks))) return rc;
    if (!recv) return MSX_ERR_ARG;
    if (count % (size_t)nranks) return MSX_ERR_ARG;
    if (count == 0) return MSX_OK;
    const size_t c = count / (size_t)nranks, esz = elem_size(dtype);
    int vec = (c * esz) % 16 == 0;
    for (int r = 0; r < nranks; ++r) {
        if (!recv[r]) return MSX_ERR_ARG;
        if (!aligned16(recv[r])) vec = 0;
        if ((uintptr_t)recv[r] % esz) return MSX_ERR_ARG;
    }
    if (dtype == MSX_F16 || dtype == MSX_I32 || op != MSX_SUM) {
        std::lock_guard<std::mutex> lk(g_mu);
        Ctx* ctx = nullptr;
        if ((rc = get_ctx(&ctx))) return rc;
        return reduce_generic(ctx, send, recv, c, dtype, op, nranks, 1, vec, (hipStream_t)stream);
    }
    if (nranks > 1) {
        bool al8 = true;
        for (int r = 0; r < nranks; ++r) al8 = al8 && ((uintptr_t)recv[r] & 7u) == 0;
        const int ll = use_ll_coll(c * esz, al8);
        if (ll < 0) return ll;
        if (ll) {
            const int rc2 = ll_coll(false, send, recv, c * esz, dtype, nranks, (hipStream_t)stream);
            if (rc2 != MSX_ERR_NOMEM || g_opt.coll_algo == 1) return rc2;
        }
    }
    const size_t work = vec ? c * esz / 16 : c;
    return hb_other(kRS, send, recv, c, dtype, nranks, vec, work, (hipStream_t)stream);
}

int msx_reducescatter(void* buf, size_t count, int dtype, int op, int nranks, void* stream)
{
    int rc = check_common(dtype, op, nranks);
    if (rc) return rc;
    if (count % (size_t)nranks) return MSX_ERR_ARG;
    if (count == 0) return MSX_OK;
    if (!buf || !aligned16(buf)) return MSX_ERR_ARG;
    const size_t esz = elem_size(dtype), row = count * esz, c = count / (size_t)nranks;
    if (nranks > 1 && (row & 15u)) return MSX_ERR_ARG;
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    for (int r = 0; r < nranks; ++r) {
        in[r] = (char*)buf + (size_t)r * row;
        out[r] = (char*)buf + (size_t)r * row + (size_t)r * c * esz;   // rank r's own share, in place
    }
    return msx_reducescatter_ex(in, out, count, dtype, op, nranks, stream);
}

int msx_allgather_ex(const void* const* send, void* const* recv, size_t count, int dtype, int nranks, void* stream)
{
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if (!send || !recv) return MSX_ERR_ARG;
    if (count == 0) return MSX_OK;
    const size_t nbytes = count * elem_size(dtype);
    int vec = nbytes % 16 == 0;
    for (int r = 0; r < nranks; ++r) {
        if (!send[r] || !recv[r]) return MSX_ERR_ARG;
        if (!aligned16(send[r]) || !aligned16(recv[r])) vec = 0;
    }
    if (nranks > 1) {
        bool al8 = true;
        for (int r = 0; r < nranks; ++r)
            al8 = al8 && ((uintptr_t)send[r] & 7u) == 0 && ((uintptr_t)recv[r] & 7u) == 0;
        const int ll = use_ll_coll(nbytes, al8);
        if (ll < 0) return ll;
        if (ll) {
            const int rc2 = ll_coll(true, send, recv, nbytes, dtype, nranks, (hipStream_t)stream);
            if (rc2 != MSX_ERR_NOMEM || g_opt.coll_algo == 1) return rc2;
        }
    }
    const size_t work = vec ? nbytes / 16 : nbytes;
    return hb_other(kAG, send, recv, nbytes, dtype, nranks, vec, work, (hipStream_t)stream);
}

int msx_allgather(void* buf, size_t count, int dtype, int op, int nranks, void* stream)
{
    (void)op;
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if (count == 0) return MSX_OK;
    if (!buf) return MSX_ERR_ARG;
    const size_t nbytes = count * elem_size(dtype), row = nbytes * (size_t)nranks;
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    for (int r = 0; r < nranks; ++r) {
        out[r] = (char*)buf + (size_t)r * row;
        in[r] = (char*)out[r] + (size_t)r * nbytes;   // rank r's contribution already sits in its slot
    }
    return msx_allgather_ex(in, out, count, dtype, nranks, stream);
}

int msx_alltoall_ex(const void* const* send, void* const* recv, size_t count, int dtype, int nranks, void* stream)
{
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if (!send || !recv) return MSX_ERR_ARG;
    if (count % (size_t)nranks) return MSX_ERR_ARG;
    if (count == 0) return MSX_OK;
    const size_t row = count * elem_size(dtype);
    const size_t nbytes = row / (size_t)nranks;
    int vec = nbytes % 16 == 0;
    for (int r = 0; r < nranks; ++r) {
        if (!send[r] || !recv[r]) return MSX_ERR_ARG;
        if (!aligned16(send[r]) || !aligned16(recv[r])) vec = 0;
        for (int q = 0; q < nranks; ++q) {   // send and recv must not overlap
            const char *s0 = (const char*)send[q], *r0 = (const char*)recv[r];
            if (s0 < r0 + row && r0 < s0 + row) return MSX_ERR_ARG;
        }
    }
    const size_t work = vec ? nbytes / 16 : nbytes;
    return hb_other(kA2A, send, recv, nbytes, dtype, nranks, vec, work, (hipStream_t)stream);
}

int msx_alltoall(void* buf, size_t count, int dtype, int op, int nranks, void* stream)
{
    (void)op;
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if (count % (size_t)nranks) return MSX_ERR_ARG;
    if (count == 0) return MSX_OK;
    if (!buf) return MSX_ERR_ARG;
    const size_t row = count * elem_size(dtype), nbytes = row / (size_t)nranks;
    void* out[kMaxRanks];
    for (int r = 0; r < nranks; ++r) out[r] = (char*)buf + (size_t)r * row;
    const int vec = aligned16(buf) && nbytes % 16 == 0;
    const size_t work = (vec ? nbytes / 16 : nbytes) * (size_t)(nranks > 1 ? nranks - 1 : 1) / 2 + 1;
    return hb_other(kA2AInplace, nullptr, out, nbytes, dtype, nranks, vec, work, (hipStream_t)stream);
}

int msx_moe_dispatch(const void* const* tokens, const int32_t* const* topk_idx, int T, int H, int K, int n_experts,
                     int dtype, int nranks, void* const* recv_tokens, int32_t* const* recv_src_token,
                     int32_t* recv_counts, size_t recv_capacity_tokens, void* plan, void* stream)
{
    return moe_dispatch_impl(tokens, topk_idx, T, H, K, n_experts, dtype, nranks, recv_tokens, nullptr,
                             recv_src_token, recv_counts, recv_capacity_tokens, plan, (hipStream_t)stream);
}

int msx_moe_dispatch_fp8(const void* const* tokens, const int32_t* const* topk_idx, int T, int H, int K,
                         int n_experts, int nranks, void* const* recv_q, float* const* recv_scales,
                         int32_t* const* recv_src_token, int32_t* recv_counts, size_t recv_capacity_tokens,
                         void* plan, void* stream)
{
    if (!recv_scales) return MSX_ERR_ARG;
    if (H <= 0 || H % 128) return MSX_ERR_ARG;
    return moe_dispatch_impl(tokens, topk_idx, T, H, K, n_experts, MSX_BF16, nranks, recv_q, recv_scales,
                             recv_src_token, recv_counts, recv_capacity_tokens, plan, (hipStream_t)stream);
}

int msx_moe_combine(const void* const* expert_out, void* const* out_tokens, int T, int H, int dtype, int nranks,
                    size_t capacity_tokens, void* plan_handle, void* stream)
{
    int rc = check_common(dtype, MSX_SUM, nranks);
    if (rc) return rc;
    if (dtype != MSX_F32 && dtype != MSX_BF16) return MSX_ERR_UNSUPPORTED;   // the sums exist for these two
    if ((rc = check_table(expert_out, nranks))) return rc;
    if ((rc = check_table((const void* const*)out_tokens, nranks))) return rc;
    if (T < 0 || H <= 0) return MSX_ERR_ARG;
    const size_t row_bytes = (size_t)H * elem_size(dtype);
    if (row_bytes % 16) return MSX_ERR_ARG;
    if (capacity_tokens > 0xffffffffull) capacity_tokens = 0xffffffffull;

    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    if ((rc = get_ctx(&c))) return rc;
    MoePlan* plan = nullptr;
    if ((rc = moe_plan_of(c, plan_handle, &plan))) return rc;
    if (plan->T != T || plan->n != nranks || !plan->slots) return MSX_ERR_ARG;   // no matching dispatch through this plan
    if (T == 0) return MSX_OK;
    const int n = nranks;
    MoeArgs a{};
    for (int i = 0; i < n; ++i) {
        a.recv[i] = const_cast<void*>(expert_out[i]);
        a.tokens[i] = out_tokens[i];
    }
    a.slots = (unsigned short*)plan->slots;
    a.base = plan->base;
    a.T = T;
    a.n = n;
    a.row_vecs = (unsigned)(row_bytes / 16);
    a.cap = (unsigned)capacity_tokens;
    // many rows of whole multiples of 64 vectors: chip-wide read and write phases, one workgroup per CU (see
    // k_moe_combine_dealt).  Automatic for 8 ranks from 32 MiB of tokens per rank, like the token pack; an explicit
    // hb_phased_min_bytes counts for every rank count.
    const size_t token_bytes = (size_t)T * row_bytes;
    const unsigned long long out_vecs = (unsigned long long)T * a.row_vecs;
    if (a.row_vecs % 64u == 0 && out_vecs % 256u == 0 && out_vecs < (1ull << 32) &&
        (unsigned long long)a.cap * row_bytes <= 0xE0000000ull &&
        (g_opt.hb_phased_min < 0 ? n == 8 && token_bytes >= ((size_t)32 << 20)
                                 : token_bytes >= (size_t)g_opt.hb_phased_min)) {
        CombineKernel kd = combine_dealt_kernel(dtype == MSX_F32);
        int dch = 1;
        if ((rc = pick_channels(c, (const void*)kd, 256, n, (size_t)out_vecs, (size_t)kCombineHeld,
                                g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels, kMaxChannels, &dch)))
            return rc;
        a.chans = dch;
        note_launch(n * dch, 256, MSX_ALGO_2PA_HB);
        return launch(kd, n * dch, 256, (hipStream_t)stream, a, dev_ctx(c));
    }
    const void* kp = dtype == MSX_F32 ? (const void*)k_moe_combine<0> : (const void*)k_moe_combine<1>;
    int chans = 1;
    // read-heavy like the reduce-scatter: 32 workgroups per rank beat more (measured at 8 x 4096 rows of 7168:
    // 0.56 ms against 0.585 ms with 128)
    if ((rc = pick_channels(c, kp, 256, n, (size_t)T * 64, 4, g_opt.hb_blocks, per_rank_cap(256, n), &chans))) return rc;
    a.chans = chans;
    note_launch(n * chans, 256, MSX_ALGO_2PA_HB);
    typedef void (*K)(MoeArgs, DevCtx);
    return launch((K)kp, n * chans, 256, (hipStream_t)stream, a, dev_ctx(c));
}

// ---- primitives -------------------------------------------------------------------------------

int msx_prim_pingpong(int iters, int grid_blocks, int block_a, int block_b, double* ns_out, void* stream)
{
    if (iters < 0 || grid_blocks < 2 || block_a < 0 || block_b < 0 || block_a >= grid_blocks ||
        block_b >= grid_blocks || block_a == block_b || !ns_out)
        return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_pingpong, 64, &resident))) return rc;
    if (grid_blocks > resident) return MSX_ERR_ARG;
    note_launch(grid_blocks, 64, 0);
    return launch(k_pingpong, grid_blocks, 64, (hipStream_t)stream, dev_ctx(c), iters, block_a, block_b,
                  c->ns_per_tick, ns_out);
}

int msx_prim_barrier(int rounds, int nranks, int blocks_per_rank, uint32_t* sem_out, void* stream)
{
    if (rounds < 0 || nranks < 1 || nranks > kMaxRanks || blocks_per_rank < 1 || blocks_per_rank > kMaxChannels)
        return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_barrier_rounds, 256, &resident))) return rc;
    if (nranks * blocks_per_rank > resident) return MSX_ERR_ARG;
    const DevCtx d = dev_ctx(c);
    if (rounds > 0 && nranks > 1) {
        note_launch(nranks * blocks_per_rank, 256, 0);
        if ((rc = launch(k_barrier_rounds, nranks * blocks_per_rank, 256, (hipStream_t)stream, d, nranks, rounds,
                         g_opt.barrier_fences)))
            return rc;
    }
    if (sem_out) return launch(k_sem_snapshot, 1, 64, (hipStream_t)stream, d, nranks, (unsigned*)sem_out);
    return MSX_OK;
}

int msx_prim_put_signal_wait(const void* src, void* staging, void* dst, size_t nbytes, int blocks_per_rank,
                             void* stream)
{
    if (!src || !staging || !dst || !aligned16(src) || !aligned16(staging) || !aligned16(dst)) return MSX_ERR_ARG;
    if (blocks_per_rank < 1 || blocks_per_rank > kMaxChannels) return MSX_ERR_ARG;
    if (nbytes == 0) return MSX_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_put_signal_wait, 256, &resident))) return rc;
    if (2 * blocks_per_rank > resident) return MSX_ERR_ARG;
    note_launch(2 * blocks_per_rank, 256, 0);
    return launch(k_put_signal_wait, 2 * blocks_per_rank, 256, (hipStream_t)stream, dev_ctx(c), src, staging, dst,
                  nbytes, blocks_per_rank);
}

int msx_prim_stream(int mode, const void* src, void* dst, size_t nbytes, int blocks, void* stream)
{
    if (mode < 0 || mode > 2 || blocks < 1 || blocks > 65536 || nbytes % 16) return MSX_ERR_ARG;
    if ((mode != 1 && (!src || !aligned16(src))) || (mode != 0 && (!dst || !aligned16(dst)))) return MSX_ERR_ARG;
    if (nbytes == 0) return MSX_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    note_launch(blocks, 256, 0);
    const size_t nvec = nbytes / 16;
    unsigned* sink = c->d.status + 15;     // a word of the status block nothing reads; written only if the data is all ones
    if (mode == 0) return launch(k_stream<0>, blocks, 256, (hipStream_t)stream, (const u32x4*)src, (u32x4*)nullptr, nvec, sink);
    if (mode == 1) return launch(k_stream<1>, blocks, 256, (hipStream_t)stream, (const u32x4*)nullptr, (u32x4*)dst, nvec, sink);
    return launch(k_stream<2>, blocks, 256, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, nvec, sink);
}

int msx_prim_ll_encode(const void* src, size_t nbytes, uint32_t flag, void* packets_out, void* stream)
{
    if (nbytes == 0) return MSX_OK;
    if (!src || !packets_out || !aligned16(packets_out)) return MSX_ERR_ARG;
    const size_t P = (nbytes + 7) / 8;
    size_t grid = (P + 255) / 256;
    if (grid > 1024) grid = 1024;
    note_launch((int)grid, 256, 0);
    return launch(k_ll_encode, (int)grid, 256, (hipStream_t)stream, src, nbytes, (unsigned)flag, (u32x4*)packets_out);
}

int msx_prim_ll_roundtrip(const void* src, void* dst, size_t nbytes, int blocks_per_rank, void* stream)
{
    if (nbytes == 0) return MSX_OK;
    if (!src || !dst) return MSX_ERR_ARG;
    if (blocks_per_rank < 1 || blocks_per_rank > kMaxChannels) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    const size_t P = (nbytes + 7) / 8;
    if (P * 16 > c->d.ll_rot_stride) return MSX_ERR_NOMEM;
    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_ll_roundtrip, 256, &resident))) return rc;
    if (2 * blocks_per_rank > resident) return MSX_ERR_ARG;
    note_launch(2 * blocks_per_rank, 256, 0);
    return launch(k_ll_roundtrip, 2 * blocks_per_rank, 256, (hipStream_t)stream, dev_ctx(c), src, dst, nbytes,
                  blocks_per_rank);
}

int msx_prim_port_put_signal_wait(const void* src, void* staging, void* dst, size_t nbytes, void* stream)
{
    if (!src || !staging || !dst || !aligned16(src) || !aligned16(staging) || !aligned16(dst)) return MSX_ERR_ARG;
    if (nbytes == 0) return MSX_OK;
    if (t_record) return MSX_ERR_UNSUPPORTED;      // the proxy is told of every launch: not a call to prepare
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c);
    if (rc) return rc;
    Port* p = nullptr;
    if ((rc = get_port(c, &p))) return rc;
    int resident = 0;
    if ((rc = resident_blocks(c, (const void*)k_port_put_signal_wait, 256, &resident))) return rc;
    if (resident < 2) return MSX_ERR_UNSUPPORTED;
    size_t readers = (nbytes + (256 * 16 * 8) - 1) / (256 * 16 * 8);   // 32 KiB per reading workgroup and pass
    if (readers < 1) readers = 1;
    if (readers > 128) readers = 128;      // half of the CUs: the proxy's copy kernel needs the others while these wait
    if ((int)readers + 1 > resident) readers = (size_t)resident - 1;
    port_announce(p, g_opt.drop_rank == 0 ? 0 : 3);   // put, signal, flush (a dropped sender pushes nothing)
    note_launch(1 + (int)readers, 256, 0);
    return launch(k_port_put_signal_wait, 1 + (int)readers, 256, (hipStream_t)stream, dev_ctx(c), p->shared_dev, src,
                  staging, dst, nbytes, (int)readers);
}

// ---- context, options, status ---------------------------------------------------------------

int msx_init(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = default_ctx(&c);
    if (rc) return rc;
    return get_static_ctx(nullptr, &c);
}

}  // extern "C"
namespace {
// Re-zero everything a context's kernels synchronise through.  Waits for the device.
int reset_ctx(Ctx* c)
{
    HIPCHK(hipDeviceSynchronize());
    if (c->fixed) {
        HIPCHK(hipMemset(c->d.sem, 0, kStaticBytes));
    } else {
        HIPCHK(hipMemset(c->d.sem, 0, (size_t)kMaxRanks * kMaxRanks * kMaxChannels * kSemStrideWords * 4));
        HIPCHK(hipMemset(c->d.expected, 0, (size_t)kMaxRanks * kMaxRanks * kMaxChannels * 4));
        HIPCHK(hipMemset(c->d.status, 0, 64));
        HIPCHK(hipMemset(c->d.call_state, 0, 64));
        HIPCHK(hipMemset(c->d.gbar, 0, kGridBarBytes));
        HIPCHK(hipMemset(c->d.ll, 0, c->d.ll_bytes));
    }
    HIPCHK(hipDeviceSynchronize());
    if (c->latch) __atomic_store_n(c->latch, 0u, __ATOMIC_RELAXED);
    if (c->port) {                       // a port channel that timed out starts over with a fresh proxy
        destroy_port(c->port);
        c->port = nullptr;
    }
    return MSX_OK;
}

}  // namespace
extern "C" {

int msx_reset(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = get_ctx(&c, false);
    if (rc) return rc;
    if ((rc = reset_ctx(c))) return rc;
    if (!t_use && g_static[c->device]) return reset_ctx(g_static[c->device]);
    return MSX_OK;
}

int msx_finalize(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MSX_ERR_ARG;
    Ctx* c = g_ctx[dev];
    g_ctx[dev] = nullptr;
    for (Prepared* p : g_prepared)
        if (p->ctx == c) p->ctx = nullptr;          // its handles can no longer run
    return destroy_ctx(c);
}

// ---- context handles ----------------------------------------------------------------------------

int msx_ctx_create(int nranks, size_t max_ll_bytes, void** ctx)
{
    if (!ctx || nranks < 1 || nranks > kMaxRanks) return MSX_ERR_ARG;
    if (max_ll_bytes != 0 && (max_ll_bytes < 4096 || max_ll_bytes > (16u << 20))) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = make_ctx(max_ll_bytes ? max_ll_bytes : g_opt.ll_max_bytes, &c);
    if (rc) return rc;
    g_made.push_back(c);
    *ctx = c;
    return MSX_OK;
}

int msx_ctx_destroy(void* ctx)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = (Ctx*)ctx;
    if (!known_ctx(c)) return MSX_ERR_ARG;
    for (size_t i = 0; i < g_made.size(); ++i)
        if (g_made[i] == c) { g_made.erase(g_made.begin() + (long)i); break; }
    if (t_use == c) t_use = nullptr;
    for (Prepared* p : g_prepared)
        if (p->ctx == c) p->ctx = nullptr;
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev != c->device) HIPCHK(hipSetDevice(c->device));
    const int rc = destroy_ctx(c);
    if (dev != c->device) HIPCHK(hipSetDevice(dev));
    return rc;
}

int msx_ctx_use(void* ctx)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (ctx && !known_ctx((Ctx*)ctx)) return MSX_ERR_ARG;
    t_use = (Ctx*)ctx;
    return MSX_OK;
}

}  // extern "C"
namespace {
// null = the context this thread's calls run on
int ctx_arg(void* ctx, Ctx** out)
{
    if (!ctx) return get_ctx(out, false);
    if (!known_ctx((Ctx*)ctx)) return MSX_ERR_ARG;
    *out = (Ctx*)ctx;
    return MSX_OK;
}

}  // namespace
extern "C" {

int msx_ctx_reset(void* ctx)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = ctx_arg(ctx, &c);
    if (rc) return rc;
    return reset_ctx(c);
}

int msx_ctx_set_max_blocks(void* ctx, int max_blocks)
{
    if (max_blocks < 0) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = ctx_arg(ctx, &c);
    if (rc) return rc;
    c->max_blocks = max_blocks;
    return MSX_OK;
}

}  // extern "C"
namespace {
// the status block of one context, read and cleared; the caller has waited for the work in question
int take_status(Ctx* c, uint32_t h[8])
{
    HIPCHK(hipMemcpy(h, c->d.status, 32, hipMemcpyDeviceToHost));
    if (h[0] != 0) HIPCHK(hipMemset(c->d.status, 0, 32));
    if (c->latch) __atomic_store_n(c->latch, 0u, __ATOMIC_RELAXED);
    return MSX_OK;
}

int status_code(const uint32_t h[8])
{
    if (h[0] == kStatusTimeout) return MSX_ERR_TIMEOUT;
    if (h[0] == kStatusCapacity) return MSX_ERR_CAPACITY;
    if (h[0] == kStatusBadIndex) return MSX_ERR_INDEX;
    return MSX_OK;
}

}  // namespace
extern "C" {

int msx_last_status(void* ctx, int* rank, int* site, unsigned* expected, unsigned* seen)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = ctx_arg(ctx, &c);
    if (rc) return rc;
    uint32_t h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if ((rc = take_status(c, h))) return rc;
    if (rank) *rank = (int)h[1];
    if (site) *site = (int)h[2];
    if (expected) *expected = h[3];
    if (seen) *seen = h[4];
    if (h[0] != 0) g_status_detail = h[6];
    return status_code(h);
}

// ---- routing plans --------------------------------------------------------------------------------

int msx_moe_plan_create(void* ctx, int max_tokens_per_rank, void** plan)
{
    if (!plan || max_tokens_per_rank < 1 || max_tokens_per_rank > 65534) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    Ctx* c = nullptr;
    int rc = ctx_arg(ctx, &c);
    if (rc) return rc;
    MoePlan* p = new MoePlan();
    p->owner = c;
    p->fixed_size = true;
    p->slots_bytes = (size_t)kMaxRanks * (size_t)max_tokens_per_rank * 16;
    if (hipMalloc(&p->slots, p->slots_bytes) != hipSuccess || hipMalloc((void**)&p->base, 64 * 4) != hipSuccess ||
        hipMemset(p->base, 0, 64 * 4) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        if (p->slots) (void)hipFree(p->slots);
        if (p->base) (void)hipFree(p->base);
        delete p;
        return MSX_ERR_NOMEM;
    }
    g_plans.push_back(p);
    *plan = p;
    return MSX_OK;
}

int msx_moe_plan_destroy(void* plan)
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (size_t i = 0; i < g_plans.size(); ++i)
        if (g_plans[i] == plan) {
            MoePlan* p = g_plans[i];
            g_plans.erase(g_plans.begin() + (long)i);
            HIPCHK(hipDeviceSynchronize());
            (void)hipFree(p->slots);
            (void)hipFree(p->base);
            delete p;
            return MSX_OK;
        }
    return MSX_ERR_ARG;
}

// ---- prepared calls ---------------------------------------------------------------------------------

}  // extern "C"
namespace {
// Runs `call` (one of the ordinary entry points) with its launches recorded instead of enqueued.
template <class F> int prepare(void** handle, F call)
{
    if (!handle) return MSX_ERR_ARG;
    if (t_record) return MSX_ERR_UNSUPPORTED;
    std::unique_ptr<Prepared> p(new Prepared());
    {
        std::lock_guard<std::mutex> lk(g_mu);
        int rc = get_ctx(&p->ctx);
        if (rc) return rc;
    }
    t_record = p.get();
    const int rc = call();
    t_record = nullptr;
    if (rc) {
        for (void* m : p->owned) (void)hipFree(m);
        return rc;
    }
    p->grid = t_grid; p->block = t_block; p->algo = t_algo;
    std::lock_guard<std::mutex> lk(g_mu);
    g_prepared.push_back(p.get());
    *handle = p.release();
    return MSX_OK;
}

}  // namespace
extern "C" {

int msx_prepare_allreduce(const void* const* send, void* const* recv, const void* const* residual, size_t count,
                          int dtype, int op, int nranks, int algo, void** handle)
{
    return prepare(handle, [&] { return msx_allreduce_ex(send, recv, residual, count, dtype, op, nranks, algo, nullptr); });
}

int msx_prepare_reducescatter(const void* const* send, void* const* recv, size_t count, int dtype, int op, int nranks,
                              void** handle)
{
    return prepare(handle, [&] { return msx_reducescatter_ex(send, recv, count, dtype, op, nranks, nullptr); });
}

int msx_prepare_allgather(const void* const* send, void* const* recv, size_t count, int dtype, int nranks, void** handle)
{
    return prepare(handle, [&] { return msx_allgather_ex(send, recv, count, dtype, nranks, nullptr); });
}

int msx_prepare_alltoall(const void* const* send, void* const* recv, size_t count, int dtype, int nranks, void** handle)
{
    return prepare(handle, [&] { return msx_alltoall_ex(send, recv, count, dtype, nranks, nullptr); });
}

int msx_prepare_moe_dispatch(const void* const* tokens, const int32_t* const* topk_idx, int T, int H, int K,
                             int n_experts, int dtype, int nranks, void* const* recv_tokens,
                             int32_t* const* recv_src_token, int32_t* recv_counts, size_t recv_capacity_tokens,
                             void* plan, void** handle)
{
    return prepare(handle, [&] {
        return msx_moe_dispatch(tokens, topk_idx, T, H, K, n_experts, dtype, nranks, recv_tokens, recv_src_token,
                                recv_counts, recv_capacity_tokens, plan, nullptr);
    });
}

int msx_prepare_moe_combine(const void* const* expert_out, void* const* out_tokens, int T, int H, int dtype, int nranks,
                            size_t capacity_tokens, void* plan, void** handle)
{
    return prepare(handle, [&] {
        return msx_moe_combine(expert_out, out_tokens, T, H, dtype, nranks, capacity_tokens, plan, nullptr);
    });
}

int msx_run(void* handle, void* stream)
{
    Prepared* p = (Prepared*)handle;
    if (!p || p->magic != kPreparedMagic || !p->ctx) return MSX_ERR_ARG;
    int rc = latched(p->ctx);
    if (rc) return rc;
    for (auto& step : p->steps) {
        const hipError_t e = step((hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    t_grid = p->grid; t_block = p->block; t_algo = p->algo;
    return MSX_OK;
}

int msx_release(void* handle)
{
    Prepared* p = (Prepared*)handle;
    if (!p) return MSX_OK;
    std::lock_guard<std::mutex> lk(g_mu);
    size_t at = g_prepared.size();
    for (size_t i = 0; i < g_prepared.size(); ++i)
        if (g_prepared[i] == p) at = i;
    if (at == g_prepared.size()) return MSX_ERR_ARG;
    g_prepared.erase(g_prepared.begin() + (long)at);
    if (!p->owned.empty()) {
        HIPCHK(hipDeviceSynchronize());          // a launch of this call may still be using its scratch
        for (void* m : p->owned) (void)hipFree(m);
    }
    p->magic = 0;
    delete p;
    return MSX_OK;
}

int msx_set_option(const char* key, const char* value)
{
    if (!key || !value) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    const std::string k(key), v(value);
    unsigned long long u = 0;
    if (k == "algo") {
        if (v == "auto") g_opt.algo = MSX_ALGO_AUTO;
        else if (v == "1pa_ll") g_opt.algo = MSX_ALGO_1PA_LL;
        else if (v == "2pa_ll") g_opt.algo = MSX_ALGO_2PA_LL;
        else if (v == "2pa_hb") g_opt.algo = MSX_ALGO_2PA_HB;
        else if (v == "2pa_hb_2phase") g_opt.algo = MSX_ALGO_2PA_HB_2PHASE;
        else if (v == "2pr_hb") g_opt.algo = MSX_ALGO_2PR_HB;
        else if (v == "plan_2pa_hb") g_opt.algo = MSX_ALGO_PLAN_2PA_HB;
        else if (v == "plan_2pr_hb") g_opt.algo = MSX_ALGO_PLAN_2PR_HB;
        else if (v == "plan_1pa_ll") g_opt.algo = MSX_ALGO_PLAN_1PA_LL;
        else if (v == "plan_2pa_ll") g_opt.algo = MSX_ALGO_PLAN_2PA_LL;
        else if (v == "2pr_port") g_opt.algo = MSX_ALGO_2PR_PORT;
        else return MSX_ERR_ARG;
        return MSX_OK;
    }
    if (k == "coll_algo") {
        if (v == "auto") g_opt.coll_algo = 0;
        else if (v == "ll") g_opt.coll_algo = 1;
        else if (v == "hb") g_opt.coll_algo = 2;
        else return MSX_ERR_ARG;
        return MSX_OK;
    }
    if (k == "drop_rank") {
        if (v == "-1") { g_opt.drop_rank = -1; return MSX_OK; }
        if (!parse_u64(value, &u) || u >= (unsigned)kMaxRanks) return MSX_ERR_ARG;
        g_opt.drop_rank = (int)u;
        return MSX_OK;
    }
    if (k == "hb_phased_min_bytes" && v == "auto") { g_opt.hb_phased_min = -1; return MSX_OK; }
    if (k == "cache_mode") {
        if (v == "auto") { g_opt.cache_mode = -1; return MSX_OK; }
        if (!parse_u64(value, &u) || u > 2) return MSX_ERR_ARG;
        g_opt.cache_mode = (int)u;
        return MSX_OK;
    }
    if (!parse_u64(value, &u)) return MSX_ERR_ARG;
    if (k == "ll_1pa_max_bytes") g_opt.ll_1pa_max = (size_t)u;
    else if (k == "ll_2pa_max_bytes") g_opt.ll_2pa_max = (size_t)u;
    else if (k == "coll_ll_max_bytes") g_opt.coll_ll_max = (size_t)u;
    else if (k == "a2a_blocks_min_bytes") g_opt.a2a_blocks_min = (size_t)u;
    else if (k == "hb_phased_min_bytes") g_opt.hb_phased_min = u > (unsigned long long)LLONG_MAX ? LLONG_MAX : (long long)u;
    else if (k == "ll_max_bytes") {
        if (u < 4096 || u > (16u << 20)) return MSX_ERR_ARG;
        g_opt.ll_max_bytes = (size_t)u;
    } else if (k == "hb_blocks_per_rank") {
        if (u > (unsigned)kMaxChannels) return MSX_ERR_ARG;
        g_opt.hb_blocks = (int)u;
    } else if (k == "ll_blocks_per_rank") {
        if (u > (unsigned)kMaxChannels) return MSX_ERR_ARG;
        g_opt.ll_blocks = (int)u;
    } else if (k == "threads") {
        if (u > 1024) return MSX_ERR_ARG;
        g_opt.threads = (int)u;
    } else if (k == "hb_unroll") {
        if (u != 0 && u != 1 && u != 2 && u != 4 && u != 8) return MSX_ERR_ARG;
        g_opt.hb_unroll = (int)u;
    } else if (k == "hb_pace") {
        if (u > 1) return MSX_ERR_ARG;
        g_opt.hb_pace = (int)u;
    } else if (k == "hb_barriers") {
        if (u > 1) return MSX_ERR_ARG;
        g_opt.hb_barriers = (int)u;
    } else if (k == "peer_outer") {
        if (u > 2) return MSX_ERR_ARG;
        g_opt.peer_outer = (int)u;
    } else if (k == "barrier_fences") {
        if (u > 3) return MSX_ERR_ARG;
        g_opt.barrier_fences = (int)u;
    } else if (k == "spin_limit") {
        if (u < 1 || u > 0x7fffffffu) return MSX_ERR_ARG;
        g_opt.spin_limit = (unsigned)u;
    } else if (k == "chaos") {
        g_opt.chaos = (unsigned)u;
    } else if (k == "epoch") {
        Ctx* c = nullptr;
        int rc = get_ctx(&c, false);
        if (rc) return rc;
        HIPCHK(hipDeviceSynchronize());
        const unsigned last = (unsigned)u - 1u;   // the next call uses exactly u (or 1 if u is 0)
        HIPCHK(hipMemcpy(c->d.call_state, &last, 4, hipMemcpyHostToDevice));
    } else if (k == "sem_base") {
        Ctx* c = nullptr;
        int rc = get_ctx(&c, false);
        if (rc) return rc;
        HIPCHK(hipDeviceSynchronize());
        const size_t ns = (size_t)kMaxRanks * kMaxRanks * kMaxChannels;
        unsigned* host = (unsigned*)malloc(ns * kSemStrideWords * 4);
        if (!host) return MSX_ERR_NOMEM;
        for (size_t i = 0; i < ns * kSemStrideWords; ++i) host[i] = (unsigned)u;
        hipError_t e1 = hipMemcpy(c->d.sem, host, ns * kSemStrideWords * 4, hipMemcpyHostToDevice);
        hipError_t e2 = hipMemcpy(c->d.expected, host, ns * 4, hipMemcpyHostToDevice);
        hipError_t e3 = hipMemcpy(c->d.gbar, host, kGridBarBytes, hipMemcpyHostToDevice);   // counters and their bases
        free(host);
        HIPCHK(e1);
        HIPCHK(e2);
        HIPCHK(e3);
        HIPCHK(hipDeviceSynchronize());
    } else {
        return MSX_ERR_ARG;
    }
    return MSX_OK;
}

int msx_get_option(const char* key, char* value_out, size_t value_len)
{
    if (!key || !value_out || value_len == 0) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    const std::string k(key);
    unsigned long long u = 0;
    if (k == "algo") {
        static const char* names[] = {"auto", "1pa_ll", "2pa_ll", "2pa_hb", "2pa_hb_2phase", "2pr_hb",
                                      "plan_2pa_hb", "plan_2pr_hb", "plan_1pa_ll", "plan_2pa_ll", "2pr_port"};
        snprintf(value_out, value_len, "%s", names[g_opt.algo]);
        return MSX_OK;
    }
    if (k == "coll_algo") {
        static const char* cn[] = {"auto", "ll", "hb"};
        snprintf(value_out, value_len, "%s", cn[g_opt.coll_algo]);
        return MSX_OK;
    }
    if (k == "drop_rank") { snprintf(value_out, value_len, "%d", g_opt.drop_rank); return MSX_OK; }
    if (k == "ll_1pa_max_bytes") u = g_opt.ll_1pa_max;
    else if (k == "ll_2pa_max_bytes") u = g_opt.ll_2pa_max;
    else if (k == "coll_ll_max_bytes") u = g_opt.coll_ll_max;
    else if (k == "a2a_blocks_min_bytes") u = g_opt.a2a_blocks_min;
    else if (k == "hb_phased_min_bytes") {
        if (g_opt.hb_phased_min < 0) { snprintf(value_out, value_len, "auto"); return MSX_OK; }
        u = (unsigned long long)g_opt.hb_phased_min;
    }
    else if (k == "ll_max_bytes") {
        int dev = 0;
        u = g_opt.ll_max_bytes;
        if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 && g_ctx[dev]) u = g_ctx[dev]->ll_limit;
    } else if (k == "hb_blocks_per_rank") u = (unsigned)g_opt.hb_blocks;
    else if (k == "ll_blocks_per_rank") u = (unsigned)g_opt.ll_blocks;
    else if (k == "threads") u = (unsigned)g_opt.threads;
    else if (k == "hb_unroll") u = (unsigned)g_opt.hb_unroll;
    else if (k == "cache_mode") {
        snprintf(value_out, value_len, "%s", g_opt.cache_mode < 0 ? "auto" : g_opt.cache_mode == 0 ? "0" : g_opt.cache_mode == 1 ? "1" : "2");
        return MSX_OK;
    }
    else if (k == "hb_barriers") u = (unsigned)g_opt.hb_barriers;
    else if (k == "hb_pace") u = (unsigned)g_opt.hb_pace;
    else if (k == "peer_outer") u = (unsigned)g_opt.peer_outer;
    else if (k == "barrier_fences") u = (unsigned)g_opt.barrier_fences;
    else if (k == "spin_limit") u = g_opt.spin_limit;
    else if (k == "chaos") u = g_opt.chaos;
    else if (k == "status_detail") u = g_status_detail;
    else if (k == "epoch") {
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 && g_ctx[dev]) {
            unsigned last = 0;
            HIPCHK(hipDeviceSynchronize());
            HIPCHK(hipMemcpy(&last, g_ctx[dev]->d.call_state, 4, hipMemcpyDeviceToHost));
            u = last;
        }
    } else return MSX_ERR_ARG;
    snprintf(value_out, value_len, "%llu", u);
    return MSX_OK;
}

int msx_status(void* stream, uint32_t info[6])
{
    HIPCHK(hipStreamSynchronize((hipStream_t)stream));
    std::lock_guard<std::mutex> lk(g_mu);
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MSX_ERR_ARG;
    Ctx* c = t_use ? t_use : g_ctx[dev];
    if (c && t_use && (!known_ctx(c) || c->device != dev)) return MSX_ERR_ARG;
    uint32_t h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int rc;
    if (c && (rc = take_status(c, h))) return rc;
    // the fixed context of msx_allreduce_ex_static has a status block of its own
    if (h[0] == 0 && !t_use && g_static[dev] && (rc = take_status(g_static[dev], h))) return rc;
    if (info)
        for (int i = 0; i < 6; ++i) info[i] = h[i];
    if (h[0] != 0) g_status_detail = h[6];
    if (c && c->port && c->port->hip_error.load() != 0) {      // the port's proxy ran into a HIP error: that is the cause
        t_hip_err = c->port->hip_error.load();
        return MSX_ERR_HIP;
    }
    return status_code(h);
}

int msx_debug_choose(size_t nbytes, int nranks, size_t ll_limit, int* algo, int* unroll, int* want_blocks)
{
    if (nranks < 1 || nranks > kMaxRanks || !algo || !unroll || !want_blocks) return MSX_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    *algo = g_opt.algo != MSX_ALGO_AUTO ? g_opt.algo : choose_algo(nbytes, nranks, ll_limit);
    choose_hb_shape(nbytes, nranks, 256, unroll, want_blocks);
    if (*algo == MSX_ALGO_2PA_HB && use_phased(nbytes, nranks, 0)) {
        *unroll = kPhasedHeld;
        *want_blocks = g_opt.hb_blocks > 0 ? g_opt.hb_blocks : kMaxChannels;
    }
    return MSX_OK;
}

int msx_debug_owner_magic(int n_experts, int nranks, uint32_t* magic)
{
    if (!magic || nranks < 1 || nranks > kMaxRanks || n_experts <= 0 || n_experts % nranks) return MSX_ERR_ARG;
    *magic = owner_magic(n_experts, n_experts / nranks);
    return MSX_OK;
}

int msx_debug_pace_update(uint32_t state[4], uint64_t took_ticks, uint32_t tiles)
{
    if (!state || tiles == 0) return MSX_ERR_ARG;
    PaceCtl p{state[0], state[1], state[2], state[3] & 3u, (state[3] >> 8) & 0x1ffu};
    pace_update(p, took_ticks, tiles);
    state[0] = p.pace; state[1] = p.good; state[2] = p.frozen; state[3] = p.misses | (p.age << 8);
    return MSX_OK;
}

int msx_debug_lower_plan_ex(int algo, int nranks, int blocks_per_rank, size_t nbytes, int threads, int held,
                            void* ops_out, size_t ops_capacity, uint32_t* start_out, size_t* ops_written)
{
    if (!plan_algo(algo) || nranks < 2 || nranks > kMaxRanks || blocks_per_rank < 1 ||
        blocks_per_rank > kMaxChannels || threads < 1 || !ops_written || held < 0 || held > 64)
        return MSX_ERR_ARG;
    const bool packets = algo == MSX_ALGO_PLAN_1PA_LL || algo == MSX_ALGO_PLAN_2PA_LL;
    if (packets ? (nbytes % 2 != 0 || held != 0) : (nbytes % (16 * (size_t)nranks) != 0)) return MSX_ERR_ARG;
    if (held && algo != MSX_ALGO_PLAN_2PA_HB) return MSX_ERR_ARG;
    std::vector<PlanOp> ops;
    std::vector<unsigned> start;
    lower_allreduce(algo, nranks, blocks_per_rank, nbytes, threads, held, &ops, &start);
    *ops_written = ops.size();
    if (!ops_out || !start_out) return MSX_OK;           // size query
    if (ops.size() > ops_capacity) return MSX_ERR_NOMEM;
    memcpy(ops_out, ops.data(), ops.size() * sizeof(PlanOp));
    memcpy(start_out, start.data(), start.size() * sizeof(unsigned));
    return MSX_OK;
}

int msx_debug_lower_plan(int algo, int nranks, int blocks_per_rank, size_t vectors_per_rank, int threads,
                         void* ops_out, size_t ops_capacity, uint32_t* start_out, size_t* ops_written)
{
    if (algo != MSX_ALGO_PLAN_2PA_HB && algo != MSX_ALGO_PLAN_2PR_HB) return MSX_ERR_ARG;
    return msx_debug_lower_plan_ex(algo, nranks, blocks_per_rank, vectors_per_rank * 16, threads, 0, ops_out,
                                   ops_capacity, start_out, ops_written);
}

int msx_last_launch(int* grid, int* block, int* algo)
{
    if (grid) *grid = t_grid;
    if (block) *block = t_block;
    if (algo) *algo = t_algo;
    return MSX_OK;
}

int msx_last_hip_error(void) { return t_hip_err; }

const char* msx_strerror(int err)
{
    switch (err) {
        case MSX_OK: return "ok";
        case MSX_ERR_ARG: return "invalid argument";
        case MSX_ERR_UNSUPPORTED: return "unsupported request";
        case MSX_ERR_HIP: return "HIP runtime error";
        case MSX_ERR_TIMEOUT: return "device-side wait timed out";
        case MSX_ERR_NOMEM: return "scratch too small or allocation failed";
        case MSX_ERR_CAPACITY: return "token dispatch receive buffer overflow";
        case MSX_ERR_INDEX: return "token dispatch: expert id out of range";
        default: return "unknown error";
    }
}

const char* msx_version(void) { return "msx 0.2 (gfx950)"; }

}  // extern "C"
