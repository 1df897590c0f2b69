/*
 * msx - collective data-movement kernels for N emulated ranks inside ONE MI355X.
 *
 * The N "GPUs" of the paper are N rank buffers in this GPU's HBM; rank r's work is done
 * by the workgroups b with b % N == r of a single kernel launch, and ranks talk to each
 * other only through device-scope flags in HBM (semaphores and LL packet flags).
 *
 * General rules for every entry point
 *   - C ABI, no exceptions, never exits.  Returns MSX_OK (0) or a negative msx_error.
 *   - Every `void* stream` is a hipStream_t (NULL = the default stream).  Calls enqueue
 *     work on that stream and return without waiting for it (the first call on a device
 *     also allocates the library's scratch and semaphores, which blocks once).
 *   - Data pointers are DEVICE pointers, 16-byte aligned, owned by the caller and kept
 *     alive until the stream has run the call.  Pointer TABLES (`const void* const*`)
 *     are HOST arrays of `nranks` device pointers; they are read during the call only.
 *   - nranks is 1..8.  count == 0 is a successful no-op.
 *   - Every call runs on a CONTEXT: the flag epoch, the semaphores and their expected values,
 *     the LL scratch.  Without further ado that is the device's default context, created by
 *     msx_init or the first call; msx_ctx_create makes more (the communicator objects of the
 *     paper's NCCL-shaped Collective API, Overview section) and msx_ctx_use selects the one
 *     the calling thread's calls run on.  All calls on ONE context must be issued on one
 *     stream or be ordered by the caller; calls on different contexts are independent and may
 *     run concurrently on different streams (see the co-residency rule below).  The state
 *     lives in device memory and is advanced by the kernels, so calls may be captured into a
 *     HIP graph and replayed (create the context before capturing).
 *   - Warm-up: the first call on a device creates the default context, and the first call of a
 *     new shape may grow scratch (ring scratch, a lowered plan, the built-in routing plan of
 *     the token dispatch): those calls allocate and wait for the device, so they must not
 *     happen during stream capture.  msx_prepare_* does all of that ahead of time; msx_run
 *     never allocates and never waits.
 *   - CO-RESIDENCY (a hard precondition).  The ranks of a call wait for each other inside ONE
 *     launch, so all its workgroups must be on the GPU at the same time.  Every launch is
 *     sized to what the otherwise idle GPU can hold, or to the context's budget
 *     (msx_ctx_set_max_blocks).  Work that occupies compute units next to a call (another
 *     stream's kernels, a second context) may keep some of its workgroups from starting; the
 *     call then times out instead of completing.  Callers that overlap contexts give each a
 *     budget such that the budgets add up to no more than the GPU holds (256 workgroups of the
 *     large-message kernels, one per compute unit).
 *   - A device-side wait that does not finish within the spin budget makes its workgroup
 *     record {rank, site, expected, seen}; a workgroup whose wait guards data it was about
 *     to consume (packets, a partial sum, a peer's rows) stops there, so no output element is
 *     ever built from data that did not arrive.  After a timeout the outputs of that call are
 *     incomplete (partly written).  Nothing hangs.  The timeout is latched in the context: every later
 *     call on it returns MSX_ERR_TIMEOUT without launching anything, until the status has been
 *     read (msx_status, msx_last_status) or the context reset (msx_reset, msx_ctx_reset; do
 *     reset: semaphore counts are out of step after a timeout).
 */
#ifndef MSX_H
#define MSX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* fp32 and bf16 sums run on the tuned kernels of every algorithm.  fp16, int32, and max / min for any
 * type, are served by AllReduce (automatic or MSX_ALGO_2PA_HB, no residual) and ReduceScatter through a
 * generic kernel; the copy collectives and the token dispatch move any 2- or 4-byte type; the combine
 * sums fp32 and bf16 only.
 * Floating point: sum = fp32 accumulation in rank order, one rounding; max / min = fp32 comparison in
 * rank order, the earlier value is kept unless the later one is strictly greater / smaller.
 * int32: sum modulo 2^32 (two's complement wrap-around), max / min signed. */
typedef enum { MSX_F32 = 0, MSX_BF16 = 1, MSX_F16 = 2, MSX_I32 = 3 } msx_dtype;
typedef enum { MSX_SUM = 0, MSX_MAX = 1, MSX_MIN = 2 } msx_op;

typedef enum {
    MSX_OK = 0,
    MSX_ERR_ARG = -1,          /* null / misaligned pointer, bad nranks, bad count, bad dtype */
    MSX_ERR_UNSUPPORTED = -2,  /* valid request this build does not implement */
    MSX_ERR_HIP = -3,          /* a HIP runtime call failed (msx_last_hip_error has the code) */
    MSX_ERR_TIMEOUT = -4,      /* a device-side wait ran out of its spin budget */
    MSX_ERR_NOMEM = -5,        /* scratch too small for the request / allocation failed */
    MSX_ERR_CAPACITY = -6,     /* token dispatch: a destination buffer overflowed */
    MSX_ERR_INDEX = -7         /* token dispatch: an expert id outside [0, n_experts) */
} msx_error;

/* AllReduce algorithms (Collectives Library section: one-phase and two-phase all-pairs). */
typedef enum {
    MSX_ALGO_AUTO = 0,      /* pick by message size */
    MSX_ALGO_1PA_LL = 1,    /* one-phase all-pairs over LL packets */
    MSX_ALGO_2PA_LL = 2,    /* two-phase all-pairs over LL packets, rotating scratch */
    MSX_ALGO_2PA_HB = 3,    /* two-phase all-pairs, HB protocol, reduce and put fused in registers */
    MSX_ALGO_2PA_HB_2PHASE = 4, /* same, but reduce-scatter to memory, barrier, all-gather put */
    MSX_ALGO_2PR_HB = 5,    /* two-phase ring over put/signal/wait hand-offs; count*elemsize must be a
                               multiple of 16*nranks, no residual.  Partial sums travel in the element
                               type (rounded at every hop) and chunk k is summed in the order k, k+1, ...,
                               so results differ from the other algorithms in the last bits.  The first
                               call of a new size (re)allocates the ring scratch and blocks. */
    MSX_ALGO_PLAN_2PA_HB = 6, /* MSX_ALGO_2PA_HB run by the generic plan-interpreter kernel (the paper's */
    MSX_ALGO_PLAN_2PR_HB = 7, /* Executor): same results as the hand-written kernel; count*elemsize must be a
                               multiple of 16*nranks, no residual; the first call of a shape lowers and uploads
                               the plan (blocks).  Large messages (where MSX_ALGO_2PA_HB runs in chip-wide read
                               and write phases) are lowered to that schedule too. */
    MSX_ALGO_PLAN_1PA_LL = 8, /* MSX_ALGO_1PA_LL and MSX_ALGO_2PA_LL run by the same interpreter from packet */
    MSX_ALGO_PLAN_2PA_LL = 9, /* operations (put packets, reduce packets, copy packets): any even byte count within
                               the LL limit, no residual. */
    MSX_ALGO_2PR_PORT = 10  /* the two-phase ring over the PortChannel, as in the paper's overlapped ring example:
                               every chunk travels in two halves, copied by the port (FIFO in host memory, CPU proxy,
                               runtime device-to-device copies) while the rank's threads reduce the other half.  Same
                               sums, same order and rounding as MSX_ALGO_2PR_HB (bit-identical results); same size
                               rule, no residual.  The proxy thread is told of every launch, so the call can be
                               neither prepared nor captured into a graph (MSX_ERR_UNSUPPORTED), and the stream must
                               not share a hardware queue with the proxy's own stream (a non-blocking stream the
                               library creates on first use; the null stream and torch's streams are fine). */
} msx_algo;

/* ------------------------------------------------------------------------------------
 * Collectives in the paper's problem statement (Background, "Collective Communications").
 * These four take ONE rank-major contiguous device buffer and work IN PLACE.
 * ---------------------------------------------------------------------------------- */

/* AllReduce: buf is [nranks][count], any count; afterwards every row holds the elementwise sum
 * of the rows.  Sum is taken in fp32 in rank order 0..nranks-1 and rounded once.  Rows whose
 * size is not a multiple of 16 bytes do not start on 16-byte boundaries and go through an
 * element-by-element kernel (correct, not fast). */
int msx_allreduce(void* buf, size_t count, int dtype, int op, int nranks, void* stream);

/* ReduceScatter: buf is [nranks][count], count % nranks == 0, c = count / nranks.
 * Afterwards elements [r*c, (r+1)*c) of row r hold the sum over rows of that range;
 * every other element is left as it was. */
int msx_reducescatter(void* buf, size_t count, int dtype, int op, int nranks, void* stream);

/* AllGather: buf is [nranks][nranks*count]; on entry row r holds its contribution in
 * elements [r*count, (r+1)*count); afterwards every row is the concatenation.  op ignored. */
int msx_allgather(void* buf, size_t count, int dtype, int op, int nranks, void* stream);

/* AllToAll (equal blocks): buf is [nranks][count], count % nranks == 0, c = count/nranks.
 * Afterwards block s of row d holds what block d of row s held.  op ignored. */
int msx_alltoall(void* buf, size_t count, int dtype, int op, int nranks, void* stream);

/* ------------------------------------------------------------------------------------
 * Out-of-place forms with one pointer per rank (send[r], recv[r] are rank r's buffers).
 * send[r] == recv[r] is allowed for allreduce and reducescatter-with-full-rows only.
 * ---------------------------------------------------------------------------------- */

/* AllReduce, optionally fused with a residual add (tensor-parallel decode epilogue):
 * recv[r][i] = round( fp32 sum_j send[j][i] (rank order) + fp32 residual[r][i] ).
 * residual may be NULL (no add); its entries may all be the same pointer.
 * algo is an msx_algo.  LL algorithms need count*elemsize <= the LL limit (msx_get_option
 * "ll_max_bytes"), else MSX_ERR_NOMEM. */
int msx_allreduce_ex(const void* const* send, void* const* recv, const void* const* residual,
                     size_t count, int dtype, int op, int nranks, int algo, void* stream);

/* msx_allreduce_ex for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, same kernels; but the
 * semaphores, the call state and the LL scratch it works on are a fixed array inside the library's code
 * object (about 6.2 MiB, which every GPU the library runs on holds until the process ends), and the call
 * itself makes no hipMalloc / hipFree and uses no allocating routine.
 *   Limits: count*elemsize <= 16 MiB per rank (else MSX_ERR_NOMEM); the LL algorithms <= 64 KiB per rank
 *   (1PA-LL <= 16 KiB), else MSX_ERR_NOMEM; MSX_ALGO_2PR_HB and the MSX_ALGO_PLAN_* forms, whose scratch
 *   grows on demand, are refused with MSX_ERR_UNSUPPORTED; the "algo" option does not apply (pass algo).
 *   The array is set up (address looked up, cleared once) by msx_init or by the first such call on a
 *   device; that first call waits for the device and therefore must not happen during stream capture
 *   (then MSX_ERR_UNSUPPORTED: run msx_init before capturing).
 *   Every call on a GPU shares that GPU's array and its flag epoch: issue these calls on one stream or
 *   order them yourself; calls that overlap on one GPU race.  They are independent of the calls that
 *   use the allocated context, and msx_status / msx_reset cover both. */
int msx_allreduce_ex_static(const void* const* send, void* const* recv, const void* const* residual,
                            size_t count, int dtype, int op, int nranks, int algo, void* stream);

/* ReduceScatter: send[r] is [count]; recv[r] is [count/nranks] = sum_j send[j][r*c + k]. */
int msx_reducescatter_ex(const void* const* send, void* const* recv, size_t count, int dtype,
                         int op, int nranks, void* stream);

/* AllGather: send[r] is [count]; recv[r] is [nranks*count], block j = send[j]. */
int msx_allgather_ex(const void* const* send, void* const* recv, size_t count, int dtype,
                     int nranks, void* stream);

/* AllToAll: send[r], recv[r] are [count], count % nranks == 0; recv[d] block s = send[s] block d.
 * send and recv must not overlap. */
int msx_alltoall_ex(const void* const* send, void* const* recv, size_t count, int dtype,
                    int nranks, void* stream);

/* ------------------------------------------------------------------------------------
 * Token-routed all-to-all (expert-parallel dispatch, the setting of the paper's DeepEP
 * experiment: hidden 7168, top-8 of 256 experts).  Expert e lives on rank
 * e / (n_experts / nranks).  Each token row goes ONCE to every distinct rank that owns one
 * of its K experts.  recv_tokens[d] is filled by source rank ascending, then token index
 * ascending.
 *   tokens[s]        device [T][H] elements of dtype (H*elemsize % 16 == 0)
 *   topk_idx[s]      device [T][K] int32 expert ids, 0 <= id < n_experts
 *   recv_tokens[d]   device [recv_capacity_tokens][H]
 *   recv_src_token[d] device [recv_capacity_tokens] int32 = s*T + t of each row, or the
 *                    whole table may be NULL
 *   recv_counts      device [nranks dst][nranks src] int32 (rows received per source)
 *   plan             a routing plan (msx_moe_plan_create) in which the call leaves where every
 *                    token went, for the msx_moe_combine that follows; NULL = the context's
 *                    built-in plan, which a later dispatch overwrites (and regrows, blocking,
 *                    when T grows)
 * Rows that would exceed recv_capacity_tokens are dropped and msx_status() then reports
 * MSX_ERR_CAPACITY; recv_counts still holds the true counts.  An expert id outside
 * [0, n_experts) sends its token nowhere on that id's account (the other ids of the token
 * count as usual) and msx_status() reports MSX_ERR_INDEX with info[4] = the id.
 * T <= 65534, K <= 32.
 * ---------------------------------------------------------------------------------- */
int msx_moe_dispatch(const void* const* tokens, const int32_t* const* topk_idx, int T, int H,
                     int K, int n_experts, int dtype, int nranks, void* const* recv_tokens,
                     int32_t* const* recv_src_token, int32_t* recv_counts,
                     size_t recv_capacity_tokens, void* plan, void* stream);

/* Routing plans: device memory for the slots of up to max_tokens_per_rank tokens of each of 8
 * ranks (16 bytes per token), owned by `ctx` (NULL = the calling thread's current context) and
 * freed with it or by msx_moe_plan_destroy.  A dispatch with more tokens than the plan was made
 * for returns MSX_ERR_NOMEM.  Both calls allocate / free and wait for the device. */
int msx_moe_plan_create(void* ctx, int max_tokens_per_rank, void** plan);
int msx_moe_plan_destroy(void* plan);

/* The same dispatch with FP8 quantisation fused into the packing (the paper's setting is "FP8
 * dispatch and BF16 combine"): tokens are bf16 [T][H], H % 128 == 0.  Each row is quantised in
 * groups of 128 elements: amax = max(|x|, 1e-4), q = E4M3(x * (448 / amax)) (OCP E4M3, round to
 * nearest even, saturating at 448), scale = amax / 448, all in fp32.
 *   recv_q[d]       device [recv_capacity_tokens][H] bytes
 *   recv_scales[d]  device [recv_capacity_tokens][H/128] float
 * Everything else as in msx_moe_dispatch; msx_moe_combine may follow it. */
int msx_moe_dispatch_fp8(const void* const* tokens, const int32_t* const* topk_idx, int T, int H,
                         int K, int n_experts, int nranks, void* const* recv_q,
                         float* const* recv_scales, int32_t* const* recv_src_token,
                         int32_t* recv_counts, size_t recv_capacity_tokens, void* plan, void* stream);

/* Combine, the way back of msx_moe_dispatch (the paper's expert-parallel experiment runs
 * "dispatch and combine").  Uses the routing the last dispatch through `plan` left there (NULL: the
 * context's built-in plan, i.e. the last dispatch without a plan), which must have had the same T
 * and nranks (else MSX_ERR_ARG).
 *   expert_out[d]  device [capacity_tokens][H]: one processed row per row destination d received,
 *                  in the order the dispatch delivered them
 *   out_tokens[s]  device [T][H]: out[s][t] = round( sum over the destination ranks of token (s,t),
 *                  ascending, in fp32 starting from the first, of its row in expert_out[d] )
 * Rows the dispatch dropped for lack of capacity are left out of the sum. */
int msx_moe_combine(const void* const* expert_out, void* const* out_tokens, int T, int H, int dtype,
                    int nranks, size_t capacity_tokens, void* plan, void* stream);

/* ------------------------------------------------------------------------------------
 * Prepared calls (Overview and Primitive API sections: channels are set up once, on the host, at
 * initialisation; the kernels only run the data path).  msx_prepare_* does everything the matching
 * call does on the host - argument checks, algorithm and launch shape, argument blocks, scratch
 * (ring scratch and lowered plans belong to the handle) - and launches nothing; msx_run(handle,
 * stream) enqueues the kernels and nothing else: no allocation, no lock, no wait.  The handle is
 * bound to the context current at prepare time, to the pointers given (the tables are read during
 * prepare only) and to the options and test hooks in force then; it dies with its context.
 * msx_run returns MSX_ERR_TIMEOUT while a timeout is latched in that context.  Token dispatch and
 * combine need an explicit plan here.  msx_release waits for the device if the handle owns scratch.
 * ---------------------------------------------------------------------------------- */
int msx_prepare_allreduce(const void* const* send, void* const* recv, const void* const* residual,
                          size_t count, int dtype, int op, int nranks, int algo, void** handle);
int msx_prepare_reducescatter(const void* const* send, void* const* recv, size_t count, int dtype,
                              int op, int nranks, void** handle);
int msx_prepare_allgather(const void* const* send, void* const* recv, size_t count, int dtype,
                          int nranks, void** handle);
int msx_prepare_alltoall(const void* const* send, void* const* recv, size_t count, int dtype,
                         int nranks, void** handle);
int msx_prepare_moe_dispatch(const void* const* tokens, const int32_t* const* topk_idx, int T, int H,
                             int K, int n_experts, int dtype, int nranks, void* const* recv_tokens,
                             int32_t* const* recv_src_token, int32_t* recv_counts,
                             size_t recv_capacity_tokens, void* plan, void** handle);
int msx_prepare_moe_combine(const void* const* expert_out, void* const* out_tokens, int T, int H,
                            int dtype, int nranks, size_t capacity_tokens, void* plan, void** handle);
int msx_run(void* handle, void* stream);
int msx_release(void* handle);

/* ------------------------------------------------------------------------------------
 * MemoryChannel primitives on their own (Primitive API figure and MemoryChannel section:
 * put / signal / wait / flush, LL put / read).  Small kernels that exercise exactly one
 * primitive pair between two emulated ranks; used by tests and by the latency table.
 * ---------------------------------------------------------------------------------- */

/* signal/wait ping-pong: workgroup block_a and workgroup block_b of a `grid_blocks`-wide
 * launch bounce a semaphore `iters` times.  ns_out (device, 1 double) = ns per round trip. */
int msx_prim_pingpong(int iters, int grid_blocks, int block_a, int block_b, double* ns_out,
                      void* stream);

/* `rounds` all-to-all barriers among nranks x blocks_per_rank workgroups (every rank signals
 * all peers, then waits on all peers).  sem_out (device, [nranks][nranks] uint32, nullable)
 * receives how far each semaphore of channel 0 advanced during the call. */
int msx_prim_barrier(int rounds, int nranks, int blocks_per_rank, uint32_t* sem_out, void* stream);

/* HB hand-off: rank 0 put()s src -> staging with 16-byte copies and signals; rank 1 waits,
 * then copies staging -> dst.  All three are device buffers of nbytes (any size). */
int msx_prim_put_signal_wait(const void* src, void* staging, void* dst, size_t nbytes,
                             int blocks_per_rank, void* stream);

/* Plain streams, the yardstick for the bandwidth kernels (no passage of the paper: a measurement aid).
 * mode 0 reads nbytes from src, 1 writes nbytes to dst, 2 copies src -> dst, with `blocks` workgroups of 256
 * threads and streaming 16-byte accesses.  src, dst: device, 16-byte aligned (the unused one may be NULL);
 * nbytes a multiple of 16.  Mode 1 fills dst with a pattern of no meaning. */
int msx_prim_stream(int mode, const void* src, void* dst, size_t nbytes, int blocks, void* stream);

/* PortChannel hand-off (port-mapped I/O, emulated): rank 0 pushes put(src -> staging), signal and
 * flush requests into a FIFO in host memory; a CPU proxy thread of the library carries them out
 * (hipMemcpyAsync device to device on its own stream; the signal is a one-wave kernel behind the copy
 * on that stream, which bumps rank 1's device-side semaphores; the flush is reported once an event
 * behind the copy has fired); rank 1 waits on its semaphores, then copies staging -> dst with its
 * threads.  The first call starts the proxy thread and allocates the FIFOs (blocks once).  If the
 * proxy runs into a HIP error it stops copying and signalling (the waiters time out) and msx_status
 * returns MSX_ERR_HIP. */
int msx_prim_port_put_signal_wait(const void* src, void* staging, void* dst, size_t nbytes, void* stream);

/* LL encode only: write ceil(nbytes/8) 16-byte packets {w0, flag, w1, flag} for src into
 * packets_out (device, 16-byte aligned, 16*ceil(nbytes/8) bytes). */
int msx_prim_ll_encode(const void* src, size_t nbytes, uint32_t flag, void* packets_out,
                       void* stream);

/* LL hand-off: rank 0 encodes src into the library scratch with the current flag, rank 1
 * polls every packet until both flags match and writes the payload to dst. */
int msx_prim_ll_roundtrip(const void* src, void* dst, size_t nbytes, int blocks_per_rank,
                          void* stream);

/* ------------------------------------------------------------------------------------
 * Context, options, status
 * ---------------------------------------------------------------------------------- */

/* Create the current device's default context now (otherwise the first call does), and set up the
 * fixed array msx_allreduce_ex_static works on. */
int msx_init(void);

/* Re-zero scratch, semaphores and the flag epoch of the calling thread's current context (and, when
 * that is the default one, of the fixed array too); clears a latched timeout.  Synchronises the device. */
int msx_reset(void);

/* Free the current device's default context.  Synchronises the device. */
int msx_finalize(void);

/* Context handles (the Collective API is NCCL-shaped: collectives run on communicator objects).
 * msx_ctx_create: a new context on the current device; nranks (1..8) = the most ranks a call on it
 * will have; max_ll_bytes = largest per-rank message of the LL algorithms (4 KiB .. 16 MiB; 0 = the
 * "ll_max_bytes" option).  Allocates about 4 MiB + 64 x max_ll_bytes and waits for the device.
 * msx_ctx_use: the calling thread's calls run on ctx from now on (NULL: back to the default context).
 * msx_ctx_set_max_blocks: no launch of this context takes more workgroups than that (0 = what the idle
 * GPU holds); see the co-residency rule at the top.
 * msx_ctx_reset / msx_ctx_destroy: as msx_reset / msx_finalize, for one context (NULL = the current
 * one, for reset).  Destroying a context invalidates its prepared calls and routing plans.
 * msx_last_status: the device-side status of ctx (NULL = current), read and cleared WITHOUT waiting:
 * call it after the stream in question has been synchronised.  Returns MSX_OK, MSX_ERR_TIMEOUT,
 * MSX_ERR_CAPACITY or MSX_ERR_INDEX; the out pointers may be NULL. */
int msx_ctx_create(int nranks, size_t max_ll_bytes, void** ctx);
int msx_ctx_destroy(void* ctx);
int msx_ctx_reset(void* ctx);
int msx_ctx_use(void* ctx);
int msx_ctx_set_max_blocks(void* ctx, int max_blocks);
int msx_last_status(void* ctx, int* rank, int* site, unsigned* expected, unsigned* seen);

/* Options (strings; numbers in decimal):
 *   "algo"            auto | 1pa_ll | 2pa_ll | 2pa_hb | 2pa_hb_2phase | 2pr_hb | plan_2pa_hb | plan_2pr_hb |
 *                     plan_1pa_ll | plan_2pa_ll | 2pr_port   (for the in-place forms)
 *   "ll_1pa_max_bytes", "ll_2pa_max_bytes"   size thresholds of the automatic choice
 *   "coll_algo"       auto | ll | hb   protocol of allgather / reducescatter (LL needs blocks that
 *                     are multiples of 8 bytes and fit the LL scratch; "ll" fails otherwise)
 *   "coll_ll_max_bytes"   auto: LL up to this many bytes per block
 *   "ll_max_bytes"    largest per-rank message the LL scratch is sized for (set before init)
 *   "hb_blocks_per_rank", "ll_blocks_per_rank", "threads"   0 = automatic
 *   "hb_unroll"       0 (by size) | 1 | 2 | 4 | 8 (8: AllGather only)   vectors in flight per thread
 *   "cache_mode"      auto | 0 | 1 | 2   fused HB AllReduce: 0 streaming loads and stores, 1 stores may stay in
 *                     the memory-side cache, 2 loads too; auto picks by the footprint of the call
 *   "hb_phased_min_bytes"   auto | bytes per rank from which the fused HB AllReduce (no residual, or one
 *                     shared by all ranks) runs in chip-wide read and write phases, one workgroup per CU; auto:
 *                     8 ranks from 40 MiB (per rank; rows, for ReduceScatter / AllGather), the AllReduce of 4 to 7
 *                     ranks without a residual from 64 MiB and of 3 ranks from 128 MiB, the AllGather of 3 to 7
 *                     ranks from 128 MiB rows and of 2 ranks from 256 MiB rows, never otherwise; an
 *                     explicit value applies to every rank count.  The token pack of msx_moe_dispatch and
 *                     msx_moe_combine have such a form for rows of whole multiples of 1 KiB (the combine also needs
 *                     T x H to be a whole number of 4 KiB tiles): auto from 32 MiB of tokens per rank (8 ranks)
 *   "hb_pace"         0 | 1   phased kernels: hold the write phases to a common wall-clock schedule, so that all
 *                     dies finish them together (the schedule is found by the kernels themselves and kept, per
 *                     launch shape, in the context)
 *   "hb_barriers"     0 | 1   start/end rank barriers in the HB kernels
 *   "peer_outer"      0 | 1 | 2   two-phase HB all-gather: one put per peer instead of peer-inner (1); out-of-place
 *                     all-to-all: 0 = by block size (block after block with the ranks in step from 4 MiB blocks, the
 *                     peer loop inside below), 1 / 2 = block after block at any size, without / with the rank
 *                     barrier between blocks
 *   "a2a_blocks_min_bytes"  that block size (default 4 MiB; a huge value keeps the peer loop inside at any size)
 *   "barrier_fences"  0..3    msx_prim_barrier only: bit 0 release fence, bit 1 acquire fence
 *   "spin_limit"      polls before a wait gives up
 *   "drop_rank"       -1, or a rank whose workgroups return at once (failure-path tests)
 *   "chaos"           0, or a seed: workgroups sleep pseudo-random times before they signal
 *   "epoch"           next LL flag value (tests of wrap-around; synchronises the device)
 *   "sem_base"        set every semaphore and expected value, and the counters of the chip-wide barrier, to
 *                     this number (wrap tests; syncs)
 * Read-only (msx_get_option): "status_detail" = for the last timeout msx_status() reported from a packet
 * poll, the source rank whose packet was still missing.
 * Unknown key or bad value -> MSX_ERR_ARG. */
int msx_set_option(const char* key, const char* value);
int msx_get_option(const char* key, char* value_out, size_t value_len);

/* Wait for `stream`, then report and clear the device-side status of the calling thread's current
 * context (a latched timeout included).  info (nullable) gets {code, rank, site, expected, seen,
 * block}.  Returns MSX_OK, MSX_ERR_TIMEOUT, MSX_ERR_CAPACITY or MSX_ERR_INDEX. */
int msx_status(void* stream, uint32_t info[6]);

/* Name and launch shape of the kernel the last call on this thread launched
 * (for profiles): grid blocks, block threads, algorithm chosen. */
int msx_last_launch(int* grid, int* block, int* algo);

/* Host logic on its own (no device is touched; usable on a machine without a GPU).
 * msx_debug_choose: what the automatic choice would run for `nbytes` per rank given an LL scratch
 * sized for ll_limit bytes, and the HB launch shape (unroll, wanted workgroups per rank; for the phased form
 * the sums a thread holds per phase, and 256 = as many workgroups as are resident).
 * msx_debug_lower_plan(_ex): the execution plan the interpreter algorithms run.  ops_out receives
 * 128-byte records {int code, peer, flags, nsrc, ndst; {int16 kind, rank} src[9], dst[8]; int dst_wt;
 * uint32 aux; uint64 first, end, step; uint32 aux2, aux3} (see csrc/msx_kernels_plan.hpp), start_out the
 * nranks*blocks_per_rank+1 list offsets.  With ops_out == NULL only *ops_written is set.  The _ex form takes
 * the message size in bytes per rank, any plan algorithm, and `held` (0, or the sums a thread holds per
 * phase: MSX_ALGO_PLAN_2PA_HB is then lowered to the read phase / write phase schedule). */
int msx_debug_choose(size_t nbytes, int nranks, size_t ll_limit, int* algo, int* unroll, int* want_blocks);
/* One step of the controller that paces the write phases of the phased kernels: state = {pace, last pace that
 * was met, frozen, misses in a row | phases met since frozen << 8} (pace in 10 ns ticks per tile, 0 = unpaced); took_ticks = how long the
 * full write phase of `tiles` tiles just took.  The same function the kernels call. */
int msx_debug_pace_update(uint32_t state[4], uint64_t took_ticks, uint32_t tiles);
/* The multiplier with which the token plan computes the owner rank of an expert, e / (n_experts / nranks), as
 * the high word of e * magic; 0 = it divides. */
int msx_debug_owner_magic(int n_experts, int nranks, uint32_t* magic);
int msx_debug_lower_plan(int algo, int nranks, int blocks_per_rank, size_t vectors_per_rank, int threads,
                         void* ops_out, size_t ops_capacity, uint32_t* start_out, size_t* ops_written);
int msx_debug_lower_plan_ex(int algo, int nranks, int blocks_per_rank, size_t nbytes, int threads, int held,
                            void* ops_out, size_t ops_capacity, uint32_t* start_out, size_t* ops_written);

int msx_last_hip_error(void);
const char* msx_strerror(int err);
const char* msx_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MSX_H */
