// HB-protocol kernels: two-phase all-pairs AllReduce (fused and two-phase), standalone
// ReduceScatter / AllGather / AllToAll.  Collectives Library section (2PA) and the
// MemoryChannel HB protocol: move large chunks with 16-byte accesses and synchronise once
// per chunk.  One workgroup set per rank; a thread reads the same vector from ALL ranks at
// once (no per-peer synchronisation inside the reduction) and, following the paper's
// note for peer-to-peer meshes, writes to all peers inside the element loop.
//
// Synchronisation policy.  The barrier at the START of a kernel only orders execution
// ("every peer has entered this call, so what earlier launches wrote into its buffers is
// final"): data written by earlier launches is already visible when a launch starts, so that
// barrier carries no fence.  The barrier at the END publishes the puts of this launch; the puts
// are write-through (st16_wt + put_drain), so it needs no L2 write-back either, except in the
// workgroups that also wrote with ordinary stores (a scalar tail, an unaligned byte path).
#pragma once
#include "msx_device.hpp"
#include "msx_hb_common.hpp"

namespace msx {

// ---- fused two-phase all-pairs: reduce chunk `rank` in registers and put it to everyone ----
// (reduce-scatter chunk-sum feeding the all-gather copy with no memory round trip; the
// fused "reduce then put" operation of the DSL's Operation Fusion paragraph, widened from
// two local buffers to all N ranks.)  In place is safe: chunk r of every row is read and
// written by rank r's threads only, and a thread loads all N values before it stores.
// RES: 0 no residual, 1 one residual shared by all ranks, 2 one residual per destination.
// CACHE: 0 streaming loads and stores (large messages), 1 stores may stay in the memory-side cache,
// 2 loads and stores may stay in the caches (the host picks by the call's footprint).
template <int DT, int U, int NR, int RES, int CACHE = 0>
__global__ __launch_bounds__(256) void k_allreduce_hb_fused(HbArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    constexpr size_t epv = DT == 0 ? 4 : 8;
    const size_t V = a.count / epv;

    // Every peer has entered the call.  Unchecked (the checked form costs 0.08 us of a 4 us call): nothing this
    // workgroup reads depends on the peers, so after a timeout here it still stores only finished sums.
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 10, false, false);

    const size_t lo = chunk_begin(V, rank, n);
    const size_t hi = chunk_begin(V, rank + 1, n);
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;

    for (size_t i = lo + rt; i < hi; i += RT * U) {
        u32x4 v[U][kMaxRanks];
        u32x4 res[U][RES == 2 ? kMaxRanks : 1];     // residual vectors, requested together with the inputs
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t idx = i + (size_t)u * RT;
            if (idx < hi) {
#pragma unroll
                for (int j = 0; j < kMaxRanks; ++j)
                    if (j < n_l) v[u][j] = CACHE == 2 ? ld16_keep(a.in[j], idx) : ld16(a.in[j], idx);
                if constexpr (RES == 1) res[u][0] = ld16(a.res[0], idx);
                if constexpr (RES == 2) {
#pragma unroll
                    for (int p = 0; p < kMaxRanks; ++p)
                        if (p < n_l) res[u][p] = ld16(a.res[p], idx);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t idx = i + (size_t)u * RT;
            if (idx < hi) {
                VecAcc<DT> acc;
                MSX_SUM_ALL(acc, v[u])
                if constexpr (RES != 2) {
                    if constexpr (RES == 1) acc.add(res[u][0]);
                    const u32x4 o = acc.pack();
#pragma unroll
                    for (int p = 0; p < kMaxRanks; ++p)
                        if (p < n_l) { if constexpr (CACHE == 0) st16_wt(a.out[p], idx, o); else st16_wt_keep(a.out[p], idx, o); }
                } else {
                    u32x4 o[kMaxRanks];
#pragma unroll
                    for (int p = 0; p < kMaxRanks; ++p)
                        if (p < n_l) {
                            VecAcc<DT> t = acc;
                            t.add(res[u][p]);
                            o[p] = t.pack();
                        }
#pragma unroll
                    for (int p = 0; p < kMaxRanks; ++p)
                        if (p < n_l) { if constexpr (CACHE == 0) st16_wt(a.out[p], idx, o[p]); else st16_wt_keep(a.out[p], idx, o[p]); }
                }
            }
        }
    }
    const bool tail = rank == 0 && chan == 0 && V * epv < a.count;
    if (tail) allreduce_tail<DT>(a, n_l, V * epv, a.count);

    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 11, tail, false);   // my puts have landed everywhere
}

// ---- two-phase form: reduce-scatter to memory, rank barrier, all-gather by put ---------------
template <int DT, int U, int NR>
__global__ __launch_bounds__(256) void k_allreduce_hb_2phase(HbArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n), rank_l = per_lane(rank);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    constexpr size_t epv = DT == 0 ? 4 : 8;
    const size_t V = a.count / epv;

    if (n > 1 && !rank_barrier<true>(c, rank, n, chan, 20, false, false)) return;

    const size_t lo = chunk_begin(V, rank, n);
    const size_t hi = chunk_begin(V, rank + 1, n);
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;

    // phase 1: chunk-sum into my own output
    for (size_t i = lo + rt; i < hi; i += RT * U) {
        u32x4 v[U][kMaxRanks];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t idx = i + (size_t)u * RT;
            if (idx < hi) { MSX_LOAD_ALL(v[u], a.in, idx) }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t idx = i + (size_t)u * RT;
            if (idx < hi) {
                VecAcc<DT> acc;
                MSX_SUM_ALL(acc, v[u])
                if (a.has_res) acc.add(ld16(a.res[0], idx));   // shared residual only (host checks)
                st16(a.out[rank], idx, acc.pack());
            }
        }
    }

    // phase boundary: every rank has finished reading the inputs, so an in-place all-gather may
    // overwrite them.  No data changes hands here (a thread re-reads only what it wrote itself).
    if (n > 1 && !rank_barrier<true>(c, rank, n, chan, 21, false, false)) return;   // a peer is missing: no puts

    // phase 2: put my reduced chunk into every peer's output
    if (a.peer_outer) {
        const char* src = (const char*)a.out[rank] + lo * 16;
        for (int k = 1; k < n; ++k) {
            int p = rank + k; if (p >= n) p -= n;
            hb_put((char*)a.out[p] + lo * 16, src, (hi - lo) * 16, rt, RT);
        }
    } else {
        for (size_t idx = lo + rt; idx < hi; idx += RT) {
            u32x4 o = ld16(a.out[rank], idx);
            settle(o);
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l && p != rank_l) st16_wt(a.out[p], idx, o);
        }
    }
    if (rank == 0 && chan == 0) allreduce_tail<DT>(a, n_l, V * epv, a.count);

    // phase 1 and hb_put use ordinary streaming stores: this form releases for real
    put_drain();
    if (n > 1) rank_barrier(c, rank, n, chan, 22, true, false);
}

// ---- standalone ReduceScatter: out[r][k] = sum_j in[j][r*c + k], k < c = count ---------------
// a.count is c (elements per block); a.in[j] is rank j's full row; a.out[r] points at the c
// results of rank r.  vec != 0 when c*elemsize is a multiple of 16 (so every block is
// 16-byte aligned); otherwise an element-wise path is used.
template <int DT, int U>
__global__ __launch_bounds__(256) void k_reducescatter_hb(HbArgs a, DevCtx c, int vec)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    constexpr size_t epv = DT == 0 ? 4 : 8;
    constexpr size_t esz = DT == 0 ? 4 : 2;
    if (a.barriers && n > 1 && !rank_barrier<true>(c, rank, n, chan, 30, false, false)) return;
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;
    const size_t blk = a.count;
    if (vec) {
        const size_t cv = blk / epv;
        const void* src[kMaxRanks];
#pragma unroll
        for (int j = 0; j < kMaxRanks; ++j) src[j] = j < n ? (const char*)a.in[j] + (size_t)rank * blk * esz : nullptr;
        for (size_t i = rt; i < cv; i += RT * U) {
            u32x4 v[U][kMaxRanks];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t idx = i + (size_t)u * RT;
                if (idx < cv) { MSX_LOAD_ALL(v[u], src, idx) }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t idx = i + (size_t)u * RT;
                if (idx < cv) {
                    VecAcc<DT> acc;
                    MSX_SUM_ALL(acc, v[u])
                    st16(a.out[rank], idx, acc.pack());
                }
            }
        }
    } else {
        for (size_t k = rt; k < blk; k += RT) {
            const size_t e = (size_t)rank * blk + k;
            float acc = load_elem<DT>(a.in[0], e);
            for (int j = 1; j < n; ++j) acc += load_elem<DT>(a.in[j], e);
            store_elem<DT>(a.out[rank], k, acc);
        }
    }
    // peers are done reading my input; my result is local, nothing to publish
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 31, false, false);
}

// ---- standalone AllGather: out[p] block r = in[r]; a.count = bytes per block ------------------
// Put-based: rank r reads its block once and writes it into every rank's output (peer loop
// inside the element loop).  A destination equal to the source (in-place) is skipped.
// KEEP: the stores may stay in the memory-side cache (blocks whose copies all fit into it)
template <int U, int KEEP = 0>
__global__ __launch_bounds__(256) void k_allgather_hb(HbArgs a, DevCtx c, int vec)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;
    const size_t nbytes = a.count;
    const char* src = (const char*)a.in[rank];
    char* dst[kMaxRanks];
    int skip = -1;                       // the destination that is the source itself (in place)
#pragma unroll
    for (int p = 0; p < kMaxRanks; ++p) {
        dst[p] = p < n ? (char*)a.out[p] + (size_t)rank * nbytes : nullptr;
        if (p < n && dst[p] == src) skip = p;
    }
    const int skip_l = per_lane(skip);
    if (vec) {
        const size_t nv = nbytes >> 4;
        for (size_t i = rt; i < nv; i += RT * U) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t iu = i + (size_t)u * RT;
                if (iu < nv) v[u] = ld16(src, iu);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) settle(v[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t iu = i + (size_t)u * RT;
                if (iu < nv) {
#pragma unroll
                    for (int p = 0; p < kMaxRanks; ++p)
                        if (p < n_l && p != skip_l) { if constexpr (KEEP) st16_wt_keep(dst[p], iu, v[u]); else st16_wt(dst[p], iu, v[u]); }
                }
            }
        }
    } else {
        for (size_t b = rt; b < nbytes; b += RT) {
            const char v = src[b];
            for (int p = 0; p < n; ++p)
                if (dst[p] != src) dst[p][b] = v;
        }
    }
    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 40, !vec, false);   // my block has landed everywhere
}

// ---- standalone AllToAll (out of place): out[d] block s = in[s] block d; a.count = bytes/block ---
// Two orders.  Small blocks (latency): the peer loop inside the vector loop, every thread loads the same vector
// of all n blocks and stores to all n destinations at once.  Large blocks (a.peer_outer): block after block,
// rank r starting with its own (destination r, r+1, ...), U vectors per thread in flight: at any moment every
// source reads one block and every destination is written by one source, 8 read and 8 write streams over the
// chip instead of 64 each; with a.peer_outer == 2 the ranks meet at a rank barrier after every block, so that
// they stay in step.  Measured at 8 x 256 MiB rows: peer loop inside 5.17-5.33 TB/s, block after block 5.40-5.46,
// in step 5.51-5.55 TB/s (128 workgroups per rank or more).
template <int KEEP>
__global__ __launch_bounds__(256) void k_alltoall_hb(HbArgs a, DevCtx c, int vec)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;
    const size_t nbytes = a.count;
    const char* src = (const char*)a.in[rank];
    if (vec && a.peer_outer) {
        constexpr int U = 8;
        const size_t nv = nbytes >> 4;
        for (int k = 0; k < n; ++k) {
            int d = rank + k; if (d >= n) d -= n;
            const char* sp = src + (size_t)d * nbytes;
            char* dp = (char*)a.out[d] + (size_t)rank * nbytes;
            for (size_t i = rt; i < nv; i += RT * U) {
                u32x4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (i + (size_t)u * RT < nv) v[u] = ld16(sp, i + (size_t)u * RT);
#pragma unroll
                for (int u = 0; u < U; ++u) settle(v[u]);
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (i + (size_t)u * RT < nv) {
                        if constexpr (KEEP) st16_wt_keep(dp, i + (size_t)u * RT, v[u]);
                        else st16_wt(dp, i + (size_t)u * RT, v[u]);
                    }
            }
            if (a.peer_outer == 2 && n > 1) { put_drain(); rank_barrier(c, rank, n, chan, 51, false, false); }
        }
    } else if (vec) {
        const size_t nv = nbytes >> 4;
        for (size_t i = rt; i < nv; i += RT) {
            u32x4 v[kMaxRanks];
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (d < n_l) v[d] = ld16(src + (size_t)d * nbytes, i);
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d) settle(v[d]);
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (d < n_l) {
                    if constexpr (KEEP) st16_wt_keep((char*)a.out[d] + (size_t)rank * nbytes, i, v[d]);
                    else st16_wt((char*)a.out[d] + (size_t)rank * nbytes, i, v[d]);
                }
        }
    } else {
        for (int d = 0; d < n; ++d) {
            char* dp = (char*)a.out[d] + (size_t)rank * nbytes;
            const char* sp = src + (size_t)d * nbytes;
            for (size_t b = rt; b < nbytes; b += RT) dp[b] = sp[b];
        }
    }
    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 50, !vec, false);
}

// ---- AllToAll in place: block (s,d) and block (d,s) swap through registers --------------------
// For a pair s<d the lower rank swaps the first half of the vectors and the higher rank the
// second half, so each vector of each pair is loaded and stored by exactly one thread.
__global__ __launch_bounds__(256) void k_alltoall_inplace(HbArgs a, DevCtx c, int vec)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    if (a.barriers && n > 1 && !rank_barrier<true>(c, rank, n, chan, 60, false, false)) return;
    const size_t RT = (size_t)a.chans * blockDim.x;
    const size_t rt = (size_t)chan * blockDim.x + threadIdx.x;
    const size_t nbytes = a.count;
    const size_t units = vec ? (nbytes >> 4) : nbytes;
    const size_t half = units / 2;
    for (int k = 1; k < n; ++k) {
        int peer = rank + k; if (peer >= n) peer -= n;
        const size_t lo = rank < peer ? 0 : half;
        const size_t hi = rank < peer ? half : units;
        char* mine = (char*)a.out[rank] + (size_t)peer * nbytes;
        char* theirs = (char*)a.out[peer] + (size_t)rank * nbytes;
        if (vec) {
            for (size_t i = lo + rt; i < hi; i += RT) {
                const u32x4 x = ld16(mine, i);
                const u32x4 y = ld16(theirs, i);
                st16_wt(mine, i, y);
                st16_wt(theirs, i, x);
            }
        } else {
            for (size_t b = lo + rt; b < hi; b += RT) {
                const char x = mine[b], y = theirs[b];
                mine[b] = y;
                theirs[b] = x;
            }
        }
    }
    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 61, !vec, false);
}

// ---- two-phase ring (2PR) over the MemoryChannel ---------------------------------------------------
// Collectives Library section, 2PR, and the overlapped ring reduce-scatter example of the DSL
// section: n chunks travel around the ring; in the reduce-scatter phase a rank adds its own
// values to the partial sum it received and passes it on (fused reduce-then-put, so the partial
// never goes through local memory), in the all-gather phase it forwards finished chunks.  Every
// hop is a real put -> signal || wait -> read hand-off: puts are write-through, the wait acquires.
// The partial sum travels in the element type, i.e. it is rounded at every hop; chunk k is
// summed in the order k, k+1, ..., k-1 (mod n).  The paper's version runs over the DMA engine
// and splits chunks in halves to overlap copy and reduction; with thread copies the same
// threads do both, so there is nothing to overlap and chunks are not split.  Inside one chip a
// ring moves 5(n-1)/n S bytes per rank against 2 S for all-pairs: this path is for comparison.
struct RingArgs {
    const void* in[kMaxRanks];
    void* out[kMaxRanks];
    void* scratch[kMaxRanks];   // per rank: n chunks of partial sums received from the previous rank
    size_t chunk_vecs;          // 16-byte vectors per chunk
    int n;
    int chans;
};

template <int DT>
__global__ __launch_bounds__(256) void k_allreduce_ring(RingArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    const int next = rank + 1 == n ? 0 : rank + 1;
    const int prev = rank == 0 ? n - 1 : rank - 1;
    const size_t cv = a.chunk_vecs;
    const size_t lo = cv * (size_t)chan / (size_t)a.chans, hi = cv * (size_t)(chan + 1) / (size_t)a.chans;
    const size_t tid = threadIdx.x, bd = blockDim.x;

    if (!rank_barrier<true>(c, rank, n, chan, 70, false, false)) return;   // everybody is done with the previous call's scratch

    // step 0: my own chunk starts its trip
    for (size_t i = lo + tid; i < hi; i += bd) {
        const size_t idx = (size_t)rank * cv + i;
        st16_wt(a.scratch[next], idx, ld16(a.in[rank], idx));
    }
    put_drain();
    channel_signal(c, rank, next, chan, 71, false);

    // reduce-scatter: n-1 hops; the last one produces my finished chunk and starts the all-gather
    for (int s = 0; s + 1 < n; ++s) {
        int j = rank - 1 - s; if (j < 0) j += n;
        const bool last = s + 2 == n;
        if (!channel_wait(c, rank, prev, chan, 72)) return;   // the partial sum never came: pass nothing on
        for (size_t i = lo + tid; i < hi; i += 2 * bd) {       // two vectors per thread in flight
            const size_t idx = (size_t)j * cv + i, idx1 = idx + bd;
            const bool two = i + bd < hi;
            const u32x4 p0 = ld16(a.scratch[rank], idx), m0 = ld16(a.in[rank], idx);
            u32x4 p1 = p0, m1 = m0;
            if (two) { p1 = ld16(a.scratch[rank], idx1); m1 = ld16(a.in[rank], idx1); }
            VecAcc<DT> a0, a1;
            a0.set(p0); a0.add(m0);
            a1.set(p1); a1.add(m1);
            const u32x4 o0 = a0.pack(), o1 = a1.pack();
            if (last) {
                st16(a.out[rank], idx, o0);
                st16_wt(a.out[next], idx, o0);
                if (two) { st16(a.out[rank], idx1, o1); st16_wt(a.out[next], idx1, o1); }
            } else {
                st16_wt(a.scratch[next], idx, o0);
                if (two) st16_wt(a.scratch[next], idx1, o1);
            }
        }
        put_drain();
        channel_signal(c, rank, next, chan, 73, false);
    }

    // all-gather: n-1 chunks arrive from the previous rank; all but the last are passed on
    for (int s = 0; s + 1 < n; ++s) {
        int j = rank - s; if (j < 0) j += n;
        if (!channel_wait(c, rank, prev, chan, 74)) return;
        if (s + 2 < n) {
            for (size_t i = lo + tid; i < hi; i += bd) {
                const size_t idx = (size_t)j * cv + i;
                st16_wt(a.out[next], idx, ld16(a.out[rank], idx));
            }
            put_drain();
            channel_signal(c, rank, next, chan, 75, false);
        }
    }
}

}  // namespace msx
