// HB-protocol kernels that alternate, over the whole chip, between a read phase and a write phase: the fused
// two-phase all-pairs AllReduce (Collectives Library section, 2PA with the DSL's fused reduce-then-put), its
// reduce-scatter half on its own, and the all-gather copy.  Compiled in a translation unit of their own
// (msx_phased*.hip): each instantiation is tens of thousands of instructions long.
#pragma once
#include "msx_device.hpp"
#include "msx_hb_common.hpp"

namespace msx {

// Launches with fewer rounds than this do not pace their write phases (see k_allreduce_hb_phased).  One round is
// enough: a paced launch ends with a barrier behind its last write phase, so that this phase is measured too,
// and the schedule a launch finds is kept for the next launch of its shape.
constexpr unsigned kPacedRounds = 1;

// ---- the fused form with the whole chip alternating between reading and writing ---------------
// Same result, same bytes and the same owner-computes layout as k_allreduce_hb_fused, for messages far
// larger than the caches.  HBM runs a pure read stream or a pure write stream faster than any mix of the
// two (measured on MI355X: 8 input streams alone 6.4-7.0 TB/s, stores alone 5.6-6.4 TB/s, every mix from
// 8:1 to 1:1 5.2-5.4 TB/s), so the launch works in rounds: every thread sums H vectors of its rank's chunk
// into registers (read phase), all workgroups meet at a barrier, every thread puts its H sums to all ranks
// (write phase), barrier.  A phase moves H x 16 B x 8 ranks x (threads of the launch) bytes, about 0.5 GB
// at H = 64: more than the memory-side cache holds, so DRAM itself sees the alternation (phases of a few
// tens of MB, tried with a plain copy, gave nothing).  One workgroup per CU (the sums take most of the
// register file); loads run two groups of G vectors x N ranks ahead.
// RES: 0 no residual, 1 one residual shared by all ranks (one more input stream).
// KIND: 0 AllReduce (a.count = elements per rank), 1 ReduceScatter on its own (a.count = elements per
// block, whole vectors; the sums go to the rank's own output only: the write phase is an eighth of the read
// phase, and keeping even that out of the reads pays.  Measured at 256 MiB rows: plain stores, which leave the
// second-level cache under the next read phase, 5.6-5.8 TB/s; write-through stores 6.0-6.2 TB/s; no barrier
// behind the write phase another 1 %).
template <int DT, int NR, int RES, int H, int KIND = 0>
__global__ __launch_bounds__(256) void k_allreduce_hb_phased(HbArgs a, DevCtx c)
{
    constexpr int G = 2, HG = H / G, NS = kMaxRanks + (RES ? 1 : 0);
    static_assert(H % (2 * G) == 0, "the read phase is unrolled in pairs of groups");
    static_assert(KIND == 0 || RES == 0, "the reduce-scatter takes no residual");
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    constexpr size_t epv = DT == 0 ? 4 : 8;
    constexpr size_t esz = DT == 0 ? 4 : 2;
    const size_t V = a.count / epv;

    GridBar gb = grid_barrier_begin(c);
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, KIND ? 32 : 12, false, false);   // every peer has entered the call (unchecked, as in k_allreduce_hb_fused)

    // the vectors [lo, hi) of every source belong to this rank
    const void* src[kMaxRanks];
#pragma unroll
    for (int j = 0; j < kMaxRanks; ++j)
        src[j] = j >= n ? nullptr : KIND ? (const void*)((const char*)a.in[j] + (size_t)rank * a.count * esz) : a.in[j];
    const size_t lo = KIND ? 0 : chunk_begin(V, rank, n);
    const size_t hi = KIND ? V : chunk_begin(V, rank + 1, n);
    const size_t tiles = (hi - lo) / 256;                // whole tiles; a tile: one vector per thread of the workgroup
    size_t most = tiles;                                 // every workgroup runs as many rounds as the longest chunk needs
    if constexpr (KIND == 0) {
        most = 0;
        for (int r = 0; r < n; ++r) {
            const size_t t = (chunk_begin(V, r + 1, n) - chunk_begin(V, r, n)) / 256;
            most = t > most ? t : most;
        }
    }
    const size_t per_round = (size_t)a.chans * H;
    const unsigned rounds = (unsigned)((most + per_round - 1) / per_round);
    const bool pacing = a.pace && rounds >= kPacedRounds;
    unsigned gen = 0;
    // what the schedule is remembered under from call to call: the shape of the launch
    // (the rank count is part of the shape: four ranks put to half as many destinations per tile as eight, and a
    // schedule inherited from an 8-rank call of the same size was met, hence kept, and 50 % too slow)
    const unsigned key = ((unsigned)a.count ^ (unsigned)(a.count >> 32)) * 2654435761u + gridDim.x * 64u + (unsigned)(DT * 8 + RES * 2 + KIND) + 1u + (unsigned)n * 7919u * 128u;
    PaceCtl ctl = pace_load(c, key);   // every workgroup reads it; workgroup 0 keeps it up to date
    unsigned pace = pacing ? ctl.pace : 0u;   // wall-clock ticks between the puts of two tiles in a full write phase (0: unpaced)
    // Tiles of a round: the AllReduce deals them out one by one (workgroup c of the rank takes every chans-th),
    // so that at any moment the 32 workgroups of a rank write one compact window of each output; with H
    // consecutive tiles per workgroup the write phase was 15 % slower (2048 separate streams over the chip,
    // against 64 windows).  The read-heavy reduce-scatter keeps consecutive tiles (its reads are 5 % faster so).
    constexpr bool kDealt = KIND == 0;
    const size_t tstep = kDealt ? (size_t)a.chans * 256 : (size_t)256;
    auto put = [&](size_t idx, u32x4 o) {
        if constexpr (KIND == 1) {
            st16_wt_keep(a.out[rank], idx, o);           // my own output; written through, so that the stores reach
                                                         // memory in this phase and not under the next read phase
        } else {
#pragma unroll
            for (int p = 0; p < kMaxRanks; ++p)
                if (p < n_l) st16_wt(a.out[p], idx, o);
        }
    };

    for (unsigned round = 0; round < rounds; ++round) {
        // my first tile of this round, and how many of my H tiles exist (all, but for a chunk's last round)
        const size_t first = kDealt ? (size_t)round * per_round + (size_t)chan : ((size_t)round * a.chans + (size_t)chan) * H;
        const size_t every = kDealt ? (size_t)a.chans : (size_t)1;
        const size_t left = first >= tiles ? 0 : (tiles - first + every - 1) / every;
        const unsigned mine = (unsigned)(left < (size_t)H ? left : (size_t)H);
        const int nq = (int)((mine + G - 1) / G);
        const size_t i0 = lo + first * 256 + threadIdx.x;
        u32x4 held[H];
        u32x4 va[G][NS], vb[G][NS];
        // all: the workgroup has all H tiles this round (every round but a chunk's last): no conditions at all,
        // so that the loads of the next groups stay in flight while a group is summed
        auto issue = [&](auto all, int g, u32x4 (&v)[G][NS]) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const size_t idx = i0 + (size_t)(g * G + i) * tstep;
                if (decltype(all)::value || (unsigned)(g * G + i) < mine) {     // uniform: whole tiles only
                    MSX_LOAD_ALL(v[i], src, idx)
                    if constexpr (RES == 1) v[i][kMaxRanks] = ld16(a.res[0], idx);
                }
            }
        };
        auto reduce = [&](int g, u32x4 (&v)[G][NS]) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                VecAcc<DT> acc;
                MSX_SUM_ALL(acc, v[i])
                if constexpr (RES == 1) acc.add(v[i][kMaxRanks]);
                held[g * G + i] = acc.pack();
            }
        };
        // read phase (static_for: the sums must stay in registers, so every index into `held` is a constant;
        // a loop this long is beyond what the unrolling pragma is honoured for)
        auto read_phase = [&](auto all) {
            constexpr bool A = decltype(all)::value;
            if (A || 0 < nq) issue(all, 0, va);
            static_for<HG / 2>([&](auto k) {
                constexpr int g = 2 * decltype(k)::value;
                if (A || g + 1 < nq) issue(all, g + 1, vb);
                if (A || g < nq) reduce(g, va);
                if (g + 2 < HG && (A || g + 2 < nq)) issue(all, g + 2, va);
                if (A || g + 1 < nq) reduce(g + 1, vb);
            });
        };
        if constexpr (NR != 0) {
            if (mine == (unsigned)H) read_phase(std::true_type{});
            else read_phase(std::false_type{});
        } else {
            read_phase(std::false_type{});     // rank count at run time: the second copy would not fit the registers
        }
        grid_barrier(c, gb, ++gen, (unsigned)rank, 13);
        // write phase.  The dies do not get equal shares of the store bandwidth (in one phase the fastest is done
        // after 45 us, the slowest after 70 us, and which is which changes from phase to phase), and the last
        // dies alone cannot fill the memory system.  So a full write phase is paced: tile h goes out no earlier
        // than h x pace after the phase began (PaceCtl picks the pace).  Fast dies are held to the common
        // schedule, the slow ones get the bandwidth that frees, and all finish together; the schedule can then
        // be tightened well below what an unpaced phase takes (measured at 1 GiB per rank: 96 us unpaced,
        // 75 us paced).
        if constexpr (NR != 0 && KIND == 0) {
            if (pacing && round > 0)       // workgroup 0's decision after the previous round
                pace = pace_clamp(__hip_atomic_load(c.gbar + kGridBarPaceWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
        const unsigned long long w0 = wall_clock64();
        auto write_phase = [&](auto all) {
            static_for<H>([&](auto k) {
                constexpr int h = decltype(k)::value;
                if constexpr (decltype(all)::value) {
                    if constexpr (KIND == 0) wait_until(w0 + (unsigned long long)((unsigned)h * pace));
                    put(i0 + (size_t)h * tstep, held[h]);
                } else if ((unsigned)h < mine) {
                    // a chunk's last round: the tiles are dealt out, so every workgroup has (nearly) as many,
                    // and the schedule per tile holds for it too
                    if constexpr (KIND == 0 && NR != 0) wait_until(w0 + (unsigned long long)((unsigned)h * pace));
                    put(i0 + (size_t)h * tstep, held[h]);
                }
            });
        };
        if constexpr (NR != 0) {
            if (mine == (unsigned)H) write_phase(std::true_type{});
            else write_phase(std::false_type{});
        } else {
            write_phase(std::false_type{});
        }
        put_drain();
        // the reduce-scatter goes straight on: its write phase is short, and nothing but the shape of the traffic
        // depends on its barriers (a workgroup reads inputs and writes its own tiles only)
        if ((round + 1 < rounds && KIND == 0) || (NR != 0 && KIND == 0 && pacing)) {
            grid_barrier(c, gb, ++gen, (unsigned)rank, 14);
            if constexpr (NR != 0 && KIND == 0) {
                if (pacing && blockIdx.x == 0) {     // workgroup 0 of rank 0, channel 0: its rounds are full to the end
                    if (mine >= (unsigned)H / 4) pace_update(ctl, wall_clock64() - w0, mine);   // also from a partial round
                    if (threadIdx.x == 0) st32_wt(c.gbar + kGridBarPaceWord, ctl.pace);
                }
            }
        }
    }
    grid_barrier_end(c, gb, gen);
    if constexpr (NR != 0 && KIND == 0) {
        if (pacing && blockIdx.x == 0 && threadIdx.x == 0) pace_save(c, ctl, key);
    }
    // what is left of the chunk behind its last whole tile (less than one vector per thread): the rank's first workgroup
    if (chan == 0) {
        const size_t idx = lo + tiles * 256 + threadIdx.x;
        if (idx < hi) {
            u32x4 v[NS];
            MSX_LOAD_ALL(v, src, idx)
            if constexpr (RES == 1) v[kMaxRanks] = ld16(a.res[0], idx);
            VecAcc<DT> acc;
            MSX_SUM_ALL(acc, v)
            if constexpr (RES == 1) acc.add(v[kMaxRanks]);
            put(idx, acc.pack());
        }
    }
    bool tail = false;
    if constexpr (KIND == 0) {
        tail = rank == 0 && chan == 0 && V * epv < a.count;
        if (tail) allreduce_tail<DT>(a, n_l, V * epv, a.count);
    }
    put_drain();
    // AllReduce: my puts have landed everywhere; ReduceScatter: the peers are done reading my input
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, KIND ? 33 : 11, tail, false);
}

// ---- standalone AllGather in chip-wide read and write phases ------------------------------------
// out[p] block r = in[r] as k_allgather_hb does (a.count = bytes per block, whole vectors).  The write phase
// is eight times the read phase; what the phases buy is that the stores run without loads between them.
// The stores carry no streaming hint: measured at 1 GiB rows 5.4-5.5 TB/s against 5.1-5.2 TB/s with it (the
// AllReduce's write phase shows no such difference).
template <int NR, int H>
__global__ __launch_bounds__(256) void k_allgather_hb_phased(HbArgs a, DevCtx c)
{
    const int n = NR ? NR : a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = NR ? NR : per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    GridBar gb = grid_barrier_begin(c);
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
    const size_t nv = nbytes >> 4, tiles = nv / 256;
    const size_t per_round = (size_t)a.chans * H;
    const unsigned rounds = (unsigned)((tiles + per_round - 1) / per_round);
    const bool pacing = a.pace && rounds >= kPacedRounds;
    unsigned gen = 0;
    const unsigned key = ((unsigned)a.count ^ (unsigned)(a.count >> 32)) * 2654435761u + gridDim.x * 64u + 32u + 1u + (unsigned)n * 7919u * 128u;
    PaceCtl ctl = pace_load(c, key);
    unsigned pace = pacing ? ctl.pace : 0u;   // wall-clock ticks between the puts of two tiles (0: unpaced)
    const size_t tstep = (size_t)a.chans * 256;      // tiles dealt out one by one, as in the AllReduce
    auto put = [&](size_t idx, u32x4 o) {
#pragma unroll
        for (int p = 0; p < kMaxRanks; ++p)
            if (p < n_l && p != skip_l) st16_wt_keep(dst[p], idx, o);
    };
    for (unsigned round = 0; round < rounds; ++round) {
        const size_t first = (size_t)round * per_round + (size_t)chan;
        const size_t left = first >= tiles ? 0 : (tiles - first + (size_t)a.chans - 1) / (size_t)a.chans;
        const unsigned mine = (unsigned)(left < (size_t)H ? left : (size_t)H);
        const size_t i0 = first * 256 + threadIdx.x;
        u32x4 held[H];
        static_for<H>([&](auto k) {
            constexpr int h = decltype(k)::value;
            if ((unsigned)h < mine) held[h] = ld16(src, i0 + (size_t)h * tstep);
        });
        static_for<H>([&](auto k) { settle(held[decltype(k)::value]); });
        grid_barrier(c, gb, ++gen, (unsigned)rank, 43);
        // paced like the AllReduce's write phase
        if (pacing && round > 0)
            pace = pace_clamp(__hip_atomic_load(c.gbar + kGridBarPaceWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        const unsigned long long w0 = wall_clock64();
        static_for<H>([&](auto k) {
            constexpr int h = decltype(k)::value;
            if ((unsigned)h < mine) {
                wait_until(w0 + (unsigned long long)((unsigned)h * pace));     // partial last rounds too: dealt tiles
                put(i0 + (size_t)h * tstep, held[h]);
            }
        });
        put_drain();
        if (round + 1 < rounds || pacing) {
            grid_barrier(c, gb, ++gen, (unsigned)rank, 44);
            if (pacing && blockIdx.x == 0) {
                if (mine >= (unsigned)H / 4) pace_update(ctl, wall_clock64() - w0, mine);
                if (threadIdx.x == 0) st32_wt(c.gbar + kGridBarPaceWord, ctl.pace);
            }
        }
    }
    if (pacing && blockIdx.x == 0 && threadIdx.x == 0) pace_save(c, ctl, key);
    grid_barrier_end(c, gb, gen);
    if (chan == 0) {
        const size_t idx = tiles * 256 + threadIdx.x;
        if (idx < nv) {
            u32x4 v = ld16(src, idx);
            settle(v);
            put(idx, v);
        }
    }
    put_drain();
    if (a.barriers && n > 1) rank_barrier(c, rank, n, chan, 40, false, false);   // my block has landed everywhere
}

}  // namespace msx
