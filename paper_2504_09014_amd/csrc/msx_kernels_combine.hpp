// The combine (the way back of the token dispatch) in chip-wide read and write phases.
//
// Same result as k_moe_combine: out[s][t] = the rows token t of source s was sent to, summed in fp32 in
// ascending destination order starting from the first, rounded once.  The output of a source rank is walked in
// dealt tiles exactly like the token array in k_moe_pack_dealt (rows are whole multiples of 64 vectors, so the 64
// vectors of a wave lie in one row); a round is a read phase in which every thread sums H tiles into registers,
// a chip-wide barrier, and a short write phase, as in the phased reduce-scatter, whose traffic mix this has.
//
// A tile has between zero and eight source rows.  Its eight loads are issued without any condition all the
// same, so that their number is fixed and the loads of the next tiles stay in flight while a tile is summed:
// they are buffer loads, and a row that does not exist gets an offset beyond the buffer, which the hardware
// answers with zeros without touching memory.  The zeros are turned into -0.0 before they are added
// (x + -0.0 = x for every x, signed zeros and NaNs included), so the sum is the sum over the rows that exist;
// a token that went nowhere gives +0.0 as in k_moe_combine.  Row offsets and the bitmap of rows that exist are
// worked out once per round, lane h for tile h, and read lane by lane.
#pragma once
#include "msx_hb_common.hpp"
#include "msx_moe_common.hpp"

namespace msx {

constexpr unsigned kCombineAbsent = 0xF0000000u;     // an offset no destination buffer reaches (the host checks)

template <int DT, int H>
__global__ __launch_bounds__(256) void k_moe_combine_dealt(MoeArgs a, DevCtx c)
{
    constexpr int G = 2, HG = H / G;
    static_assert(H % (2 * G) == 0 && H <= 64, "unrolled in pairs of groups; one lane per held tile");
    constexpr unsigned kSign = DT == 0 ? 0x80000000u : 0x80008000u;
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    if (n > 1 && !rank_barrier<true>(c, rank, n, chan, 220, false, false)) return;   // every peer's rows are final
    GridBar gb = grid_barrier_begin(c);
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave_first = __builtin_amdgcn_readfirstlane(threadIdx.x & ~63u);
    const unsigned rv = a.row_vecs;
    const unsigned nv = (unsigned)a.T * rv;                       // a multiple of 256, below 2^32 (the host checks)
    const unsigned tiles = nv / 256u;
    const unsigned per_round = (unsigned)a.chans * (unsigned)H;
    const unsigned rounds = (tiles + per_round - 1u) / per_round;
    unsigned base[kMaxRanks];
    __amdgpu_buffer_rsrc_t rs[kMaxRanks];
#pragma unroll
    for (int d = 0; d < kMaxRanks; ++d) {
        base[d] = a.base[rank * 8 + d];
        rs[d] = __builtin_amdgcn_make_buffer_rsrc(a.recv[d < n ? d : 0], 0, (int)(a.cap * rv * 16u), 0x00020000);
    }
    char* out = (char*)a.tokens[rank];
    const unsigned short* slots = a.slots + (size_t)rank * a.T * 8;
    const unsigned tstep = (unsigned)a.chans * 256u;              // vectors between two of my tiles
    const unsigned lane_bytes = lane * 16u;
    unsigned gen = 0;

    for (unsigned round = 0; round < rounds; ++round) {
        const unsigned first = round * per_round + (unsigned)chan;
        const unsigned left = first >= tiles ? 0u : (tiles - first + (unsigned)a.chans - 1u) / (unsigned)a.chans;
        const unsigned mine = left < (unsigned)H ? left : (unsigned)H;
        const unsigned v0 = first * 256u + wave_first;            // the wave's first vector in my first tile
        // lane h: where the wave's share of tile h starts in each destination's buffer, and which rows exist
        unsigned off[kMaxRanks], exist = 0u;
        {
            const unsigned v = v0 + lane * tstep;
            const unsigned t = v / rv, col = v - t * rv;
            u32x4 pk = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
            if (lane < mine) pk = *(const u32x4*)(slots + (size_t)t * 8);
            const unsigned row[kMaxRanks] = {pk.x & 0xffffu, pk.x >> 16, pk.y & 0xffffu, pk.y >> 16,
                                             pk.z & 0xffffu, pk.z >> 16, pk.w & 0xffffu, pk.w >> 16};
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d) {
                const unsigned r = base[d] + row[d];
                const bool go = d < n && row[d] != 0xffffu && r < a.cap;
                off[d] = go ? (r * rv + col) * 16u : kCombineAbsent;
                exist |= go ? 1u << d : 0u;
            }
        }
        u32x4 held[H];
        u32x4 va[G][kMaxRanks], vb[G][kMaxRanks];
        auto issue = [&](auto all, int g, u32x4 (&v)[G][kMaxRanks]) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int h = g * G + i;
                if (decltype(all)::value || (unsigned)h < mine) {
#pragma unroll
                    for (int d = 0; d < kMaxRanks; ++d) {
                        const unsigned o = (unsigned)__builtin_amdgcn_readlane((int)off[d], h);
                        v[i][d] = __builtin_amdgcn_raw_buffer_load_b128(rs[d], (int)(o + lane_bytes), 0, 2);   // streaming
                    }
                }
            }
        };
        auto reduce = [&](auto all, int g, u32x4 (&v)[G][kMaxRanks]) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int h = g * G + i;
                if (decltype(all)::value || (unsigned)h < mine) {
                    const unsigned bits = (unsigned)__builtin_amdgcn_readlane((int)exist, h);
                    const unsigned sign = bits ? kSign : 0u;          // a token that went nowhere: +0.0
                    VecAcc<DT> acc;
#pragma unroll
                    for (int d = 0; d < kMaxRanks; ++d) {
                        const unsigned m = (bits >> d) & 1u ? 0u : sign;
                        const u32x4 x = {v[i][d].x | m, v[i][d].y | m, v[i][d].z | m, v[i][d].w | m};
                        if (d == 0) acc.set(x); else acc.add(x);
                    }
                    held[h] = acc.pack();
                }
            }
        };
        auto read_phase = [&](auto all) {
            constexpr bool A = decltype(all)::value;
            const int nq = (int)((mine + G - 1) / G);
            if (A || 0 < nq) issue(all, 0, va);
            static_for<HG / 2>([&](auto k) {
                constexpr int g = 2 * decltype(k)::value;
                if (A || g + 1 < nq) issue(all, g + 1, vb);
                if (A || g < nq) reduce(all, g, va);
                if (g + 2 < HG && (A || g + 2 < nq)) issue(all, g + 2, va);
                if (A || g + 1 < nq) reduce(all, g + 1, vb);
            });
        };
        if (mine == (unsigned)H) read_phase(std::true_type{});
        else read_phase(std::false_type{});
        static_for<H>([&](auto k) { settle(held[decltype(k)::value]); });
        grid_barrier(c, gb, ++gen, (unsigned)rank, 222);
        // write phase: my own output only, written through so that the stores reach memory in this phase and not
        // under the next read phase; short, so nobody waits behind it
        static_for<H>([&](auto k) {
            constexpr unsigned h = (unsigned)decltype(k)::value;
            if (h < mine) st16_wt_keep_at(out + ((size_t)v0 + (size_t)h * tstep) * 16, lane_bytes, held[h]);
        });
        put_drain();
    }
    grid_barrier_end(c, gb, gen);
    if (n > 1) rank_barrier(c, rank, n, chan, 221, false, false);   // peers are done reading my rows
}

}  // namespace msx
