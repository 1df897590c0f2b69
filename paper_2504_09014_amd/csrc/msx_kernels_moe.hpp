// Token-routed all-to-all (expert-parallel dispatch).  The paper evaluates this exchange
// in its DeepEP experiment (hidden 7168, top-8 of 256 experts) but does not describe the
// packing; the order built here is: destination buffer d holds rows by source rank
// ascending, then by token index ascending, one row per (token, distinct destination).
//
//   plan  : one workgroup per source rank.  Marks each token's destination ranks, turns
//           the marks into stable per-destination slots with a workgroup prefix sum,
//           exchanges the 8 per-destination counts with all peers over LL packets, and
//           derives where this source's rows start inside every destination buffer.
//   pack  : many workgroups per rank, one wave per token: the row is read once and put
//           into every destination (peer loop inside the row loop), then a rank barrier.
#pragma once
#include "msx_device.hpp"
#include "msx_moe_common.hpp"

namespace msx {


constexpr int kPlanThreads = 1024;

// workgroup-wide exclusive prefix sum of two packed counters (4 x 16-bit fields each)
__device__ __forceinline__ void block_exscan2(unsigned long long& x, unsigned long long& y,
                                              unsigned long long* lds, unsigned long long& tx,
                                              unsigned long long& ty)
{
    const int lane = (int)(threadIdx.x & 63u), wave = (int)(threadIdx.x >> 6);
    unsigned long long ix = x, iy = y;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        unsigned long long ux = __shfl_up(ix, d, 64), uy = __shfl_up(iy, d, 64);
        if (lane >= d) { ix += ux; iy += uy; }
    }
    if (lane == 63) { lds[wave * 2] = ix; lds[wave * 2 + 1] = iy; }
    __syncthreads();
    unsigned long long bx = 0, by = 0, sx = 0, sy = 0;
    const int nw = (int)(blockDim.x >> 6);
    for (int w = 0; w < nw; ++w) {
        if (w == wave) { bx = sx; by = sy; }
        sx += lds[w * 2]; sy += lds[w * 2 + 1];
    }
    tx = sx; ty = sy;                  // totals
    x = bx + ix - x; y = by + iy - y;  // exclusive
    __syncthreads();
}

__global__ __launch_bounds__(kPlanThreads) void k_moe_plan(MoeArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)blockIdx.x;           // one workgroup per source rank
    const CallTag tag = call_begin(c);
    if (rank == c.drop_rank) { call_end(c, tag); return; }
    __shared__ unsigned long long scan_lds[2 * (kPlanThreads / 64)];
    __shared__ unsigned cnt[kMaxRanks][kMaxRanks];   // [src][dst]
    const int T = a.T, K = a.K;
    const int per_thread = (T + (int)blockDim.x - 1) / (int)blockDim.x;
    const int t0 = (int)threadIdx.x * per_thread;
    const int t1 = min(T, t0 + per_thread);
    const int* topk = a.topk[rank];

    // destination marks of a token: one bit per rank that owns one of its K experts; an id outside
    // [0, n_experts) marks nothing and is reported (the call goes on without it).  The owner of expert e is
    // e / per_rank: by multiplication (a division by a run-time value is some thirty instructions, and every
    // thread does dozens of them: 10 of the kernel's 17 us at 4096 tokens and 8 experts per token)
    int bad_id = 0;
    bool bad = false;
    const unsigned magic = a.per_rank_magic;
    auto owner = [&](int e) -> unsigned { return magic ? __umulhi((unsigned)e, magic) : (unsigned)(e / a.per_rank); };
    auto marks = [&](int t) -> unsigned {
        unsigned mask = 0;
        if (K == 8) {                                    // the common case: two 16-byte loads per token
            const u32x4 lo = *(const u32x4*)(topk + (size_t)t * 8), hi = *(const u32x4*)(topk + (size_t)t * 8 + 4);
            const int e[8] = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (e[k] >= 0 && e[k] < a.n_experts) mask |= 1u << owner(e[k]);
                else { bad = true; bad_id = e[k]; }
        } else {
            for (int k = 0; k < K; ++k) {
                const int e = topk[(size_t)t * K + k];
                if (e >= 0 && e < a.n_experts) mask |= 1u << owner(e);
                else { bad = true; bad_id = e; }
            }
        }
        return mask;
    };

    // pass 1: my tokens' destination marks, counted per destination (16-bit fields); the marks of the
    // first few tokens stay in registers for pass 2
    constexpr int kKeep = 8;
    unsigned kept[kKeep];
    unsigned long long cx = 0, cy = 0;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const int t = t0 + i;
        kept[i] = t < t1 ? marks(t) : 0u;
    }
    for (int t = t0; t < t1; ++t) {
        const int i = t - t0;
        unsigned mask = 0;
        if (i < kKeep) {
#pragma unroll
            for (int q = 0; q < kKeep; ++q) mask = q == i ? kept[q] : mask;
        } else {
            mask = marks(t);
        }
        for (int d = 0; d < 4; ++d) {
            cx += (unsigned long long)((mask >> d) & 1u) << (16 * d);
            cy += (unsigned long long)((mask >> (d + 4)) & 1u) << (16 * d);
        }
    }
    if (bad) report(c, kStatusBadIndex, (unsigned)rank, 202u, (unsigned)a.n_experts, (unsigned)bad_id);
    unsigned long long totx, toty;
    block_exscan2(cx, cy, scan_lds, totx, toty);   // cx, cy now hold the slots my first token gets

    // pass 2: stable slots
    unsigned short* slots = a.slots + ((size_t)rank * T) * 8;
    for (int t = t0; t < t1; ++t) {
        const int i = t - t0;
        unsigned mask = 0;
        if (i < kKeep) {
#pragma unroll
            for (int q = 0; q < kKeep; ++q) mask = q == i ? kept[q] : mask;
        } else {
            mask = marks(t);
        }
        unsigned s[8];
        for (int d = 0; d < 4; ++d) {
            const unsigned b0 = (mask >> d) & 1u, b1 = (mask >> (d + 4)) & 1u;
            s[d] = b0 ? (unsigned)((cx >> (16 * d)) & 0xffffu) : 0xffffu;
            s[d + 4] = b1 ? (unsigned)((cy >> (16 * d)) & 0xffffu) : 0xffffu;
            cx += (unsigned long long)b0 << (16 * d);
            cy += (unsigned long long)b1 << (16 * d);
        }
        u32x4 pk = {s[0] | (s[1] << 16), s[2] | (s[3] << 16), s[4] | (s[5] << 16), s[6] | (s[7] << 16)};
        *(u32x4*)(slots + (size_t)t * 8) = pk;
    }

    // exchange counts: my 8 per-destination counts go to every peer as 4 LL packets
    const __amdgpu_buffer_rsrc_t rs = ll_resource(c);
    const unsigned rot_off = tag.rot * c.ll_rot_stride;
    const unsigned tid = threadIdx.x;
    if (tid < 8) cnt[rank][tid] = (unsigned)(((tid < 4 ? totx : toty) >> (16 * (tid & 3))) & 0xffffu);
    __syncthreads();
    if (tid < (unsigned)n * 4u) {
        const int p = (int)(tid >> 2);
        const unsigned q = tid & 3u;
        if (p != rank)
            ll_store(rs, (unsigned)p * c.ll_rank_stride + rot_off + ((unsigned)rank * 4u + q) * 16u,
                     cnt[rank][2 * q], cnt[rank][2 * q + 1], tag.flag);
    }
    if (tid < (unsigned)n * 4u) {
        const int j = (int)(tid >> 2);
        const unsigned q = tid & 3u;
        if (j != rank) {
            u32x4 v = {0, 0, 0, 0};
            bool ready = false;
            for (unsigned spins = 0; !ready && spins <= c.spin_limit; ++spins) {
                poll_fence();
                v = ll_load(rs, (unsigned)rank * c.ll_rank_stride + rot_off + ((unsigned)j * 4u + q) * 16u);
                ready = ll_ready(v, tag.flag);
            }
            if (!ready) report(c, kStatusTimeout, (unsigned)rank, 200u, tag.flag, v.y);
            cnt[j][2 * q] = v.x;
            cnt[j][2 * q + 1] = v.z;
        }
    }
    __syncthreads();
    // where my rows start in destination d: after the rows of all lower source ranks
    if (tid < 8) {
        unsigned b = 0;
        for (int s = 0; s < rank; ++s) b += cnt[s][tid];
        a.base[rank * 8 + (int)tid] = (int)tid < n ? b : 0u;
    }
    // as a destination I publish how many rows each source sends me
    if (tid < (unsigned)n) a.recv_counts[rank * n + (int)tid] = (int)cnt[tid][rank];
    // overflow check for my own buffer
    if (tid == 0) {
        unsigned tot = 0;
        for (int s = 0; s < n; ++s) tot += cnt[s][rank];
        if (tot > a.cap) report(c, kStatusCapacity, (unsigned)rank, 201u, a.cap, tot);
    }
    call_end(c, tag);
}

__global__ __launch_bounds__(256) void k_moe_pack(MoeArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    const int lane = (int)(threadIdx.x & 63u);
    const int waves = (int)(blockDim.x >> 6);
    const int wave = chan * waves + (int)(threadIdx.x >> 6);
    const int total_waves = a.chans * waves;
    unsigned base[kMaxRanks];
#pragma unroll
    for (int d = 0; d < kMaxRanks; ++d) base[d] = a.base[rank * 8 + d];
    const char* tokens = (const char*)a.tokens[rank];
    const size_t row_bytes = (size_t)a.row_vecs * 16;

    for (int t = wave; t < a.T; t += total_waves) {
        const u32x4 pk = *(const u32x4*)(a.slots + ((size_t)rank * a.T + t) * 8);
        unsigned row[kMaxRanks];
        row[0] = pk.x & 0xffffu; row[1] = pk.x >> 16; row[2] = pk.y & 0xffffu; row[3] = pk.y >> 16;
        row[4] = pk.z & 0xffffu; row[5] = pk.z >> 16; row[6] = pk.w & 0xffffu; row[7] = pk.w >> 16;
        char* dst[kMaxRanks];
#pragma unroll
        for (int d = 0; d < kMaxRanks; ++d) {
            const unsigned r = base[d] + row[d];
            const bool go = d < n_l && row[d] != 0xffffu && r < a.cap;
            dst[d] = go ? (char*)a.recv[d] + (size_t)r * row_bytes : nullptr;
            if (go && a.has_src && lane == 0) st32_wt(a.recv_src[d] + r, (unsigned)(rank * a.T + t));
        }
        const char* src = tokens + (size_t)t * row_bytes;
        // four vectors per lane in flight; the row is read once and stored to every destination
        for (unsigned i = (unsigned)lane; i < a.row_vecs; i += 256u) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i + 64u * u < a.row_vecs) v[u] = ld16(src, i + 64u * u);
#pragma unroll
            for (int u = 0; u < 4; ++u) settle(v[u]);
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (dst[d]) {
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i + 64u * u < a.row_vecs) st16_wt(dst[d], i + 64u * u, v[u]);
                }
        }
    }
    put_drain();
    if (n > 1) rank_barrier(c, rank, n, chan, 210, false, false);   // write-through puts: all rows destined to me have landed
}

// ---- pack in chip-wide read and write phases: a dealt copy of the rank's whole token array ------------
// Same rows to the same places as k_moe_pack, for many rows that are whole multiples of 64 vectors.  The T rows
// of a rank are one linear array, and this form walks it exactly as k_allgather_hb_phased walks its block: tiles
// of 256 vectors dealt out one by one over the rank's workgroups, H of them held per thread and round, all
// workgroups meeting at the chip-wide barrier between reading and writing (the pack writes about five times
// what it reads), stores without the streaming hint, write phases on the shared paced schedule (PaceCtl).
// The 64 vectors of a wave always lie in one row, so the row's slots are wave-uniform: lane h fetches those of
// held tile h in the read phase, the write phase takes them out of that lane into scalar registers, and they
// decide, without any per-lane condition or load, which destinations the wave's vector goes to.  At any
// moment the 32 workgroups of a rank write 128 KiB of consecutive source, about nine rows of 14 KiB, and the rows one
// source sends to one destination are consecutive there: every (source, destination) pair writes one compact
// window.  Measured at 8 x 4096 rows of 7168 bf16, top-8 of 256 experts, plan and pack together: 0.548 ms
// against 0.625 ms with the schedule off and 0.61-0.64 ms for the free-running k_moe_pack.  A form that held
// 4 whole rows per wave (each wave writing 1 KiB pieces 14 KiB apart) reached 0.59-0.61 ms, one in which a
// workgroup shared a row (4 KiB pieces) 0.60 ms.  One workgroup per CU.
typedef const __attribute__((address_space(4))) u32x4* UniformVecPtr;

template <int H>
__global__ __launch_bounds__(256) void k_moe_pack_dealt(MoeArgs a, DevCtx c, int pace_on)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    if (rank == c.drop_rank) return;
    GridBar gb = grid_barrier_begin(c);
    const unsigned lane = threadIdx.x & 63u;
    const unsigned wave_first = __builtin_amdgcn_readfirstlane(threadIdx.x & ~63u);   // of the wave, in the tile
    const unsigned rv = a.row_vecs;
    const unsigned nv = (unsigned)a.T * rv;                       // the host keeps this below 2^32
    const unsigned tiles = nv / 256u;
    const unsigned per_round = (unsigned)a.chans * (unsigned)H;
    const unsigned rounds = (tiles + per_round - 1u) / per_round;
    const bool pacing = pace_on && rounds >= 1u;
    const unsigned key = ((unsigned)a.T * 40503u + rv) * 2654435761u + gridDim.x * 64u + 56u + 1u;
    PaceCtl ctl = pace_load(c, key);
    unsigned pace = pacing ? ctl.pace : 0u;
    unsigned base[kMaxRanks];
#pragma unroll
    for (int d = 0; d < kMaxRanks; ++d) base[d] = a.base[rank * 8 + d];
    const char* src = (const char*)a.tokens[rank];
    const unsigned short* slots = a.slots + (size_t)rank * a.T * 8;
    const unsigned tstep = (unsigned)a.chans * 256u;              // vectors between two of my tiles
    const unsigned step_rows = tstep / rv, step_cols = tstep % rv;
    unsigned gen = 0;

    // the vector `held`, the wave's share [v, v + 64) of the array starting at column `col` of row t
    auto put = [&](unsigned t, unsigned col, u32x4 pk, u32x4 held) {
        unsigned row[kMaxRanks];
        row[0] = pk.x & 0xffffu; row[1] = pk.x >> 16; row[2] = pk.y & 0xffffu; row[3] = pk.y >> 16;
        row[4] = pk.z & 0xffffu; row[5] = pk.z >> 16; row[6] = pk.w & 0xffffu; row[7] = pk.w >> 16;
#pragma unroll
        for (int d = 0; d < kMaxRanks; ++d) {
            const unsigned slot = base[d] + row[d];
            if (d < n && row[d] != 0xffffu && slot < a.cap) {     // wave-uniform
                st16_wt_keep(a.recv[d], (size_t)slot * rv + col + lane, held);
                if (a.has_src && col == 0u && lane == 0u) st32_wt(a.recv_src[d] + slot, (unsigned)(rank * a.T) + t);
            }
        }
    };

    for (unsigned round = 0; round < rounds; ++round) {
        const unsigned first = round * per_round + (unsigned)chan;
        const unsigned left = first >= tiles ? 0u : (tiles - first + (unsigned)a.chans - 1u) / (unsigned)a.chans;
        const unsigned mine = left < (unsigned)H ? left : (unsigned)H;
        const unsigned v0 = first * 256u + wave_first;            // the wave's first vector in my first tile
        u32x4 held[H];
        static_for<H>([&](auto k) {
            constexpr unsigned h = (unsigned)decltype(k)::value;
            if (h < mine) held[h] = ld16(src, (size_t)v0 + (size_t)h * tstep + lane);
        });
        // the slots of the rows my tiles lie in: lane h fetches those of tile h, the write phase reads them lane by lane
        u32x4 pks = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
        static_assert(H <= 64, "one lane per held tile");
        if (lane < mine) pks = *(const u32x4*)(slots + (size_t)((v0 + lane * tstep) / rv) * 8);
        static_for<H>([&](auto k) { settle(held[decltype(k)::value]); });
        settle(pks);
        grid_barrier(c, gb, ++gen, (unsigned)rank, 215);
        if (pacing && round > 0)
            pace = pace_clamp(__hip_atomic_load(c.gbar + kGridBarPaceWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        unsigned t = v0 / rv, col = v0 % rv;
        const unsigned long long w0 = wall_clock64();
        static_for<H>([&](auto k) {
            constexpr unsigned h = (unsigned)decltype(k)::value;
            if (h < mine) {
                wait_until(w0 + (unsigned long long)(h * pace));
                const u32x4 pk = {(unsigned)__builtin_amdgcn_readlane((int)pks.x, (int)h), (unsigned)__builtin_amdgcn_readlane((int)pks.y, (int)h),
                                  (unsigned)__builtin_amdgcn_readlane((int)pks.z, (int)h), (unsigned)__builtin_amdgcn_readlane((int)pks.w, (int)h)};
                put(t, col, pk, held[h]);
                t += step_rows; col += step_cols;
                if (col >= rv) { col -= rv; ++t; }
            }
        });
        put_drain();
        if (round + 1 < rounds || pacing) {
            grid_barrier(c, gb, ++gen, (unsigned)rank, 216);
            if (pacing && blockIdx.x == 0) {
                if (mine >= (unsigned)H / 4) pace_update(ctl, wall_clock64() - w0, mine);
                if (threadIdx.x == 0) st32_wt(c.gbar + kGridBarPaceWord, ctl.pace);
            }
        }
    }
    if (pacing && blockIdx.x == 0 && threadIdx.x == 0) pace_save(c, ctl, key);
    grid_barrier_end(c, gb, gen);
    if (chan == 0) {                                              // what is left behind the last whole tile
        const unsigned v = tiles * 256u + wave_first;
        if (v < nv) {
            const u32x4 x = ld16(src, (size_t)v + lane);
            const u32x4 pk = *(UniformVecPtr)(slots + (size_t)(v / rv) * 8);   // a scalar load: wave-uniform address
            put(v / rv, v % rv, pk, x);
        }
    }
    put_drain();
    if (n > 1) rank_barrier(c, rank, n, chan, 210, false, false);   // write-through puts: all rows destined to me have landed
}

// ---- pack with FP8 quantisation ---------------------------------------------------------------------
// The "FP8 dispatch" of the paper's expert-parallel setting: the bf16 row is read once, quantised
// in registers to E4M3 in groups of 128 elements (amax = max(|x|, 1e-4), q = e4m3(x * (448/amax)),
// scale = amax/448, fp32 throughout) and the 1-byte row plus its fp32 scales are put into every
// destination.  A lane holds 8 elements; the 16 lanes of a group share their maximum by shuffles.
// a.recv[d] = quantised rows [cap][H] bytes, a.recv_scales[d] = [cap][H/128] floats.
struct MoeFp8Args {
    float* recv_scales[kMaxRanks];
    unsigned groups;        // H / 128
};

// One lane's 16 consecutive bf16 elements (two input vectors) -> 16 E4M3 codes and the scale of their group of
// 128 (the 8 lanes of a group share their maximum by shuffles; every one of them returns the group's scale).
__device__ __forceinline__ u32x4 fp8_quantise16(u32x4 v0, u32x4 v1, float& scale)
{
    const unsigned w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    float x[16];
#pragma unroll
    for (int k = 0; k < 8; ++k) { x[2 * k] = bf16_lo(w[k]); x[2 * k + 1] = bf16_hi(w[k]); }
    float amax = 1e-4f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const float m = fabsf(x[k]);
        amax = m > amax ? m : amax;                  // a NaN never wins the comparison
    }
#pragma unroll
    for (int m = 4; m >= 1; m >>= 1) {
        const float o = __shfl_xor(amax, m, 64);
        amax = o > amax ? o : amax;
    }
    const float inv = 448.0f / amax;
    float y[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) y[k] = x[k] * inv;
    scale = amax / 448.0f;
    return u32x4{e4m3_quad(y[0], y[1], y[2], y[3]), e4m3_quad(y[4], y[5], y[6], y[7]),
                 e4m3_quad(y[8], y[9], y[10], y[11]), e4m3_quad(y[12], y[13], y[14], y[15])};
}

__global__ __launch_bounds__(256) void k_moe_pack_fp8(MoeArgs a, MoeFp8Args f, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    const int lane = (int)(threadIdx.x & 63u);
    const int waves = (int)(blockDim.x >> 6);
    const int wave = chan * waves + (int)(threadIdx.x >> 6);
    const int total_waves = a.chans * waves;
    unsigned base[kMaxRanks];
#pragma unroll
    for (int d = 0; d < kMaxRanks; ++d) base[d] = a.base[rank * 8 + d];
    const char* tokens = (const char*)a.tokens[rank];
    const unsigned row_vecs = a.row_vecs;                    // 16-byte vectors of the bf16 row = H / 8
    const size_t src_row = (size_t)row_vecs * 16, q_row = (size_t)row_vecs * 8;

    for (int t = wave; t < a.T; t += total_waves) {
        const u32x4 pk = *(const u32x4*)(a.slots + ((size_t)rank * a.T + t) * 8);
        unsigned row[kMaxRanks];
        row[0] = pk.x & 0xffffu; row[1] = pk.x >> 16; row[2] = pk.y & 0xffffu; row[3] = pk.y >> 16;
        row[4] = pk.z & 0xffffu; row[5] = pk.z >> 16; row[6] = pk.w & 0xffffu; row[7] = pk.w >> 16;
        char* dq[kMaxRanks];
        float* ds[kMaxRanks];
#pragma unroll
        for (int d = 0; d < kMaxRanks; ++d) {
            const unsigned r = base[d] + row[d];
            const bool go = d < n_l && row[d] != 0xffffu && r < a.cap;
            dq[d] = go ? (char*)a.recv[d] + (size_t)r * q_row : nullptr;
            ds[d] = go ? f.recv_scales[d] + (size_t)r * f.groups : nullptr;
            if (go && a.has_src && lane == 0) st32_wt(a.recv_src[d] + r, (unsigned)(rank * a.T + t));
        }
        const char* src = tokens + (size_t)t * src_row;
        // a lane quantises 16 consecutive elements (two vectors in, one 16-byte vector out); the 8 lanes of a
        // group share their maximum; the next pair of vectors is requested before this one is stored
        const unsigned units = row_vecs >> 1;
        unsigned i = (unsigned)lane;
        u32x4 v0 = {0u, 0u, 0u, 0u}, v1 = v0;
        if (i < units) { v0 = ld16(src, 2u * i); v1 = ld16(src, 2u * i + 1u); }
        while (i < units) {
            const unsigned nx = i + 64u;
            u32x4 n0 = {0u, 0u, 0u, 0u}, n1 = n0;
            if (nx < units) { n0 = ld16(src, 2u * nx); n1 = ld16(src, 2u * nx + 1u); }
            float scale;
            const u32x4 q = fp8_quantise16(v0, v1, scale);
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (dq[d]) {
                    st16_wt(dq[d], i, q);
                    if ((lane & 7) == 0) st32_wt(ds[d] + (i >> 3), __float_as_uint(scale));
                }
            v0 = n0; v1 = n1; i = nx;
        }
    }
    put_drain();
    if (n > 1) rank_barrier(c, rank, n, chan, 230, false, false);
}

// ---- combine: the way back ------------------------------------------------------------------------
// Source rank s gathers, for each of its tokens, the processed rows from the destination ranks the
// token was sent to (same plan as the dispatch) and sums them in fp32 in ascending rank order,
// starting from the first, with one rounding.  A get-style read of the peers' buffers: every row is
// read once and every output row written once.  a.recv[] are the peers' processed rows (read),
// a.tokens[] (cast away const by the host) the per-source outputs.
template <int DT>
__global__ __launch_bounds__(256) void k_moe_combine(MoeArgs a, DevCtx c)
{
    const int n = a.n;
    const int rank = (int)(blockIdx.x % (unsigned)n);
    const int chan = (int)(blockIdx.x / (unsigned)n);
    const int n_l = per_lane(n);   // per-lane copies for conditions (see per_lane)
    if (rank == c.drop_rank) return;
    if (n > 1 && !rank_barrier<true>(c, rank, n, chan, 220, false, false)) return;   // every peer's rows are final
    const int lane = (int)(threadIdx.x & 63u);
    const int waves = (int)(blockDim.x >> 6);
    const int wave = chan * waves + (int)(threadIdx.x >> 6);
    const int total_waves = a.chans * waves;
    unsigned base[kMaxRanks];
#pragma unroll
    for (int d = 0; d < kMaxRanks; ++d) base[d] = a.base[rank * 8 + d];
    char* out = (char*)a.tokens[rank];
    const size_t row_bytes = (size_t)a.row_vecs * 16;

    for (int t = wave; t < a.T; t += total_waves) {
        const u32x4 pk = *(const u32x4*)(a.slots + ((size_t)rank * a.T + t) * 8);
        unsigned row[kMaxRanks];
        row[0] = pk.x & 0xffffu; row[1] = pk.x >> 16; row[2] = pk.y & 0xffffu; row[3] = pk.y >> 16;
        row[4] = pk.z & 0xffffu; row[5] = pk.z >> 16; row[6] = pk.w & 0xffffu; row[7] = pk.w >> 16;
        const char* src[kMaxRanks];
#pragma unroll
        for (int d = 0; d < kMaxRanks; ++d) {
            const unsigned r = base[d] + row[d];
            const bool go = d < n_l && row[d] != 0xffffu && r < a.cap;
            src[d] = go ? (const char*)a.recv[d] + (size_t)r * row_bytes : nullptr;
        }
        char* dst = out + (size_t)t * row_bytes;
        for (unsigned i = (unsigned)lane; i < a.row_vecs; i += 128u) {
            const unsigned i1 = i + 64u;
            const bool two = i1 < a.row_vecs;
            u32x4 v0[kMaxRanks], v1[kMaxRanks];
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (src[d]) {
                    v0[d] = ld16(src[d], i);
                    if (two) v1[d] = ld16(src[d], i1);
                }
            VecAcc<DT> a0, a1;
            bool first = true;
#pragma unroll
            for (int d = 0; d < kMaxRanks; ++d)
                if (src[d]) {
                    if (first) { a0.set(v0[d]); if (two) a1.set(v1[d]); first = false; }
                    else { a0.add(v0[d]); if (two) a1.add(v1[d]); }
                }
            const u32x4 zero = {0, 0, 0, 0};
            st16(dst, i, first ? zero : a0.pack());
            if (two) st16(dst, i1, first ? zero : a1.pack());
        }
    }
    if (n > 1) rank_barrier(c, rank, n, chan, 221, false, false);   // peers are done reading my rows
}

}  // namespace msx
