"""CPU tests of the library's host logic (no device is touched): the automatic algorithm choice,
the launch shapes, and the lowering of AllReduce to execution plans.  A lowered plan is RUN here
by a small sequential simulator over numpy buffers (one float per 16-byte vector), with a
scheduler that advances workgroups until they block, so the test also shows that the plan cannot
deadlock and that every wait is matched by exactly one signal."""
import ctypes as C
import os

import numpy as np
import pytest


class PlanRef(C.Structure):
    _fields_ = [("kind", C.c_int16), ("rank", C.c_int16)]


class PlanOp(C.Structure):
    _fields_ = [("code", C.c_int), ("peer", C.c_int), ("flags", C.c_int), ("nsrc", C.c_int), ("ndst", C.c_int),
                ("src", PlanRef * 9), ("dst", PlanRef * 8), ("dst_wt", C.c_int), ("aux", C.c_uint32),
                ("first", C.c_uint64), ("end", C.c_uint64), ("step", C.c_uint64),
                ("aux2", C.c_uint32), ("aux3", C.c_uint32)]


END, BARRIER, SIGNAL, WAIT, REDUCE_PUT, DRAIN, PUT_PACKET, REDUCE_PACKET, COPY_PACKET, REDUCE_HOLD, GRID_BARRIER, \
    PUT_HELD = range(12)
IN, OUT, SCRATCH = range(3)


@pytest.fixture(scope="module")
def L():
    import paper_2504_09014_amd as msx
    return msx.lib()


def lower(L, algo, n, chans, vecs_per_rank, threads):
    written = C.c_size_t(0)
    assert L.msx_debug_lower_plan(algo, n, chans, vecs_per_rank, threads, None, 0, None, C.byref(written)) == 0
    ops = (PlanOp * written.value)()
    start = (C.c_uint32 * (n * chans + 1))()
    assert C.sizeof(PlanOp) == 128
    assert L.msx_debug_lower_plan(algo, n, chans, vecs_per_rank, threads, ops, written.value, start,
                                  C.byref(written)) == 0
    return ops, list(start)


def lower_ex(L, algo, n, chans, nbytes, threads, held=0):
    written = C.c_size_t(0)
    assert L.msx_debug_lower_plan_ex(algo, n, chans, nbytes, threads, held, None, 0, None, C.byref(written)) == 0
    ops = (PlanOp * written.value)()
    start = (C.c_uint32 * (n * chans + 1))()
    assert L.msx_debug_lower_plan_ex(algo, n, chans, nbytes, threads, held, ops, written.value, start,
                                     C.byref(written)) == 0
    return ops, list(start)


def simulate(ops, start, n, chans, threads, x, ring_order_rounding=None):
    """x: [n, V] float64 'vectors' (for packet operations: one value per 8-byte packet).  Returns out [n, V].
    Each workgroup runs until it blocks.  LL scratch: per rank a dict byte offset -> value (a packet that is
    there carries the call's flag); the chip-wide barrier: a generation count per workgroup."""
    V = x.shape[1]
    ll = [dict() for _ in range(n)]
    grid_gen = [0] * (n * chans)
    held = [dict() for _ in range(n * chans)]
    bufs = {IN: x.copy(), OUT: np.full((n, V), np.nan), SCRATCH: np.full((n, V), np.nan)}
    sem = np.zeros((n, n, chans), np.int64)          # [recv][send][chan]
    expected = np.zeros((n, n, chans), np.int64)
    pc = [start[b] for b in range(n * chans)]
    barrier_phase = [0] * (n * chans)                # 0: must signal, 1: waiting
    done = [False] * (n * chans)
    touched = np.zeros((3, n, V), np.int32)

    def step(b):
        """run workgroup b until it blocks or ends; return True if it made progress"""
        rank, chan = b % n, b // n
        progressed = False
        while True:
            op = ops[pc[b]]
            if op.code == END:
                done[b] = True
                return True
            if op.code == BARRIER:
                if barrier_phase[b] == 0:
                    for p in range(n):
                        if p != rank:
                            sem[p, rank, chan] += 1
                    barrier_phase[b] = 1
                    progressed = True
                ok = all(sem[rank, p, chan] >= expected[rank, p, chan] + 1 for p in range(n) if p != rank)
                if not ok:
                    return progressed
                for p in range(n):
                    if p != rank:
                        expected[rank, p, chan] += 1
                barrier_phase[b] = 0
            elif op.code == SIGNAL:
                sem[op.peer, rank, chan] += 1
            elif op.code == WAIT:
                if sem[rank, op.peer, chan] < expected[rank, op.peer, chan] + 1:
                    return progressed
                expected[rank, op.peer, chan] += 1
            elif op.code == REDUCE_PUT:
                idx = np.concatenate([np.arange(op.first + t, op.end, op.step) for t in range(threads)]) \
                    if op.first < op.end else np.zeros(0, np.int64)
                idx = idx.astype(np.int64)
                acc = bufs[op.src[0].kind][op.src[0].rank, idx].copy()
                for k in range(1, op.nsrc):
                    acc = acc + bufs[op.src[k].kind][op.src[k].rank, idx]
                    if ring_order_rounding is not None:
                        acc = ring_order_rounding(acc)
                assert not np.any(np.isnan(acc)), "read of a vector nobody has written"
                for k in range(op.ndst):
                    d = op.dst[k]
                    bufs[d.kind][d.rank, idx] = acc
                    touched[d.kind, d.rank, idx] += 1
                    # data another rank will read must be written through (no fence follows)
                    if d.rank != rank:
                        assert op.dst_wt & (1 << k), "remote destination written with an ordinary store"
            elif op.code == DRAIN:
                pass
            elif op.code == PUT_PACKET:
                for t in range(threads):
                    for q in range(op.first + t, op.end, op.step):
                        for p_ in range(n):
                            if (op.dst_wt >> p_) & 1 and op.aux2 * p_ + q < V:
                                assert p_ != rank
                                off = op.aux3 + op.peer * op.aux + q * 16
                                assert off not in ll[p_], "a packet slot written twice in one call"
                                ll[p_][off] = bufs[op.src[0].kind][op.src[0].rank, op.aux2 * p_ + q]
            elif op.code == REDUCE_PACKET:
                qs = [q for t in range(threads) for q in range(op.first + t, op.end, op.step) if op.aux2 + q < V]
                need = [op.aux3 + j * op.aux + q * 16 for q in qs for j in range(n) if j != op.peer]
                if not all(o in ll[rank] for o in need):
                    return progressed                                  # still polling
                for q in qs:
                    k = op.aux2 + q
                    acc = None
                    for j in range(n):                                 # rank order, mine among them
                        v = bufs[op.src[0].kind][op.src[0].rank, k] if j == op.peer else ll[rank][op.aux3 + j * op.aux + q * 16]
                        acc = v if acc is None else acc + v
                    bufs[op.dst[0].kind][op.dst[0].rank, k] = acc
                    touched[op.dst[0].kind, op.dst[0].rank, k] += 1
                    for p_ in range(n):
                        if (op.dst_wt >> p_) & 1:
                            off = op.aux3 + n * op.aux + op.peer * op.aux + q * 16
                            assert off not in ll[p_]
                            ll[p_][off] = acc
            elif op.code == COPY_PACKET:
                want = [(j, q) for t in range(threads) for q in range(op.first + t, op.end, op.step)
                        for j in range(n) if j != op.peer and op.aux2 * j + q < V]
                if not all(op.aux3 + j * op.aux + q * 16 in ll[rank] for j, q in want):
                    return progressed
                for j, q in want:
                    bufs[op.dst[0].kind][op.dst[0].rank, op.aux2 * j + q] = ll[rank][op.aux3 + j * op.aux + q * 16]
                    touched[op.dst[0].kind, op.dst[0].rank, op.aux2 * j + q] += 1
            elif op.code == REDUCE_HOLD:
                held[b] = {}
                for t in range(threads):
                    for h in range(op.aux):
                        i = op.first + t + h * op.step
                        acc = bufs[op.src[0].kind][op.src[0].rank, i]
                        for k in range(1, op.nsrc):
                            acc = acc + bufs[op.src[k].kind][op.src[k].rank, i]
                        held[b][(t, h)] = acc
            elif op.code == PUT_HELD:
                for t in range(threads):
                    for h in range(op.aux):
                        i = op.first + t + h * op.step
                        for k in range(op.ndst):
                            d = op.dst[k]
                            bufs[d.kind][d.rank, i] = held[b][(t, h)]
                            touched[d.kind, d.rank, i] += 1
            elif op.code == GRID_BARRIER:
                if barrier_phase[b] == 0:
                    grid_gen[b] += 1
                    barrier_phase[b] = 1
                    progressed = True
                if min(grid_gen) < grid_gen[b]:
                    return progressed
                barrier_phase[b] = 0
            else:
                raise AssertionError(f"unknown op {op.code}")
            pc[b] += 1
            progressed = True

    for _ in range(100000):
        if all(done):
            break
        any_progress = False
        for b in np.random.default_rng(len(ops)).permutation(n * chans):   # scrambled, deterministic order
            if not done[b]:
                any_progress |= step(int(b))
        assert any_progress, "the plan deadlocks"
    assert all(done)
    # every signal was consumed by exactly one wait
    off = ~np.eye(n, dtype=bool)
    assert np.array_equal(sem[off], expected[off])
    return bufs[OUT], touched


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("chans,threads,cv", [(1, 4, 1), (3, 4, 7), (2, 8, 64), (5, 16, 333)])
def test_lowered_all_pairs_plan_computes_the_allreduce(L, n, chans, threads, cv):
    V = cv * n
    ops, start = lower(L, 6, n, chans, V, threads)
    rng = np.random.default_rng(V)
    x = rng.integers(-1000, 1001, (n, V)).astype(np.float64)
    out, touched = simulate(ops, start, n, chans, threads, x)
    assert np.array_equal(out, np.tile(x.sum(0), (n, 1)))
    assert np.all(touched[OUT] == 1)                              # every output vector is written exactly once
    assert np.all(touched[SCRATCH] == 0)


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("chans,threads,cv", [(1, 4, 1), (3, 4, 7), (2, 8, 64), (5, 16, 333)])
def test_lowered_ring_plan_computes_the_allreduce_in_ring_order(L, n, chans, threads, cv):
    V = cv * n
    ops, start = lower(L, 7, n, chans, V, threads)
    rng = np.random.default_rng(V + 1)
    x = rng.standard_normal((n, V)) * np.exp(rng.standard_normal((n, V)) * 3)
    x = x.astype(np.float32).astype(np.float64)
    rnd = lambda a: a.astype(np.float32).astype(np.float64)        # partial sums travel as fp32
    out, touched = simulate(ops, start, n, chans, threads, x, ring_order_rounding=rnd)
    want = np.empty(V)
    for k in range(n):                                            # chunk k: k, k+1, ..., k-1 (mod n)
        sl = slice(k * cv, (k + 1) * cv)
        acc = x[k, sl].astype(np.float32)
        for h in range(1, n):
            acc = (acc + x[(k + h) % n, sl].astype(np.float32)).astype(np.float32)
        want[sl] = acc
    assert np.array_equal(out, np.tile(want, (n, 1)))
    assert np.all(touched[OUT] == 1)
    # each rank's scratch receives every chunk but the one that ends its trip there... exactly n-1 chunks
    assert np.all(touched[SCRATCH].reshape(n, n, cv).sum(axis=2) // cv <= 1)
    assert np.all(touched[SCRATCH].sum(axis=1) == (n - 1) * cv)


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("chans,threads,P", [(1, 4, 1), (3, 4, 7), (2, 8, 64), (5, 16, 333), (1, 64, 8 * 64 + 1)])
@pytest.mark.parametrize("algo", [8, 9])
def test_lowered_packet_plans_compute_the_allreduce(L, algo, n, chans, threads, P):
    """1PA and 2PA over LL packets as lowered plans: every packet slot is written once, every poll is
    answered, every output packet is produced exactly once, sums are taken in rank order."""
    ops, start = lower_ex(L, algo, n, chans, P * 8, threads)
    codes = [ops[k].code for k in range(start[0], start[1])]
    assert codes == ([PUT_PACKET, REDUCE_PACKET, END] if algo == 8 else [PUT_PACKET, REDUCE_PACKET, COPY_PACKET, END])
    rng = np.random.default_rng(P + n)
    x = rng.integers(-1000, 1001, (n, P)).astype(np.float64)
    out, touched = simulate(ops, start, n, chans, threads, x)
    assert np.array_equal(out, np.tile(x.sum(0), (n, 1)))
    assert np.all(touched[OUT] == 1)


@pytest.mark.parametrize("chans,threads,held,cv", [(1, 4, 4, 4 * 4 * 3), (3, 4, 4, 4 * 50 + 3), (2, 8, 8, 8 * 8 * 2 * 2),
                                                   (4, 4, 64, 4 * 300 + 1), (2, 4, 4, 3)])
def test_lowered_phased_plan_computes_the_allreduce(L, chans, threads, held, cv):
    """The read phase / write phase schedule as a plan: all workgroups pass the same number of chip-wide
    barriers, no workgroup holds more than `held` tiles, every output vector is written exactly once."""
    n = 8
    V = cv * n
    ops, start = lower_ex(L, 6, n, chans, V * 16, threads, held)
    per_wg = []
    for b in range(n * chans):
        lst = [ops[k] for k in range(start[b], start[b + 1])]
        per_wg.append(sum(1 for o in lst if o.code == GRID_BARRIER))
        assert all(o.aux <= held for o in lst if o.code in (REDUCE_HOLD, PUT_HELD))
        assert lst[0].code == BARRIER and lst[-2].code == BARRIER and lst[-1].code == END
    assert len(set(per_wg)) == 1
    rng = np.random.default_rng(V)
    x = rng.integers(-1000, 1001, (n, V)).astype(np.float64)
    out, touched = simulate(ops, start, n, chans, threads, x)
    assert np.array_equal(out, np.tile(x.sum(0), (n, 1)))
    assert np.all(touched[OUT] == 1)


def test_lower_plan_argument_checks(L):
    w = C.c_size_t(0)
    assert L.msx_debug_lower_plan(3, 8, 1, 64, 256, None, 0, None, C.byref(w)) == -1      # not a plan algorithm
    assert L.msx_debug_lower_plan(6, 1, 1, 64, 256, None, 0, None, C.byref(w)) == -1      # one rank
    assert L.msx_debug_lower_plan(6, 8, 1, 63, 256, None, 0, None, C.byref(w)) == -1      # not divisible
    assert L.msx_debug_lower_plan(6, 8, 2, 64, 256, None, 0, None, C.byref(w)) == 0 and w.value == 16 * 5
    ops = (PlanOp * 4)()
    start = (C.c_uint32 * 17)()
    assert L.msx_debug_lower_plan(6, 8, 2, 64, 256, ops, 4, start, C.byref(w)) == -5       # buffer too small
    assert L.msx_debug_lower_plan_ex(8, 8, 1, 1001, 256, 0, None, 0, None, C.byref(w)) == -1   # odd byte count
    assert L.msx_debug_lower_plan_ex(9, 8, 1, 1000, 256, 64, None, 0, None, C.byref(w)) == -1  # packets hold nothing
    assert L.msx_debug_lower_plan_ex(7, 8, 1, 1024, 256, 64, None, 0, None, C.byref(w)) == -1  # the ring neither
    assert L.msx_debug_lower_plan_ex(8, 8, 1, 1000, 256, 0, None, 0, None, C.byref(w)) == 0 and w.value == 8 * 3


def test_automatic_choice_and_launch_shapes(L):
    a, u, w = C.c_int(), C.c_int(), C.c_int()
    ll = 4 << 20

    def choose(nbytes, n=8):
        assert L.msx_debug_choose(nbytes, n, ll, C.byref(a), C.byref(u), C.byref(w)) == 0
        return a.value, u.value, w.value

    assert choose(1024)[0] == 1 and choose(2048)[0] == 1          # tiny: one-phase LL
    assert choose(2049)[0] == 3 and choose(1 << 30)[0] == 3       # everything else: fused HB
    assert choose(1024, n=1)[0] == 3                              # a single rank is a copy
    # launch shapes: one pass with one vector per thread up to 2 MiB per rank, two up to 4 MiB, then 32, then
    # 128 workgroups per rank (1024 in all)
    assert choose(64 << 10) == (3, 1, 2)
    assert choose(1 << 20) == (3, 1, 32)
    assert choose(2 << 20) == (3, 1, 64)
    assert choose(4 << 20) == (3, 2, 64)
    assert choose(32 << 20) == (3, 1, 32)
    assert choose((40 << 20) - 16) == (3, 1, 128)
    # 8 ranks from 40 MiB: chip-wide read / write phases, 64 sums held per thread, every resident workgroup
    assert choose(40 << 20) == (3, 64, 256)
    assert choose(64 << 20) == (3, 64, 256)
    assert choose(1 << 30) == (3, 64, 256)
    assert choose(1 << 30, n=7) == (3, 1, 146)
    # thresholds follow the options
    import paper_2504_09014_amd as msx
    old = msx.get_option("ll_2pa_max_bytes")
    msx.set_option("ll_2pa_max_bytes", str(256 << 10))
    try:
        assert choose(128 << 10)[0] == 2 and choose(512 << 10)[0] == 3
        assert choose(3 << 20)[0] == 3
    finally:
        msx.set_option("ll_2pa_max_bytes", old)
    assert L.msx_debug_choose(1024, 0, ll, C.byref(a), C.byref(u), C.byref(w)) == -1


def test_write_phase_pacing_controller_finds_and_keeps_the_tightest_schedule(L):
    """The controller of the paced write phases, run against a model of the memory system: a phase held to a
    schedule s (ticks per tile) takes s * tiles + tail when the schedule can be met, and the unpaced time when
    it is too tight (nobody is held back then).  It must settle just above the cliff, hold there, recover when
    the cliff moves, and never leave [0, 1500] ticks per tile."""
    L.msx_debug_pace_update.argtypes = [C.POINTER(C.c_uint32), C.c_uint64, C.c_uint32]
    tiles, tail, unpaced = 64, 250, 9600                        # 10 ns ticks: 96 us unpaced

    def run(state, cliff, rounds):
        took_log = []
        for _ in range(rounds):
            s = state[0]
            took = unpaced if s == 0 or s * tiles < cliff else s * tiles + tail
            took_log.append(took)
            assert L.msx_debug_pace_update(state, took, tiles) == 0
            assert 0 <= state[0] <= 1500
        return took_log

    state = (C.c_uint32 * 4)(0, 0, 0, 0)
    log = run(state, cliff=7000, rounds=16)                     # the system can do 70 us, not less
    assert log[0] == unpaced and state[2] == 1                  # learnt from an unpaced phase, frozen by the end
    assert 7000 <= state[0] * tiles <= 7000 * 13 // 12 + tiles  # within one tightening step above the cliff
    assert sum(t == unpaced for t in log) <= 2                  # the first phase and the one miss that found the cliff
    assert all(t <= 7000 * 13 // 12 + tail + tiles for t in log[-8:])
    held = state[0]
    run(state, cliff=7000, rounds=8)
    assert state[0] == held                                     # frozen: stays
    # ... but not for ever: after 256 phases that met it, it tries one step tighter, misses, and is back
    log = run(state, cliff=7000, rounds=300)
    assert state[0] == held and state[2] == 1 and sum(t == unpaced for t in log) == 1
    # a frozen schedule that has become far too loose (the cliff moved down) is found out the same way
    loose = (C.c_uint32 * 4)(held, held, 1, 0)
    run(loose, cliff=3500, rounds=256 * 9)
    assert 3500 <= loose[0] * tiles <= 3500 * 13 // 12 + tiles, loose[0]
    log = run(state, cliff=9000, rounds=12)                     # conditions change: the old schedule is too tight now
    assert sum(t == unpaced for t in log) <= 6 and 9000 <= state[0] * tiles <= 9000 * 13 // 12 + tiles
    # a system on which pacing gains nothing (no schedule below the unpaced time can be met): the search ends
    # within the tolerance of the unpaced time and does no harm (no phase ever takes longer than unpaced)
    state = (C.c_uint32 * 4)(0, 0, 0, 0)
    log = run(state, cliff=unpaced, rounds=20)
    assert unpaced * 15 // 16 <= state[0] * tiles <= unpaced + 2 * tiles and max(log) <= unpaced + tail + 2 * tiles
    # nonsense input leaves the state alone or clamps it
    junk = (C.c_uint32 * 4)(0, 0, 0, 0)
    assert L.msx_debug_pace_update(junk, 10 ** 9, tiles) == 0 and junk[0] == 0      # over a millisecond: ignored
    assert L.msx_debug_pace_update(junk, 99999, 1) == 0 and junk[0] == 0            # would exceed the clamp
    assert L.msx_debug_pace_update(None, 100, tiles) == -1


def test_write_phase_pacing_controller_stays_inside_its_clamp_on_any_input(L):
    """Whatever a phase reports (clock glitches, a phase that took no time, one tile, thousands of tiles, a state
    left behind by another shape), the pace stays within [0, 1500] ticks per tile and the remembered good
    schedule too: a wave is never told to wait longer than 15 us per tile."""
    L.msx_debug_pace_update.argtypes = [C.POINTER(C.c_uint32), C.c_uint64, C.c_uint32]
    rng = np.random.default_rng(11)
    for trial in range(200):
        state = (C.c_uint32 * 4)(*[int(v) for v in rng.integers(0, 1501, 2)], int(rng.integers(0, 2)), int(rng.integers(0, 3)))
        # pace, good (<= 1500, as pace_load leaves them), frozen, misses
        for _ in range(60):
            took = int(rng.choice([0, 1, int(rng.integers(0, 2000)), int(rng.integers(0, 99999)), 99999, 100000, 2 ** 40]))
            tiles = int(rng.choice([1, 2, 16, 63, 64, int(rng.integers(1, 5000))]))
            assert L.msx_debug_pace_update(state, took, tiles) == 0
            assert state[0] <= 1500 and state[1] <= 1500 and state[2] <= 1 and (state[3] & 0xff) <= 3 and (state[3] >> 8) < 256, \
                (trial, list(state), took, tiles)


def test_owner_of_an_expert_by_multiplication_equals_the_division(L):
    """The token plan computes e // (n_experts // nranks) as (e * magic) >> 32: exact for every expert id of
    every shape the library uses the multiplier for, and the library divides where it would not be."""
    for nranks in range(1, 9):
        for per in [1, 2, 3, 7, 31, 32, 33, 100, 255, 256, 1000, 4096, 8191]:
            n_experts = per * nranks
            m = C.c_uint32(0)
            assert L.msx_debug_owner_magic(n_experts, nranks, C.byref(m)) == 0
            if per == 1 or n_experts >= 65536:
                assert m.value == 0
                continue
            e = np.arange(n_experts, dtype=np.uint64)
            assert np.array_equal((e * np.uint64(m.value)) >> np.uint64(32), e // np.uint64(per)), (nranks, per)
    m = C.c_uint32(0)
    assert L.msx_debug_owner_magic(10, 3, C.byref(m)) == -1


def test_bench_refuses_more_than_one_gpu_and_names_the_reason():
    """The ranks are emulated inside one GPU: `bench.py --gpus N` with N above 1 must exit with a message that
    says so, before anything touches a device."""
    import subprocess
    import sys as _sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([_sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_metric_is_the_baseline_metric():
    import json
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = open(os.path.join(root, "bench.py")).read()
    m = re.search(r'"metric": ("[^\n]*?"),', src)
    assert m and json.loads(m.group(1)) == json.load(open(os.path.join(root, "BASELINE.json")))["metric"]
