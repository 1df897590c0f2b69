"""GPU tests of the boundary around the kernels: context handles, prepared calls, routing-plan
objects, the latched timeout, bad expert ids, in-place AllReduce of any count.  Results are
compared bit for bit with the CPU oracle, like every other GPU test here."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2504_09014_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def msx():
    import paper_2504_09014_amd as m
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no fallback path")
    m.init()
    yield m
    m.ctx_use(None)
    for k, v in [("drop_rank", "-1"), ("chaos", "0"), ("spin_limit", str(1 << 20)), ("algo", "auto")]:
        m.set_option(k, v)
    m.reset()


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.uint16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


def _oracle(orc, x):
    return orc.allreduce_bf16(_bits(x)) if x.dtype == torch.bfloat16 else orc.allreduce_f32(_bits(x))


# ---------------------------------------------------------------- contexts

def test_two_contexts_on_two_streams_interleaved(msx, orc):
    """Two communicators, each with half the GPU as its budget, issue calls turn by turn on two
    streams without any ordering between the streams; every result is bit-exact."""
    n = 8
    a, b = msx.ctx_create(n), msx.ctx_create(n, 1 << 20)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        for ctx in (a, b):
            msx.ctx_set_max_blocks(ctx, 128)
        cases = []
        for i, (count, algo) in enumerate([(512, 1), (4096 + 24, 2), (65536, 3), (300000, 3), (8 * 1024, 4),
                                           (2048, 2), (1 << 21, 3), (40000, 5)]):
            x = synth.normal(n, count, seed=700 + i)
            send = [x[r].clone().cuda() for r in range(n)]
            recv = [torch.full_like(s, float("nan")) for s in send]
            cases.append((x, send, recv, algo))
        torch.cuda.synchronize()
        for rep in range(3):
            for i, (x, send, recv, algo) in enumerate(cases):
                ctx, st = (a, sa) if (i + rep) % 2 == 0 else (b, sb)
                msx.ctx_use(ctx)
                msx.allreduce_ex(send, recv, None, algo=algo, stream=st)
            torch.cuda.synchronize()
            for ctx in (a, b):
                assert msx.last_status(ctx)[0] == 0
            for x, send, recv, algo in cases:
                want = orc.allreduce_ring(_bits(x)) if algo == 5 else _oracle(orc, x)
                for r in (0, 3, 7):
                    assert np.array_equal(_bits(recv[r]), want if want.ndim == 1 else want[r]), (algo, r, rep)
                for t in recv:
                    t.fill_(float("nan"))
        # the default context was not touched by any of it and still works
        msx.ctx_use(None)
        x = cases[1][0]
        out = [torch.empty_like(s) for s in cases[1][1]]
        msx.allreduce_ex(cases[1][1], out, None, algo=2)
        msx.check_status()
        assert np.array_equal(_bits(out[5]), _oracle(orc, x))
    finally:
        msx.ctx_use(None)
        torch.cuda.synchronize()
        msx.ctx_destroy(a)
        msx.ctx_destroy(b)
    with pytest.raises(msx.MsxError):
        msx.ctx_use(a)                                   # a destroyed handle is refused


def test_context_budget_limits_every_launch(msx, orc):
    n = 8
    ctx = msx.ctx_create(n)
    try:
        msx.ctx_use(ctx)
        msx.ctx_set_max_blocks(ctx, 64)
        x = synth.normal(n, 1 << 22, seed=31)
        send = [x[r].clone().cuda() for r in range(n)]
        recv = [torch.empty_like(s) for s in send]
        for algo in (2, 3, 4, 5, 6):
            if algo == 2:
                msx.allreduce_ex([s[:65536] for s in send], [r[:65536] for r in recv], None, algo=algo)
            else:
                msx.allreduce_ex(send, recv, None, algo=algo)
            grid, block, _ = msx.last_launch()
            assert grid <= 64 and grid % n == 0, (algo, grid)
        msx.check_status()
        assert np.array_equal(_bits(recv[2]), _oracle(orc, x))
    finally:
        msx.ctx_use(None)
        msx.ctx_destroy(ctx)


# ---------------------------------------------------------------- the latched timeout

@pytest.mark.parametrize("algo", [1, 2, 3, 4, 5, 6])
def test_a_timeout_stops_later_calls_and_leaves_no_stale_results(msx, orc, algo):
    n, count = 8, 8192
    x = synth.normal(n, count, seed=44)
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.full_like(s, 777.0) for s in send]
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "5")
    try:
        msx.allreduce_ex(send, recv, None, algo=algo)
        torch.cuda.synchronize()
        # nothing was read yet: the next call is refused on the host, without waiting for anything
        with pytest.raises(msx.MsxError) as e:
            msx.allreduce_ex(send, recv, None, algo=algo)
        assert e.value.code == -4
        with pytest.raises(msx.MsxError) as e:
            msx.allgather_ex([s[:64] for s in send], [r[:512] for r in recv])
        assert e.value.code == -4
        # whatever was stored is a finished sum: no output element was built from data that never came
        want = orc.allreduce_ring(_bits(x)) if algo == 5 else _oracle(orc, x)
        for r in range(n):
            got = _bits(recv[r])
            w = want if want.ndim == 1 else want[r]
            untouched = got == _bits(torch.tensor([777.0], dtype=torch.bfloat16))[0]
            assert np.all(untouched | (got == w)), (algo, r)
        rc, info = msx.status()
        assert rc == -4
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    msx.allreduce_ex(send, recv, None, algo=algo)
    msx.check_status()
    want = orc.allreduce_ring(_bits(x)) if algo == 5 else _oracle(orc, x)
    assert np.array_equal(_bits(recv[6]), want if want.ndim == 1 else want[6])


# ---------------------------------------------------------------- prepared calls

@pytest.mark.parametrize("algo", [0, 1, 2, 3, 4, 5, 6, 7])
def test_prepared_allreduce_runs_many_times(msx, orc, algo):
    n = 8
    count = 4096 if algo in (1, 2) else 8 * 4096
    x = synth.normal(n, count, seed=50 + algo)
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.full_like(s, float("nan")) for s in send]
    p = msx.prepare_allreduce(send, recv, None, algo=algo)
    want = orc.allreduce_ring(_bits(x)) if algo in (5, 7) else _oracle(orc, x)
    try:
        for k in range(4):
            for t in recv:
                t.fill_(float("nan"))
            p.run()
            if k == 1:
                msx.allreduce_ex(send, recv, None, algo=algo)      # an ordinary call in between
            msx.check_status()
            for r in (0, 4, 7):
                assert np.array_equal(_bits(recv[r]), want if want.ndim == 1 else want[r]), (algo, k, r)
    finally:
        p.release()
    assert p.handle is None


def test_prepared_calls_with_residual_and_other_collectives(msx, orc):
    n, count = 8, 8 * 1000
    x = synth.normal(n, count, seed=61)
    res = synth.normal(1, count, seed=62)[0]
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.empty_like(s) for s in send]
    rr = [res.cuda()] * n
    p = msx.prepare_allreduce(send, recv, rr)
    p.run()
    msx.check_status()
    assert np.array_equal(_bits(recv[3]), orc.allreduce_residual_bf16(_bits(x), _bits(res)))
    p.release()
    part = [torch.empty(count // n, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    full = [torch.empty(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    full2 = [torch.empty(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    prs, pag, pa2 = msx.prepare_reducescatter(send, part), msx.prepare_allgather(part, full), msx.prepare_alltoall(send, full2)
    for _ in range(2):
        prs.run()
        pag.run()                   # AllGather of ReduceScatter = AllReduce
        pa2.run()
    msx.check_status()
    want = _oracle(orc, x)
    for r in range(n):
        assert np.array_equal(_bits(full[r]), want)
    xa = _bits(x).reshape(n, n, count // n)
    for d in (0, 5):
        assert np.array_equal(_bits(full2[d]).reshape(n, count // n), xa[:, d, :])
    for p in (prs, pag, pa2):
        p.release()


def test_prepared_call_dies_with_its_context(msx):
    n = 8
    ctx = msx.ctx_create(n)
    msx.ctx_use(ctx)
    send = [torch.zeros(1024, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    p = msx.prepare_allreduce(send, send)
    p.run()
    torch.cuda.synchronize()
    msx.ctx_use(None)
    msx.ctx_destroy(ctx)
    with pytest.raises(msx.MsxError) as e:
        p.run()
    assert e.value.code == -1
    p.release()


# ---------------------------------------------------------------- routing plans, bad ids

def test_two_routing_plans_interleaved_and_prepared(msx, orc):
    n, T, H, K, E = 8, 300, 64, 8, 256
    plans = [msx.moe_plan_create(T), msx.moe_plan_create(T)]
    sets = []
    for i in range(2):
        tokens = synth.moe_tokens(n, T, H, seed=80 + i)
        topk = synth.moe_routing(n, T, K, E, seed=80 + i)
        tok = [tokens[r].clone().cuda() for r in range(n)]
        idx = [topk[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros((n * T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
        out = [torch.empty((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        sets.append((tokens, topk, tok, idx, recv, counts, out))
    try:
        # dispatch A, dispatch B, combine A, combine B: each combine finds its own routing
        for i in range(2):
            _, _, tok, idx, recv, counts, _ = sets[i]
            msx.moe_dispatch(tok, idx, E, recv, counts, plan=plans[i])
        for i in range(2):
            msx.moe_combine(sets[i][4], sets[i][6], plan=plans[i])
        msx.check_status()
        for i in range(2):
            tokens, topk, tok, idx, recv, counts, out = sets[i]
            want_recv, _, want_counts, rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, n * T)
            assert rc == 0 and np.array_equal(counts.cpu().numpy(), want_counts)
            want_out, _ = orc.moe_combine_bf16(np.stack([_bits(t) for t in recv]), topk.numpy(), E)
            for s in range(n):
                assert np.array_equal(_bits(recv[s]), want_recv[s]), (i, s)
                assert np.array_equal(_bits(out[s]), want_out[s]), (i, s)
        # the same pair as prepared calls
        tokens, topk, tok, idx, recv, counts, out = sets[0]
        pd = msx.prepare_moe_dispatch(tok, idx, E, recv, counts, plans[0])
        pc = msx.prepare_moe_combine(recv, out, plans[0])
        want_out, _ = orc.moe_combine_bf16(np.stack([_bits(t) for t in recv]), topk.numpy(), E)
        for _ in range(2):
            for t in out:
                t.zero_()
            pd.run()
            pc.run()
            msx.check_status()
            assert np.array_equal(_bits(out[4]), want_out[4])
        pd.release()
        pc.release()
        # a plan made for fewer tokens refuses, and so does a prepared dispatch without a plan
        small = msx.moe_plan_create(T // 2)
        with pytest.raises(msx.MsxError) as e:
            msx.moe_dispatch(tok, idx, E, recv, counts, plan=small)
        assert e.value.code == -5
        msx.moe_plan_destroy(small)
        with pytest.raises(msx.MsxError) as e:
            msx.prepare_moe_dispatch(tok, idx, E, recv, counts, None)
        assert e.value.code == -1
    finally:
        torch.cuda.synchronize()
        for p in plans:
            msx.moe_plan_destroy(p)


def test_expert_id_out_of_range_is_reported(msx, orc):
    n, T, H, K, E = 8, 100, 32, 8, 256
    tokens = synth.moe_tokens(n, T, H, seed=90)
    topk = synth.moe_routing(n, T, K, E, seed=90)
    for bad in (256, -1, 1 << 30):
        tk = topk.clone()
        tk[3, 17, 2] = bad
        assert orc.moe_dispatch(_bits(tokens), tk.numpy(), E, n * T)[3] == -2      # the oracle refuses it too
        tok = [tokens[r].clone().cuda() for r in range(n)]
        idx = [tk[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros((n * T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
        msx.moe_dispatch(tok, idx, E, recv, counts)
        rc, info = msx.status()
        assert rc == -7 and info[0] == 3 and info[1] == 3 and info[2] == 202, (bad, rc, info)
        assert info[4] == bad & 0xFFFFFFFF
        assert "expert id" in msx.strerror(rc)
    # K other than 8 takes the scalar path of the plan kernel
    tk = synth.moe_routing(n, T, 3, E, seed=91)
    tk[0, 0, 0] = 999
    idx = [tk[r].clone().cuda() for r in range(n)]
    msx.moe_dispatch(tok, idx, E, recv, counts)
    assert msx.status()[0] == -7


# ---------------------------------------------------------------- in-place AllReduce, any count

@pytest.mark.parametrize("n,count,dtype", [(8, 3, torch.float32), (8, 1001, torch.bfloat16), (5, 77, torch.bfloat16),
                                           (3, 1, torch.float32), (8, 100003, torch.bfloat16), (7, 4097, torch.float32)])
def test_in_place_allreduce_takes_rows_that_are_not_16_byte_multiples(msx, orc, n, count, dtype):
    x = synth.normal(n, count, seed=count, dtype=dtype)
    buf = x.clone().cuda()
    msx.allreduce(buf)
    msx.check_status()
    want = _oracle(orc, x)
    got = _bits(buf)
    for r in range(n):
        assert np.array_equal(got[r].view(np.uint32) if dtype == torch.float32 else got[r],
                              want.view(np.uint32) if dtype == torch.float32 else want), r
