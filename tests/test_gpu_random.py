"""Seeded random sweep over the AllReduce entry points: rank counts, sizes (ragged tails included),
dtypes, algorithms, in place or not, residual modes and scrambled workgroup timing, each case
compared bit for bit with the CPU oracle."""
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
    m.set_option("chaos", "0")


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.uint16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


@pytest.mark.parametrize("seed", range(6))
def test_random_allreduce_cases(msx, orc, seed):
    rng = np.random.default_rng(1000 + seed)
    ll_limit = int(msx.get_option("ll_max_bytes"))
    for case in range(60):
        n = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        bf16 = bool(rng.integers(0, 2))
        esz = 2 if bf16 else 4
        count = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 300000)]))
        algo = int(rng.choice([0, 1, 2, 3, 4, 5, 6, 7]))
        res_mode = int(rng.choice([0, 0, 1, 2]))
        inplace = bool(rng.integers(0, 2))
        if algo in (5, 6, 7):                                   # ring / interpreter: whole vectors per chunk, no residual
            count = max(1, count // (16 * n // esz)) * (16 * n // esz)
            res_mode = 0
        if algo == 4 and res_mode == 2:
            res_mode = 1
        if algo == 1 and count * esz > ll_limit // 4:
            algo = 3
        dtype = torch.bfloat16 if bf16 else torch.float32
        x = synth.normal(n, count, seed=seed * 100 + case, dtype=dtype)
        res = None
        if res_mode:
            res = synth.normal(n if res_mode == 2 else 1, count, seed=seed * 100 + case + 50, dtype=dtype)
        msx.set_option("chaos", str(int(rng.integers(0, 50))))
        # a third of the cases: the fused HB kernel in its phased form (by default only for very large messages),
        # with few workgroups per rank so that small inputs still take several rounds
        force_phased = bool(rng.integers(0, 3) == 0)
        msx.set_option("hb_phased_min_bytes", "0" if force_phased else "auto")
        msx.set_option("hb_blocks_per_rank", str(int(rng.choice([0, 1, 2, 3]))) if force_phased else "0")
        send = [x[r].clone().cuda() for r in range(n)]
        recv = send if inplace else [torch.full_like(s, float("nan")) for s in send]
        rtab = None
        if res_mode == 1:
            shared = res[0].cuda()
            rtab = [shared] * n
        elif res_mode == 2:
            rtab = [res[r].clone().cuda() for r in range(n)]
        msx.allreduce_ex(send, recv, rtab, algo=algo)
        msx.check_status()
        xb = _bits(x)
        for r in range(n):
            if algo in (5, 7) and n > 1:
                want = orc.allreduce_ring(xb)
            elif res_mode == 0:
                want = orc.allreduce_bf16(xb) if bf16 else orc.allreduce_f32(xb)
            else:
                rr = _bits(res[r if res_mode == 2 else 0])
                want = orc.allreduce_residual_bf16(xb, rr) if bf16 else orc.allreduce_residual_f32(xb, rr)
            got = _bits(recv[r])
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), \
                dict(seed=seed, case=case, n=n, bf16=bf16, count=count, algo=algo, res=res_mode, inplace=inplace,
                     phased=force_phased, rank=r)
    msx.set_option("chaos", "0")
    msx.set_option("hb_phased_min_bytes", "auto")
    msx.set_option("hb_blocks_per_rank", "0")


@pytest.mark.parametrize("seed", range(4))
def test_random_reducescatter_allgather_alltoall_cases(msx, orc, seed):
    """HB and packet forms, in place and out of place, every element type; reduce-scatter also with max / min."""
    rng = np.random.default_rng(2000 + seed)
    tdt = [torch.float32, torch.bfloat16, torch.float16, torch.int32]
    view = lambda t, dt: t.view(torch.uint16).numpy() if dt in (1, 2) else t.numpy()
    for case in range(50):
        n = int(rng.choice([1, 2, 3, 5, 8]))
        dt = int(rng.integers(0, 4))
        op = int(rng.choice([0, 0, 1, 2]))
        c = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 40000)]))
        coll_algo = str(rng.choice(["auto", "hb", "ll"]))
        inplace = bool(rng.integers(0, 2))
        if inplace:
            c = max(8, c // 8 * 8)                              # the rows of an in-place buffer are 16-byte aligned
        if coll_algo == "ll" and ((c * (2 if dt in (1, 2) else 4)) % 8 or dt >= 2 or op):
            coll_algo = "hb"                                    # packets carry whole 8-byte units of fp32 / bf16 sums
        tag = dict(seed=seed, case=case, n=n, dt=dt, op=op, c=c, coll=coll_algo, inplace=inplace)
        msx.set_option("coll_algo", coll_algo)
        msx.set_option("chaos", str(int(rng.integers(0, 50))))
        force_phased = bool(rng.integers(0, 3) == 0)             # reduce-scatter / all-gather in chip-wide phases
        msx.set_option("hb_phased_min_bytes", "0" if force_phased else "auto")
        msx.set_option("hb_blocks_per_rank", str(int(rng.choice([0, 1, 2]))) if force_phased else "0")
        tag["phased"] = force_phased
        try:
            g = torch.Generator().manual_seed(seed * 1000 + case)
            if dt == 3:
                x = torch.randint(-2**31, 2**31, (n, n * c), generator=g, dtype=torch.int64).to(torch.int32)
            else:
                x = (torch.randn(n, n * c, generator=g) * 3).to(tdt[dt])
            xb = view(x, dt)
            # reduce-scatter
            want = orc.allreduce_any(xb, dt, op).reshape(n, c)
            if inplace:
                buf = x.clone().cuda()
                msx.reducescatter(buf, op=op)
                msx.check_status()
                got = buf.cpu()
                got = view(got, dt)
                for r in range(n):
                    assert np.array_equal(got[r, r * c:(r + 1) * c].view(np.uint8), want[r].view(np.uint8)), ("rs", tag, r)
                    keep = np.ones(n * c, bool)
                    keep[r * c:(r + 1) * c] = False
                    assert np.array_equal(got[r][keep].view(np.uint8), xb[r][keep].view(np.uint8)), ("rs untouched", tag, r)
            else:
                send = [x[r].clone().cuda() for r in range(n)]
                recv = [torch.zeros(c, dtype=tdt[dt], device="cuda") for _ in range(n)]
                msx.reducescatter_ex(send, recv, op=op)
                msx.check_status()
                for r in range(n):
                    got = recv[r].cpu()
                    got = view(got, dt)
                    assert np.array_equal(got.view(np.uint8), want[r].view(np.uint8)), ("rs", tag, r)
            # all-gather of the first block of every row, all-to-all of the whole rows
            y = x[:, :c].contiguous()
            yb = view(y, dt)
            want_ag = orc.allgather(yb)
            want_a2a = orc.alltoall(xb)
            if inplace:
                buf = torch.zeros((n, n * c), dtype=tdt[dt])
                for r in range(n):
                    buf[r, r * c:(r + 1) * c] = y[r]
                buf = buf.cuda()
                msx.allgather(buf)
                got = buf.cpu()
                a2a = x.clone().cuda()
                msx.alltoall(a2a)
                got2 = a2a.cpu()
            else:
                send = [y[r].clone().cuda() for r in range(n)]
                recv = [torch.zeros(n * c, dtype=tdt[dt], device="cuda") for _ in range(n)]
                msx.allgather_ex(send, recv)
                got = torch.stack([t.cpu() for t in recv])
                send2 = [x[r].clone().cuda() for r in range(n)]
                recv2 = [torch.zeros(n * c, dtype=tdt[dt], device="cuda") for _ in range(n)]
                msx.alltoall_ex(send2, recv2)
                got2 = torch.stack([t.cpu() for t in recv2])
            msx.check_status()
            got, got2 = view(got, dt), view(got2, dt)
            assert np.array_equal(got.view(np.uint8), want_ag.view(np.uint8)), ("ag", tag)
            assert np.array_equal(got2.view(np.uint8), want_a2a.view(np.uint8)), ("a2a", tag)
        finally:
            msx.set_option("coll_algo", "auto")
            msx.set_option("chaos", "0")
            msx.set_option("hb_phased_min_bytes", "auto")
            msx.set_option("hb_blocks_per_rank", "0")


@pytest.mark.parametrize("seed", range(3))
def test_random_dispatch_and_combine_cases(msx, orc, seed):
    """Token counts, hidden sizes, top-k widths, expert counts and rank counts at random; receive buffers
    sometimes too small (rows beyond the capacity are dropped and reported on both sides)."""
    rng = np.random.default_rng(3000 + seed)
    for case in range(12):
        n = int(rng.choice([1, 2, 4, 8]))
        T = int(rng.integers(1, 200))
        H = int(rng.choice([8, 64, 512, 1000 // 8 * 8, 1536, 2048]))   # rows of 64, 192, 256 vectors can take the phased pack
        per_rank = int(rng.choice([1, 2, 4]))
        E = n * per_rank
        K = int(rng.integers(1, min(E, 8) + 1))
        tight = bool(rng.integers(0, 4) == 0)
        tag = dict(seed=seed, case=case, n=n, T=T, H=H, E=E, K=K, tight=tight)
        tokens = synth.moe_tokens(n, T, H, seed=seed * 100 + case)
        topk = synth.moe_routing(n, T, K, E, seed=seed * 100 + case)
        full = orc.moe_dispatch(_bits(tokens).reshape(n, T, H), topk.numpy(), E)
        most = int(full[2].sum(axis=1).max())
        cap = max(1, most // 2) if tight and most > 1 else max(1, most)
        recv_w, src_w, counts_w, rc_w = orc.moe_dispatch(_bits(tokens).reshape(n, T, H), topk.numpy(), E, cap=cap)
        # half of the cases: the pack in chip-wide read / write phases (by default only for many long rows), with
        # few workgroups per rank so that it takes several rounds
        force_phased = bool(rng.integers(0, 2))
        msx.set_option("hb_phased_min_bytes", "0" if force_phased else "auto")
        msx.set_option("hb_blocks_per_rank", str(int(rng.choice([0, 1, 2]))) if force_phased else "0")
        tag["phased"] = force_phased
        tok = [tokens[r].clone().cuda() for r in range(n)]
        idx = [topk[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros((cap, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
        src = [torch.full((cap,), -1, dtype=torch.int32, device="cuda") for _ in range(n)]
        counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
        msx.moe_dispatch(tok, idx, E, recv, counts, src)
        rc, info = msx.status()
        assert (rc == -6) == (rc_w != 0), (tag, rc, info, rc_w)
        assert rc in (0, -6), (tag, rc, info)
        # the counts are what was routed (also when rows had to be dropped), the rows that fit are the first `cap`
        assert np.array_equal(counts.cpu().numpy(), full[2]), tag
        for d in range(n):
            used = int(min(cap, full[2][d].sum()))
            assert np.array_equal(src[d].cpu().numpy()[:used], src_w[d][:used]), (tag, d)
            assert np.array_equal(_bits(recv[d])[:used], recv_w[d][:used]), (tag, d)
        if rc == 0:
            # the way back: the "experts" scale every row by a small integer that depends on the destination
            y = [(recv[d].float() * float(d % 3 + 1)).to(torch.bfloat16) for d in range(n)]
            out = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
            msx.moe_combine(y, out)
            msx.check_status()
            yb = np.stack([_bits(t) for t in y])
            want, rc2 = orc.moe_combine_bf16(yb, topk.numpy(), E)
            assert rc2 == 0
            for s in range(n):
                assert np.array_equal(_bits(out[s]), want[s]), (tag, s)
    msx.set_option("hb_phased_min_bytes", "auto")
    msx.set_option("hb_blocks_per_rank", "0")
