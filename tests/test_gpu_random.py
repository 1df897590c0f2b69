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
                dict(seed=seed, case=case, n=n, bf16=bf16, count=count, algo=algo, res=res_mode, inplace=inplace, rank=r)
    msx.set_option("chaos", "0")
