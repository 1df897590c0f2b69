"""The entry point that allocates nothing (msx_allreduce_ex_static) against msx_allreduce_ex,
through the C ABI: same inputs, bit-identical outputs, two calls in a row, the second smaller
(the fixed scratch array keeps the first call's packets and counters)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2504_09014_amd import synth

pytestmark = pytest.mark.gpu

ALGOS = {"auto": 0, "1pa_ll": 1, "2pa_ll": 2, "2pa_hb": 3, "2pa_hb_2phase": 4}


@pytest.fixture(scope="module")
def msx():
    import paper_2504_09014_amd as m
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no fallback path")
    m.init()
    return m


def _table(ts):
    return C.cast((C.c_void_p * len(ts))(*[t.data_ptr() for t in ts]), C.POINTER(C.c_void_p))


def _call(msx, fn, x, algo, res=None):
    n = x.shape[0]
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.full_like(s, float("nan")) for s in send]
    rt = _table(res) if res is not None else None
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    dt = msx.BF16 if x.dtype == torch.bfloat16 else msx.F32
    rc = fn(_table(send), _table(recv), rt, x.shape[1], dt, msx.SUM, n, algo, st)
    assert rc == 0, msx.strerror(rc)
    msx.check_status()
    return [r.cpu().view(torch.uint16 if x.dtype == torch.bfloat16 else torch.int32).numpy() for r in recv]


@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("n", [8, 5])
def test_two_calls_in_a_row_match_the_allocating_entry_point(msx, orc, algo, n):
    L = msx.lib()
    big, small = (8192, 1000) if algo == "1pa_ll" else (32768, 4104) if algo == "2pa_ll" else (262144 + 24, 3000)
    for count, seed in [(big, 11), (small, 12)]:          # the second call is the smaller one
        x = synth.normal(n, count, seed=seed)
        want = _call(msx, L.msx_allreduce_ex, x, ALGOS[algo])
        got = _call(msx, L.msx_allreduce_ex_static, x, ALGOS[algo])
        ref = orc.allreduce_bf16(synth.bf16_bits(x))
        for r in range(n):
            assert np.array_equal(got[r], want[r]), (algo, n, count, r)
            assert np.array_equal(got[r], ref), (algo, n, count, r)


def test_fp32_with_residual_and_limits(msx, orc):
    L = msx.lib()
    n = 8
    x = synth.int_valued_f32(n, 5000, seed=5)
    res = [synth.int_valued_f32(1, 5000, seed=6)[0].cuda()] * n
    a = _call(msx, L.msx_allreduce_ex, x, 0, res)
    b = _call(msx, L.msx_allreduce_ex_static, x, 0, res)
    for r in range(n):
        assert np.array_equal(a[r], b[r])
    # beyond the fixed array: refused, nothing launched
    t = [torch.zeros(16, device="cuda")] * n
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.msx_allreduce_ex_static(_table(t), _table(t), None, (16 << 20) // 4 + 4, msx.F32, 0, n, 0, st) == -5
    assert L.msx_allreduce_ex_static(_table(t), _table(t), None, (80 << 10) // 4, msx.F32, 0, n, 2, st) == -5
    assert L.msx_allreduce_ex_static(_table(t), _table(t), None, 1024, msx.F32, 0, n, 5, st) == -2
    assert L.msx_allreduce_ex_static(_table(t), _table(t), None, 1024, msx.F32, 0, n, 6, st) == -2


def test_no_device_allocation_happens_inside_the_call(msx):
    n = 8
    x = synth.normal(n, 4096, seed=3)
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.empty_like(s) for s in send]
    msx.allreduce_ex_static(send, recv, algo=2)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for algo in (0, 1, 2, 3, 4):
        msx.allreduce_ex_static(send, recv, algo=algo)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    msx.check_status()
