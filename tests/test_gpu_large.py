"""Config 3: bandwidth-path AllReduce at 64 MiB, 256 MiB and 1 GiB per rank (bf16, 8 ranks,
out of place), in the launch configuration the benchmark times.

64 MiB is compared with the oracle in full.  At 256 MiB and 1 GiB the oracle runs on
deterministic windows (start and end of every rank's chunk, a band around every chunk
boundary, 48 seeded 64 KiB windows) and an on-GPU comparison checks that all 8 outputs are
bitwise identical, so a fault anywhere outside the windows still shows on at least the
cross-rank check or as a wrong window."""
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
    return m


def _bits(t):
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()


def _windows(count, n, rng):
    w = 32768                                              # 64 KiB of bf16
    spans = []
    chunk = count // n
    for r in range(n):
        lo = r * chunk
        spans += [(lo, min(count, lo + (1 << 19))), (max(0, lo + chunk - (1 << 19)), lo + chunk),
                  (max(0, lo - 2048), min(count, lo + 2048))]
    for s in rng.integers(0, count - w, 48):
        spans.append((int(s), int(s) + w))
    spans.append((count - 4096, count))
    return spans


# 3, 8 and 24 MiB: the cache-keeping forms of the fused kernel (loads and stores / stores only); 4 GiB: 2^31
# elements per rank (64-bit indexing everywhere), 64 rounds of the phased kernel with paced write phases
@pytest.mark.parametrize("mib,algo", [(3, 3), (8, 3), (24, 3), (64, 3), (64, 4), (256, 3), (1024, 3), (4096, 3)])
def test_config3_large_allreduce(msx, orc, mib, algo):
    n = 8
    count = mib * (1 << 20) // 2
    x = synth.normal(n, count, seed=mib, device="cuda")     # generated on the GPU by torch
    send = [x[r] for r in range(n)]
    recv = [torch.empty(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.allreduce_ex(send, recv, None, algo=algo)
    msx.check_status()
    for r in range(1, n):
        assert torch.equal(recv[r].view(torch.int16), recv[0].view(torch.int16)), r
    if mib <= 64:
        want = orc.allreduce_bf16(_bits(x))
        assert np.array_equal(_bits(recv[0]), want)
        assert np.array_equal(_bits(recv[5]), want)
    else:
        rng = np.random.default_rng(mib)
        for lo, hi in _windows(count, n, rng):
            want = orc.allreduce_bf16(_bits(x[:, lo:hi]))
            assert np.array_equal(_bits(recv[0][lo:hi]), want), (lo, hi)
            assert np.array_equal(_bits(recv[6][lo:hi]), want), (lo, hi)
    del x, send, recv
    torch.cuda.empty_cache()


def test_large_in_place_allreduce_256mib(msx, orc):
    n, count = 8, 128 << 20
    x = synth.normal(n, count, seed=7, device="cuda")
    keep = {}
    rng = np.random.default_rng(1)
    spans = _windows(count, n, rng)
    for lo, hi in spans:
        keep[(lo, hi)] = orc.allreduce_bf16(_bits(x[:, lo:hi]))
    msx.allreduce(x)
    msx.check_status()
    for r in range(1, n):
        assert torch.equal(x[r].view(torch.int16), x[0].view(torch.int16)), r
    for (lo, hi), want in keep.items():
        assert np.array_equal(_bits(x[3, lo:hi]), want), (lo, hi)
    del x
    torch.cuda.empty_cache()


@pytest.mark.parametrize("block_mib", [2, 32, 128])
def test_large_reducescatter_allgather_alltoall(msx, orc, block_mib):
    """The standalone collectives at the sizes the benchmark times (rows of 16 MiB, 256 MiB and 1 GiB: the
    cache-keeping stores, the streaming forms and the deep-unrolled AllGather).  The oracle checks seeded
    sample columns of every block; on the GPU every output is compared in full with what the copy collectives
    must produce, and the reduce-scatter with the same columns summed by the AllReduce kernel."""
    n = 8
    c = block_mib * (1 << 20) // 2                           # bf16 elements per block
    rng = np.random.default_rng(block_mib)
    cols = np.unique(np.concatenate([rng.integers(0, c, 4096), np.arange(0, 4096), np.arange(c - 4096, c)]))
    ti = torch.from_numpy(cols).cuda()

    # AllGather: block r of every output is rank r's input
    part = [synth.normal(1, c, seed=100 + r, device="cuda")[0] for r in range(n)]
    full = [torch.empty(n * c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.allgather_ex(part, full)
    msx.check_status()
    ref = torch.cat(part)
    for r in range(n):
        assert torch.equal(full[r].view(torch.int16), ref.view(torch.int16)), r
    small = np.stack([_bits(p[ti]) for p in part])
    want = orc.allgather(small)                                # [n, n * K]
    for r in (0, 5):
        got = _bits(full[r].view(n, c)[:, ti].reshape(-1))
        assert np.array_equal(got, want[r]), r

    # AllToAll of the gathered rows: out[d] block s = in[s] block d (all inputs are equal here, so also
    # scramble them first: row s gets its blocks rotated by s)
    rows = [torch.roll(full[s].view(n, c), shifts=s, dims=0).reshape(-1).contiguous() for s in range(n)]
    out = [torch.empty(n * c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.alltoall_ex(rows, out)
    msx.check_status()
    for d in range(n):
        expect = torch.stack([rows[s].view(n, c)[d] for s in range(n)]).reshape(-1)
        assert torch.equal(out[d].view(torch.int16), expect.view(torch.int16)), d
    small = np.stack([_bits(rows[s].view(n, c)[:, ti].reshape(-1)) for s in range(n)])
    want = orc.alltoall(small)
    for d in (0, 3):
        assert np.array_equal(_bits(out[d].view(n, c)[:, ti].reshape(-1)), want[d]), d
    del full, out

    # ReduceScatter of those rows
    rs = [torch.empty(c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.reducescatter_ex(rows, rs)
    msx.check_status()
    want = orc.reducescatter(small)                            # [n, K]
    for r in range(n):
        assert np.array_equal(_bits(rs[r][ti]), want[r]), r
    # ... and in full against the AllReduce kernel's sums of the same rows (same order, same rounding)
    ar = [torch.empty(n * c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.allreduce_ex(rows, ar, None)
    msx.check_status()
    for r in range(n):
        assert torch.equal(rs[r].view(torch.int16), ar[0].view(n, c)[r].view(torch.int16)), r
