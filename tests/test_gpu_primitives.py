"""GPU tests of the MemoryChannel primitives on their own (through the C ABI)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def msx():
    import paper_2504_09014_amd as m
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no fallback path")
    m.init()
    yield m
    for k, v in [("drop_rank", "-1"), ("chaos", "0"), ("spin_limit", str(1 << 20))]:
        m.set_option(k, v)


def _rand_bytes(n, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randint(0, 256, (n,), generator=g, dtype=torch.uint8)


def test_pingpong_runs_and_reports_a_latency(msx):
    for a, b in [(0, 1), (0, 8), (3, 12)]:
        ns = msx.prim_pingpong(200, 16, a, b)
        assert 50.0 < ns < 1e6, (a, b, ns)


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("chans", [1, 5])
def test_barrier_rounds_advance_every_semaphore_by_k(msx, n, chans):
    before = msx.prim_barrier(0, n, chans)
    k = 17
    after = msx.prim_barrier(k, n, chans)
    diff = (after - before).astype(np.uint32)
    want = np.full((n, n), k, np.uint32)
    np.fill_diagonal(want, 0)
    assert np.array_equal(diff, want)


def test_barrier_survives_counter_wraparound(msx):
    msx.set_option("sem_base", str(2 ** 32 - 3))
    try:
        before = msx.prim_barrier(0, 8, 2)
        assert np.all(before[~np.eye(8, dtype=bool)] == 2 ** 32 - 3)
        after = msx.prim_barrier(10, 8, 2)
        assert np.all(after[~np.eye(8, dtype=bool)] == 7)          # wrapped past zero
    finally:
        msx.reset()


@pytest.mark.parametrize("nbytes", [1, 15, 16, 17, 4096 + 3, (1 << 20) + 5, 8 << 20])
@pytest.mark.parametrize("chans", [1, 7])
def test_put_signal_wait_hands_over_the_bytes(msx, nbytes, chans):
    src_h = _rand_bytes(nbytes, nbytes)
    src = src_h.cuda()
    staging = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    msx.set_option("chaos", "5")
    try:
        msx.prim_put_signal_wait(src, staging, dst, chans)
        msx.check_status()
    finally:
        msx.set_option("chaos", "0")
    assert torch.equal(dst.cpu(), src_h)
    assert torch.equal(staging.cpu(), src_h)


@pytest.mark.parametrize("nvec", [1, 255, 1024 * 4 + 3, 1 << 18])
@pytest.mark.parametrize("blocks", [1, 3, 64])
def test_stream_probe_copies_and_stays_inside_its_buffers(msx, nvec, blocks):
    """the copy mode moves every vector; read and write modes touch nothing outside [0, nbytes)"""
    nbytes = nvec * 16
    pad = 256
    src_h = _rand_bytes(nbytes + 2 * pad, nvec)
    src = src_h.cuda()
    dst = torch.full((nbytes + 2 * pad,), 0x5A, dtype=torch.uint8, device="cuda")
    msx.prim_stream(2, src[pad:pad + nbytes], dst[pad:pad + nbytes], blocks)
    msx.check_status()
    got = dst.cpu()
    assert torch.equal(got[pad:pad + nbytes], src_h[pad:pad + nbytes])
    assert torch.all(got[:pad] == 0x5A) and torch.all(got[pad + nbytes:] == 0x5A)
    msx.prim_stream(0, src[pad:pad + nbytes], None, blocks)
    dst.fill_(0x5A)
    msx.prim_stream(1, None, dst[pad:pad + nbytes], blocks)
    msx.check_status()
    got = dst.cpu()
    assert torch.all(got[:pad] == 0x5A) and torch.all(got[pad + nbytes:] == 0x5A)
    assert torch.equal(src.cpu(), src_h)


@pytest.mark.parametrize("nbytes", [1, 3, 4, 5, 8, 9, 16, 17, 1024, 1027, 100_001])
def test_ll_encode_is_byte_identical_to_the_cpu_encoder(msx, orc, nbytes):
    payload = _rand_bytes(nbytes, 77 + nbytes)
    flag = 0xA5A50000 + nbytes
    got = msx.prim_ll_encode(payload.cuda(), flag)
    msx.check_status()
    want = orc.ll_encode_buf(payload.numpy(), flag).view(np.uint8)
    assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.parametrize("nbytes", [1, 7, 8, 9, 1024, 4099, 1 << 20])
@pytest.mark.parametrize("chans", [1, 3])
def test_ll_roundtrip_delivers_payload(msx, nbytes, chans):
    payload = _rand_bytes(nbytes, 11 + nbytes)
    dst = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
    msx.set_option("chaos", "9")
    try:
        msx.prim_ll_roundtrip(payload.cuda(), dst, chans)
        msx.check_status()
    finally:
        msx.set_option("chaos", "0")
    assert torch.equal(dst.cpu(), payload)


def test_a_missing_peer_times_out_instead_of_hanging(msx):
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "1")
    try:
        src = _rand_bytes(4096, 1).cuda()
        dst = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        staging = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        # rank 1 (the waiter) is dropped here, so nothing waits: no timeout
        msx.prim_put_signal_wait(src, staging, dst, 1)
        rc, _ = msx.status()
        assert rc == 0
        msx.reset()                      # the unanswered signal must not satisfy the next wait
        msx.set_option("drop_rank", "0")
        # now the sender is gone: the waiter must give up and say who it was waiting for
        msx.prim_put_signal_wait(src, staging, dst, 1)
        rc, info = msx.status()
        assert rc == -4 and info[0] == 1 and info[1] == 1 and info[2] == 321
        # LL: the poller gives up too
        msx.prim_ll_roundtrip(src, dst, 1)
        rc, info = msx.status()
        assert rc == -4 and info[2] == 331
        # barrier with a dead rank
        msx.set_option("drop_rank", "3")
        msx.lib().msx_prim_barrier(2, 8, 1, None, None)
        rc, info = msx.status()
        assert rc == -4 and info[2] == 310
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    # after a reset everything works again
    after = msx.prim_barrier(3, 8, 1)
    assert np.all(after[~np.eye(8, dtype=bool)] == 3)


@pytest.mark.parametrize("nbytes", [16, 4096 + 3, (1 << 20) + 5, 64 << 20])
def test_port_channel_put_signal_wait_flush(msx, nbytes):
    src_h = _rand_bytes(nbytes, 5 + nbytes)
    src = src_h.cuda()
    staging = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    for _ in range(3):                                    # semaphore and FIFO positions carry over
        dst.zero_()
        torch.cuda.synchronize()
        msx.prim_port_put_signal_wait(src, staging, dst)
        msx.check_status()
        assert torch.equal(dst.cpu(), src_h)
    assert torch.equal(staging.cpu(), src_h)


def test_port_channel_waiter_times_out_without_a_sender(msx):
    src = _rand_bytes(4096, 3).cuda()
    staging = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "0")
    try:
        msx.prim_port_put_signal_wait(src, staging, dst)
        rc, info = msx.status()
        assert rc == -4 and info[2] == 502
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    msx.prim_port_put_signal_wait(src, staging, dst)      # a fresh proxy serves the next call
    msx.check_status()
    assert torch.equal(dst, src)
