"""GPU parity tests of ReduceScatter, AllGather, AllToAll (in-place and per-rank forms) and
of the token-routed dispatch, against the CPU oracle.  All comparisons are bit-exact."""
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
    m.set_option("coll_algo", "auto")


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.uint16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


def _data(n, count, dtype, seed):
    if dtype == torch.float32:
        return synth.int_valued_f32(n, count, seed=seed)
    return synth.normal(n, count, seed=seed)


def _tagged(n, count):
    """every element names its row and column: a misplaced one is attributable"""
    return ((torch.arange(n, dtype=torch.int64)[:, None] << 24) | torch.arange(count, dtype=torch.int64)[None, :]) \
        .to(torch.int32).view(torch.float32)


@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("c", [1, 3, 8, 64, 1000, 4096, 65536 + 8])
def test_reducescatter_matches_oracle(msx, orc, n, dtype, c):
    count = n * c
    x = _data(n, count, dtype, seed=c)
    want = orc.reducescatter(_bits(x))
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.zeros(c, dtype=dtype, device="cuda") for _ in range(n)]
    msx.reducescatter_ex(send, recv)
    msx.check_status()
    for r in range(n):
        assert np.array_equal(_bits(recv[r]), want[r]), (n, c, r)
    esz = 4 if dtype == torch.float32 else 2
    if (count * esz) % 16 == 0:
        buf = x.clone().cuda()
        msx.reducescatter(buf)
        msx.check_status()
        got, orig = _bits(buf), _bits(x)
        for r in range(n):
            assert np.array_equal(got[r, r * c:(r + 1) * c], want[r])
            mask = np.ones(count, bool)
            mask[r * c:(r + 1) * c] = False
            assert np.array_equal(got[r, mask], orig[r, mask])          # the rest is untouched


@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("c", [1, 5, 8, 1000, 4096, 65536 + 24])
def test_allgather_matches_oracle(msx, orc, n, dtype, c):
    x = _tagged(n, c) if dtype == torch.float32 else synth.normal(n, c, seed=c)
    want = orc.allgather(_bits(x))
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.zeros(n * c, dtype=dtype, device="cuda") for _ in range(n)]
    msx.allgather_ex(send, recv)
    msx.check_status()
    for r in range(n):
        assert np.array_equal(_bits(recv[r]).view(np.uint8), want[r].view(np.uint8)), (n, c, r)
    # in place: row r holds its block in slot r, the rest is garbage to be overwritten
    buf = torch.full((n, n * c), 7.0, dtype=dtype)
    for r in range(n):
        buf[r, r * c:(r + 1) * c] = x[r]
    buf = buf.cuda()
    msx.allgather(buf)
    msx.check_status()
    assert np.array_equal(_bits(buf).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("c", [1, 5, 8, 1000, 4096, 65536 + 24])
def test_alltoall_matches_oracle(msx, orc, n, dtype, c):
    count = n * c
    x = _tagged(n, count) if dtype == torch.float32 else synth.normal(n, count, seed=c + 1)
    want = orc.alltoall(_bits(x))
    send = [x[r].clone().cuda() for r in range(n)]
    recv = [torch.zeros(count, dtype=dtype, device="cuda") for _ in range(n)]
    msx.alltoall_ex(send, recv)
    msx.check_status()
    for r in range(n):
        assert np.array_equal(_bits(recv[r]).view(np.uint8), want[r].view(np.uint8)), (n, c, r)
    buf = x.clone().cuda()
    msx.alltoall(buf)
    msx.check_status()
    assert np.array_equal(_bits(buf).view(np.uint8), want.view(np.uint8))
    msx.alltoall(buf)                                   # applying it twice restores the input
    msx.check_status()
    assert np.array_equal(_bits(buf).view(np.uint8), _bits(x).view(np.uint8))


@pytest.mark.parametrize("n", [2, 5, 8])
@pytest.mark.parametrize("order", [1, 2])
def test_alltoall_block_after_block(msx, orc, n, order):
    """The order the large blocks take (every source on one block at a time, the ranks in step with order 2),
    forced at sizes the oracle likes: ragged ends, fewer vectors than threads, several passes per block."""
    msx.set_option("peer_outer", str(order))
    try:
        for c, blocks in [(8, 0), (8 * 300 + 16, 2), (8 * 256 * 8 * 3 + 8, 1), (8 * 70001, 4), (1 << 21, 0)]:
            count = n * c
            x = synth.normal(n, count, seed=c + order)
            want = orc.alltoall(_bits(x))
            send = [x[r].clone().cuda() for r in range(n)]
            recv = [torch.zeros(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
            msx.set_option("hb_blocks_per_rank", str(blocks))
            msx.set_option("chaos", str(c % 97 + 1))
            msx.alltoall_ex(send, recv)
            msx.check_status()
            for r in range(n):
                assert np.array_equal(_bits(recv[r]), want[r]), (n, c, r)
    finally:
        msx.set_option("peer_outer", "0")
        msx.set_option("hb_blocks_per_rank", "0")
        msx.set_option("chaos", "0")


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("c", [4, 8, 100, 4096, 65536 + 8, 262144])
def test_ll_packet_allgather_and_reducescatter(msx, orc, n, dtype, c):
    esz = 4 if dtype == torch.float32 else 2
    msx.set_option("coll_algo", "ll")
    msx.set_option("chaos", "13")
    try:
        # ReduceScatter over packets
        x = _data(n, n * c, dtype, seed=c + 3)
        send = [x[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros(c, dtype=dtype, device="cuda") for _ in range(n)]
        msx.reducescatter_ex(send, recv)
        msx.check_status()
        assert msx.last_launch()[2] == 2                      # really the packet kernel
        want = orc.reducescatter(_bits(x))
        for r in range(n):
            assert np.array_equal(_bits(recv[r]), want[r]), (n, c, r)
        # AllGather over packets, out of place and in place
        y = _tagged(n, c) if dtype == torch.float32 else synth.normal(n, c, seed=c)
        want = orc.allgather(_bits(y))
        send = [y[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros(n * c, dtype=dtype, device="cuda") for _ in range(n)]
        msx.allgather_ex(send, recv)
        msx.check_status()
        assert msx.last_launch()[2] == 1
        for r in range(n):
            assert np.array_equal(_bits(recv[r]).view(np.uint8), want[r].view(np.uint8)), (n, c, r)
        buf = torch.full((n, n * c), 7.0, dtype=dtype)
        for r in range(n):
            buf[r, r * c:(r + 1) * c] = y[r]
        buf = buf.cuda()
        msx.allgather(buf)
        msx.check_status()
        assert np.array_equal(_bits(buf).view(np.uint8), want.view(np.uint8))
    finally:
        msx.set_option("coll_algo", "auto")
        msx.set_option("chaos", "0")


def test_ll_packet_collectives_refuse_what_they_cannot_serve(msx):
    msx.set_option("coll_algo", "ll")
    try:
        send = [torch.zeros(3, dtype=torch.bfloat16, device="cuda") for _ in range(8)]      # 6-byte blocks
        recv = [torch.zeros(24, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
        with pytest.raises(msx.MsxError) as e:
            msx.allgather_ex(send, recv)
        assert e.value.code == -2
        big = int(msx.get_option("ll_max_bytes"))                                            # too large for the scratch
        send = [torch.zeros(big, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
        recv = [torch.zeros(8 * big, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
        with pytest.raises(msx.MsxError) as e:
            msx.allgather_ex(send, recv)
        assert e.value.code == -5
    finally:
        msx.set_option("coll_algo", "auto")


def test_allgather_of_reducescatter_equals_allreduce_on_gpu(msx, orc):
    n, c = 8, 12345 * 8
    x = synth.normal(n, n * c, seed=42)
    send = [x[r].clone().cuda() for r in range(n)]
    part = [torch.zeros(c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    full = [torch.zeros(n * c, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.set_option("chaos", "3")
    msx.reducescatter_ex(send, part)
    msx.allgather_ex(part, full)
    msx.set_option("chaos", "0")
    msx.check_status()
    want = orc.allreduce_bf16(_bits(x))
    for r in range(n):
        assert np.array_equal(_bits(full[r]), want)


# ---------------------------------------------------------------- token dispatch

def _dispatch(msx, tokens, topk, n_experts, cap):
    n, T, H = tokens.shape
    tok = [tokens[r].clone().cuda() for r in range(n)]
    idx = [topk[r].clone().cuda() for r in range(n)]
    recv = [torch.zeros((cap, H), dtype=tokens.dtype, device="cuda") for _ in range(n)]
    src = [torch.full((cap,), -1, dtype=torch.int32, device="cuda") for _ in range(n)]
    counts = torch.full((n, n), -1, dtype=torch.int32, device="cuda")
    msx.moe_dispatch(tok, idx, n_experts, recv, counts, src)
    rc, info = msx.status()
    return recv, src, counts, rc, info


@pytest.mark.parametrize("n,T,H,K,E", [(8, 96, 24, 8, 256), (8, 1000, 64, 8, 256), (4, 333, 8, 2, 16),
                                       (2, 5000, 40, 1, 2), (8, 1, 8, 8, 256), (1, 77, 16, 4, 8)])
def test_moe_dispatch_small_shapes(msx, orc, n, T, H, K, E):
    tokens = synth.moe_tokens(n, T, H, seed=T)
    topk = synth.moe_routing(n, T, K, E, seed=T)
    cap = n * T
    want_recv, want_src, want_counts, orc_rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, cap)
    assert orc_rc == 0
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == 0, info
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    for d in range(n):
        assert np.array_equal(src[d].cpu().numpy(), want_src[d]), d
        assert np.array_equal(_bits(recv[d]), want_recv[d]), d


@pytest.mark.parametrize("n,T,H,K,E,blocks", [(8, 1000, 512, 8, 256, 1), (8, 301, 7168, 8, 256, 2), (4, 333, 8192, 2, 16, 0),
                                              (2, 77, 1536, 1, 4, 1), (8, 3, 512, 8, 64, 1)])
def test_moe_dispatch_in_read_and_write_phases(msx, orc, n, T, H, K, E, blocks):
    """The pack kernel that alternates between chip-wide read and write phases (by default: 8 ranks, 32 MiB of
    tokens per rank; rows of whole multiples of 64 vectors), forced here; one or two workgroups per rank make
    dozens of rounds, the last one partial, with the write phases paced; token arrays that end inside a tile, and one
    smaller than a tile.  Twice in a row: the second call starts from the schedule the first one left."""
    tokens = synth.moe_tokens(n, T, H, seed=21)
    topk = synth.moe_routing(n, T, K, E, seed=21)
    cap = n * T
    want_recv, want_src, want_counts, orc_rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, cap)
    assert orc_rc == 0
    old = msx.get_option("hb_phased_min_bytes")
    msx.set_option("hb_phased_min_bytes", "0")
    msx.set_option("hb_blocks_per_rank", str(blocks))
    msx.set_option("chaos", "9")
    try:
        for rep in range(2):
            recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
            grid = msx.last_launch()[0]
            assert grid == n * blocks if blocks else (grid % n == 0 and 200 <= grid <= 256), (grid, n, blocks)
            assert rc == 0, info
            assert np.array_equal(counts.cpu().numpy(), want_counts)
            for d in range(n):
                assert np.array_equal(src[d].cpu().numpy(), want_src[d]), (rep, d)
                assert np.array_equal(_bits(recv[d]), want_recv[d]), (rep, d)
    finally:
        msx.set_option("hb_phased_min_bytes", old)
        msx.set_option("hb_blocks_per_rank", "0")
        msx.set_option("chaos", "0")


def test_phased_dispatch_and_combine_replay_in_a_hip_graph(msx, orc):
    """Dispatch (plan + pack in read and write phases, paced) and combine captured once and replayed with other
    tokens and routings of the same shape; an eager dispatch of another shape between the replays."""
    n, T, H, K, E = 8, 301, 1536, 4, 64
    cap = n * T
    cases = [(synth.moe_tokens(n, T, H, seed=60 + i), synth.moe_routing(n, T, K, E, seed=60 + i)) for i in range(3)]
    tok = [cases[0][0][r].clone().cuda() for r in range(n)]
    idx = [cases[0][1][r].clone().cuda() for r in range(n)]
    recv = [torch.zeros((cap, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    src = [torch.full((cap,), -1, dtype=torch.int32, device="cuda") for _ in range(n)]
    counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
    out = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    old = msx.get_option("hb_phased_min_bytes")
    msx.set_option("hb_phased_min_bytes", "0")
    msx.set_option("hb_blocks_per_rank", "2")
    try:
        msx.moe_dispatch(tok, idx, E, recv, counts, src)          # warm-up outside the capture (plan scratch)
        msx.moe_combine(recv, out)
        msx.check_status()
        st = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(st):
            with torch.cuda.graph(g, stream=st):
                msx.moe_dispatch(tok, idx, E, recv, counts, src)
                msx.moe_combine(recv, out)
        torch.cuda.synchronize()
        for i, (tokens, topk) in enumerate(cases):
            for r in range(n):
                tok[r].copy_(tokens[r])
                idx[r].copy_(topk[r])
                recv[r].zero_()
                src[r].fill_(-1)
                out[r].zero_()
            counts.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            msx.check_status()
            want_recv, want_src, want_counts, rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, cap)
            assert rc == 0
            assert np.array_equal(counts.cpu().numpy(), want_counts), i
            for d in range(n):
                used = int(want_counts[d].sum())
                assert np.array_equal(src[d].cpu().numpy()[:used], want_src[d][:used]), (i, d)
                assert np.array_equal(_bits(recv[d])[:used], want_recv[d][:used]), (i, d)
            want_out, rc2 = orc.moe_combine_bf16(np.stack([_bits(t) for t in recv]), topk.numpy(), E)
            assert rc2 == 0
            for s_ in range(n):
                assert np.array_equal(_bits(out[s_]), want_out[s_]), (i, s_)
            # an eager dispatch of another shape in between: the plan scratch and the pacing slots are shared
            t2 = synth.moe_tokens(n, 40, 512, seed=90 + i)
            k2 = synth.moe_routing(n, 40, 2, E, seed=90 + i)
            r2, s2, c2, rc3, info = _dispatch(msx, t2, k2, E, n * 40)
            assert rc3 == 0, info
            w2 = orc.moe_dispatch(_bits(t2), k2.numpy(), E, n * 40)
            assert np.array_equal(c2.cpu().numpy(), w2[2])
    finally:
        msx.set_option("hb_phased_min_bytes", old)
        msx.set_option("hb_blocks_per_rank", "0")


def test_moe_dispatch_special_routings(msx, orc):
    n, T, H, E = 8, 200, 32, 256
    tokens = synth.moe_tokens(n, T, H, seed=5)
    routes = {
        "all to rank 3": torch.arange(96, 104, dtype=torch.int32).repeat(n, T, 1),
        "one expert per rank": torch.arange(0, 256, 32, dtype=torch.int32).repeat(n, T, 1),
        "duplicates": torch.zeros((n, T, 8), dtype=torch.int32),
    }
    for name, topk in routes.items():
        want_recv, want_src, want_counts, _ = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, n * T)
        recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, n * T)
        assert rc == 0, (name, info)
        assert np.array_equal(counts.cpu().numpy(), want_counts), name
        for d in range(n):
            assert np.array_equal(src[d].cpu().numpy(), want_src[d]), (name, d)
            assert np.array_equal(_bits(recv[d]), want_recv[d]), (name, d)


def test_moe_dispatch_reports_overflow_and_keeps_true_counts(msx, orc):
    n, T, H, E = 8, 64, 8, 256
    tokens = synth.moe_tokens(n, T, H, seed=6)
    topk = torch.arange(0, 256, 32, dtype=torch.int32).repeat(n, T, 1)      # everything everywhere
    cap = T * 3                                                            # needs T * 8
    want_recv, _, _, orc_rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, cap)
    assert orc_rc == -1
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == -6 and info[0] == 2
    assert np.all(counts.cpu().numpy() == T)
    for d in range(n):
        assert np.array_equal(_bits(recv[d]), want_recv[d])                 # the rows that fit are right


def test_config5_moe_dispatch_full_size(msx, orc):
    n, T, H, K, E = 8, 4096, 7168, 8, 256
    tokens = synth.moe_tokens(n, T, H, seed=0)
    topk = synth.moe_routing(n, T, K, E, seed=0)
    cap = 24576                                                            # expected 21.7k rows per rank
    want_recv, want_src, want_counts, orc_rc = orc.moe_dispatch(_bits(tokens), topk.numpy(), E, cap)
    assert orc_rc == 0
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == 0, info
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    assert abs(want_counts.sum() / (n * T) - 5.295) < 0.03
    for d in range(n):
        assert np.array_equal(src[d].cpu().numpy(), want_src[d]), d
        assert np.array_equal(_bits(recv[d]), want_recv[d]), d


# ---------------------------------------------------------------- combine

@pytest.mark.parametrize("n,T,H,K,E", [(8, 96, 24, 8, 256), (8, 1000, 64, 8, 256), (4, 333, 8, 2, 16), (1, 77, 16, 4, 8)])
def test_moe_combine_small_shapes(msx, orc, n, T, H, K, E):
    tokens = synth.moe_tokens(n, T, H, seed=T + 1)
    topk = synth.moe_routing(n, T, K, E, seed=T + 1)
    cap = n * T
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == 0, info
    # "expert output": fresh random rows, so the sum is not just a multiple of the token
    y = synth.normal(n, cap * H, seed=77).view(n, cap, H)
    ydev = [y[d].clone().cuda() for d in range(n)]
    out = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.set_option("chaos", "21")
    msx.moe_combine(ydev, out)
    msx.set_option("chaos", "0")
    msx.check_status()
    want, orc_rc = orc.moe_combine_bf16(_bits(y), topk.numpy(), E)
    assert orc_rc == 0
    for s in range(n):
        assert np.array_equal(_bits(out[s]), want[s]), s


@pytest.mark.parametrize("n,T,H,K,E,blocks", [(8, 1000, 512, 8, 256, 1), (8, 300, 7168, 8, 256, 2), (4, 332, 8192, 2, 16, 0),
                                              (2, 76, 1536, 1, 4, 1), (8, 4, 512, 8, 64, 1), (8, 64, 512, 3, 8, 3)])
def test_moe_combine_in_read_and_write_phases(msx, orc, n, T, H, K, E, blocks):
    """The combine that alternates between chip-wide read and write phases (by default: 8 ranks, 32 MiB of tokens
    per rank; rows of whole multiples of 64 vectors, outputs of whole tiles), forced here; one to three
    workgroups per rank make many rounds, the last one partial.  A tile's absent rows are read as zeros from
    beyond the buffer and added as -0.0, so the "expert output" carries what that could get wrong: -0.0 and +0.0
    in all rows of a token, NaNs, infinities."""
    tokens = synth.moe_tokens(n, T, H, seed=31)
    topk = synth.moe_routing(n, T, K, E, seed=31)
    cap = n * T
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == 0, info
    y = synth.normal(n, cap * H, seed=78).view(n, cap, H).clone()
    yb = y.view(torch.int16)
    yb[:, :, 0] = -32768                                       # -0.0 in every row: the sum must stay -0.0
    yb[:, :, 1] = 0                                            # +0.0 in every row
    yb[:, ::2, 2] = -32768                                     # mixed zeros
    yb[:, ::2, 3] = 0x7FC0                                     # NaN in some rows
    yb[:, ::3, 4] = 0x7F80                                     # +inf in some rows
    ydev = [y[d].clone().cuda() for d in range(n)]
    out = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    want, orc_rc = orc.moe_combine_bf16(_bits(y), topk.numpy(), E)
    assert orc_rc == 0
    old = msx.get_option("hb_phased_min_bytes")
    msx.set_option("hb_phased_min_bytes", "0")
    msx.set_option("hb_blocks_per_rank", str(blocks))
    msx.set_option("chaos", "21")
    try:
        for rep in range(2):
            msx.moe_combine(ydev, out)
            grid = msx.last_launch()[0]
            assert grid == n * blocks if blocks else (grid % n == 0 and 200 <= grid <= 256), (grid, n, blocks)
            msx.check_status()
            for s_ in range(n):
                assert np.array_equal(_bits(out[s_]), want[s_]), (rep, s_)
                out[s_].fill_(float("nan"))
    finally:
        msx.set_option("hb_phased_min_bytes", old)
        msx.set_option("hb_blocks_per_rank", "0")
        msx.set_option("chaos", "0")


def test_moe_combine_needs_a_matching_dispatch(msx):
    y = [torch.zeros((16, 8), dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    out = [torch.zeros((12345, 8), dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.moe_combine(y, out)
    assert e.value.code == -1


def test_config5_moe_combine_full_size(msx, orc):
    n, T, H, K, E = 8, 4096, 7168, 8, 256
    tokens = synth.moe_tokens(n, T, H, seed=0)
    topk = synth.moe_routing(n, T, K, E, seed=0)
    cap = 24576
    recv, src, counts, rc, info = _dispatch(msx, tokens, topk, E, cap)
    assert rc == 0, info
    # combine what was dispatched (rows stay on the GPU): out = fan-out copies of the token summed
    out = [torch.empty((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.moe_combine(recv, out)
    msx.check_status()
    y = np.stack([_bits(r) for r in recv])
    want, orc_rc = orc.moe_combine_bf16(y, topk.numpy(), E)
    assert orc_rc == 0
    for s in range(n):
        assert np.array_equal(_bits(out[s]), want[s]), s


# ---------------------------------------------------------------- FP8 dispatch

@pytest.mark.parametrize("n,T,H,K,E", [(8, 96, 128, 8, 256), (8, 500, 512, 8, 256), (4, 333, 256, 2, 16), (8, 64, 7168, 8, 256)])
def test_moe_dispatch_fp8_matches_quantise_then_dispatch(msx, orc, n, T, H, K, E):
    tokens = synth.moe_tokens(n, T, H, seed=T + 5)
    tokens[0, 0, :128] = 0                                      # an all-zero group (amax clamps at 1e-4)
    tokens[0, 1, 5] = 1000.0                                    # an outlier that sets its group's scale
    tokens[1 % n, 2, 7] = float("inf")
    topk = synth.moe_routing(n, T, K, E, seed=T + 5)
    cap = n * T
    tb = _bits(tokens)
    q, scales = orc.fp8_quantize_rows(tb.reshape(n * T, H))
    want_q, want_src, want_counts, orc_rc = orc.moe_dispatch(q.reshape(n, T, H), topk.numpy(), E, cap)
    want_s, _, _, _ = orc.moe_dispatch(scales.reshape(n, T, H // 128), topk.numpy(), E, cap)
    assert orc_rc == 0
    tok = [tokens[r].clone().cuda() for r in range(n)]
    idx = [topk[r].clone().cuda() for r in range(n)]
    rq = [torch.zeros((cap, H), dtype=torch.uint8, device="cuda") for _ in range(n)]
    rs = [torch.zeros((cap, H // 128), dtype=torch.float32, device="cuda") for _ in range(n)]
    src = [torch.full((cap,), -1, dtype=torch.int32, device="cuda") for _ in range(n)]
    counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
    msx.moe_dispatch_fp8(tok, idx, E, rq, rs, counts, src)
    msx.check_status()
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    for d in range(n):
        assert np.array_equal(src[d].cpu().numpy(), want_src[d]), d
        assert np.array_equal(rq[d].cpu().numpy(), want_q[d]), d
        assert np.array_equal(rs[d].cpu().numpy().view(np.uint32), want_s[d].view(np.uint32)), d


def test_e4m3_encoder_on_gpu_covers_every_code_and_tie(msx, orc):
    # one row whose groups hold hand-picked values scaled so that x * (448 / amax) hits exact
    # codes, ties and the subnormal range: group amax is pinned to 448 by one element
    vals = [orc.e4m3_to_f32(c) for c in range(0x7F)]
    probes = []
    for a, b in zip(vals[:-1], vals[1:]):
        probes += [a, (a + b) / 2]                               # every code and every tie
    probes += [448.0, -448.0, 0.0, -0.0]
    probes = [p for p in probes if float(torch.tensor(p).bfloat16()) == p]     # representable in bf16
    H = 128 * ((len(probes) + 126) // 127)
    row = torch.zeros(H)
    k = 0
    for g in range(H // 128):
        row[g * 128] = 448.0
        for j in range(1, 128):
            if k < len(probes):
                row[g * 128 + j] = probes[k]
                k += 1
    tokens = row.bfloat16().view(1, 1, H).repeat(8, 1, 1)
    topk = torch.arange(0, 256, 32, dtype=torch.int32).repeat(8, 1, 1)
    q, scales = orc.fp8_quantize_rows(_bits(tokens).reshape(8, H))
    tok = [tokens[r].clone().cuda() for r in range(8)]
    idx = [topk[r].clone().cuda() for r in range(8)]
    rq = [torch.zeros((8, H), dtype=torch.uint8, device="cuda") for _ in range(8)]
    rs = [torch.zeros((8, H // 128), dtype=torch.float32, device="cuda") for _ in range(8)]
    counts = torch.zeros((8, 8), dtype=torch.int32, device="cuda")
    msx.moe_dispatch_fp8(tok, idx, 256, rq, rs, counts)
    msx.check_status()
    assert np.all(counts.cpu().numpy() == 1)
    assert np.all(scales == 1.0)
    for d in range(8):
        assert np.array_equal(rq[d].cpu().numpy(), q), d


def test_fp8_pack_special_values(msx, orc):
    """NaN, infinities, signed zeros, values under the 1e-4 floor of the group maximum and the largest bf16
    magnitudes: groups of their own, every code and every scale bit for bit against the oracle."""
    H = 128 * 8
    row = torch.zeros(H)
    rng = np.random.default_rng(5)
    g = lambda k: slice(128 * k, 128 * k + 128)
    row[g(0)] = torch.tensor(rng.standard_normal(128), dtype=torch.float32)
    row[3] = float("nan"); row[77] = float("nan")
    row[g(1)] = torch.tensor(rng.standard_normal(128), dtype=torch.float32)
    row[128 + 9] = float("inf")
    row[g(2)] = torch.tensor(rng.standard_normal(128), dtype=torch.float32)
    row[256 + 100] = float("-inf"); row[256 + 5] = float("nan")
    row[g(3)] = torch.tensor(rng.standard_normal(128) * 1e-6, dtype=torch.float32)       # all under the floor
    row[g(4)] = torch.tensor(rng.standard_normal(128), dtype=torch.float32) * 3e38       # overflows bf16 in places
    row[g(5)] = 0.0
    row[640 + 1] = -0.0; row[640 + 2] = 1.0; row[640 + 3] = -1e-6; row[640 + 4] = 1e-6
    row[g(6)] = torch.tensor(rng.standard_normal(128), dtype=torch.float32) * 1e-30
    row[g(7)] = torch.tensor(rng.integers(-448, 449, 128), dtype=torch.float32)
    tokens = row.bfloat16().view(1, 1, H).repeat(8, 1, 1)
    topk = torch.arange(0, 256, 32, dtype=torch.int32).repeat(8, 1, 1)
    q, scales = orc.fp8_quantize_rows(_bits(tokens).reshape(8, H))
    assert 0x7F in q[0] and 0x80 in q[0] and np.isinf(scales[0]).any()
    tok = [tokens[r].clone().cuda() for r in range(8)]
    idx = [topk[r].clone().cuda() for r in range(8)]
    rq = [torch.zeros((8, H), dtype=torch.uint8, device="cuda") for _ in range(8)]
    rs = [torch.zeros((8, H // 128), dtype=torch.float32, device="cuda") for _ in range(8)]
    counts = torch.zeros((8, 8), dtype=torch.int32, device="cuda")
    msx.moe_dispatch_fp8(tok, idx, 256, rq, rs, counts)
    msx.check_status()
    for d in range(8):
        assert np.array_equal(rq[d].cpu().numpy(), q), (d, np.nonzero(rq[d].cpu().numpy() != q))
        assert np.array_equal(rs[d].cpu().numpy().view(np.uint32), scales.view(np.uint32)), d


# ---------------------------------------------------------------- fp16 and max / min

# fp32 / bf16 sums are the tuned paths, tested above: here every other (type, operator) pair
@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("dt,op", [(0, 1), (0, 2), (1, 1), (1, 2), (2, 0), (2, 1), (2, 2), (3, 0), (3, 1), (3, 2)])
def test_fp16_and_max_min_allreduce_reducescatter(msx, orc, n, dt, op):
    tdt = [torch.float32, torch.bfloat16, torch.float16, torch.int32][dt]
    for count in [1, 7, 8 * n, 1000 * n, 70001 * n]:
        g = torch.Generator().manual_seed(count + dt + 10 * op)
        if dt == 3:
            x = torch.randint(-2**31, 2**31, (n, count), generator=g, dtype=torch.int64).to(torch.int32)   # sums wrap
        else:
            xf = torch.randn(n, count, generator=g) * 3
            if count > 100:
                xf[0, 5] = float("inf")
                xf[n - 1, 6] = float("-inf")
                xf[0, 7] = 6.0e-6                               # fp16 subnormal territory
            x = xf.to(tdt)
        bits = x.view(torch.uint16).numpy() if dt in (1, 2) else x.numpy()
        want = orc.allreduce_any(bits, dt, op)
        send = [x[r].clone().cuda() for r in range(n)]
        recv = [torch.zeros_like(t) for t in send]
        msx.set_option("chaos", "4")
        msx.allreduce_ex(send, recv, None, op=op)
        msx.check_status()
        for r in range(n):
            got = recv[r].cpu()
            got = got.view(torch.uint16).numpy() if dt in (1, 2) else got.numpy()
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (n, dt, op, count, r)
        if count % n == 0:
            c = count // n
            part = [torch.zeros(c, dtype=tdt, device="cuda") for _ in range(n)]
            msx.reducescatter_ex(send, part, op=op)
            msx.check_status()
            for r in range(n):
                got = part[r].cpu()
                got = got.view(torch.uint16).numpy() if dt in (1, 2) else got.numpy()
                assert np.array_equal(got.view(np.uint8), want[r * c:(r + 1) * c].view(np.uint8)), (n, dt, op, count, r)
        msx.set_option("chaos", "0")


def test_generic_reduce_refuses_what_it_does_not_cover(msx):
    send = [torch.zeros(64, dtype=torch.float16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, send)                      # residual with fp16
    assert e.value.code == -2
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, None, algo=1)              # no LL form for fp16
    assert e.value.code == -2
    f = [torch.zeros(64, dtype=torch.float32, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(f, f, None, algo=5, op=msx.MAX)        # no ring form for max
    assert e.value.code == -2
    i = [torch.zeros(64, dtype=torch.int32, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(i, i, None, algo=2)                    # no LL form for int32
    assert e.value.code == -2


@pytest.mark.parametrize("dtype", [torch.float16, torch.int32])
def test_combine_refuses_types_it_has_no_sum_for(msx, dtype):
    n, T, H, K, E = 2, 4, 8, 1, 2
    tok = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    idx = [torch.zeros((T, K), dtype=torch.int32, device="cuda") for _ in range(n)]
    recv = [torch.zeros((n * T, H), dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    src = [torch.zeros((n * T,), dtype=torch.int32, device="cuda") for _ in range(n)]
    counts = torch.zeros((n, n), dtype=torch.int32, device="cuda")
    msx.moe_dispatch(tok, idx, E, recv, counts, src)
    msx.check_status()
    y = [torch.zeros((n * T, H), dtype=dtype, device="cuda") for _ in range(n)]
    out = [torch.zeros((T, H), dtype=dtype, device="cuda") for _ in range(n)]
    with pytest.raises(msx.MsxError) as e:
        msx.moe_combine(y, out)
    assert e.value.code == -2


def test_copy_collectives_take_int32(msx, orc):
    n, c = 8, 999
    x = torch.randint(-2**31, 2**31, (n, n * c), dtype=torch.int64).to(torch.int32)
    want = orc.alltoall(x.numpy())
    buf = x.clone().cuda()
    msx.alltoall(buf)
    msx.check_status()
    assert np.array_equal(buf.cpu().numpy(), want)
    y = x[:, :c].contiguous()
    recv = [torch.zeros(n * c, dtype=torch.int32, device="cuda") for _ in range(n)]
    msx.allgather_ex([y[r].cuda() for r in range(n)], recv)
    msx.check_status()
    assert np.array_equal(torch.stack([t.cpu() for t in recv]).numpy(), orc.allgather(y.numpy()))


def test_copy_collectives_take_fp16(msx, orc):
    n, c = 8, 1000
    x = (torch.randn(n, n * c) * 3).half()
    want = orc.alltoall(x.view(torch.uint16).numpy())
    buf = x.clone().cuda()
    msx.alltoall(buf)
    msx.check_status()
    assert np.array_equal(buf.cpu().view(torch.uint16).numpy(), want)


# ---------------------------------------------------------------- ReduceScatter / AllGather in chip-wide phases

@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_phased_reducescatter_and_allgather_match_oracle(msx, orc, n, dtype):
    """The forms that alternate between chip-wide read and write phases (by default: 8 ranks, rows from 64 MiB),
    forced at sizes the oracle likes: 1 or 2 workgroups per rank make several rounds of 64 tiles of 256 vectors
    (the last round partial), blocks end in a partial tile; in place and out of place."""
    epv = 4 if dtype == torch.float32 else 8
    old = msx.get_option("hb_phased_min_bytes")
    msx.set_option("hb_phased_min_bytes", "0")
    try:
        for blocks, vecs in [(1, 256 * 64 * 2 + 256 * 3 + 5), (2, 256 * 64 * 2 * 2 + 256), (1, 200), (0, 256 * 9 + 1)]:
            c = vecs * epv
            msx.set_option("hb_blocks_per_rank", str(blocks))
            msx.set_option("chaos", str(3 + blocks))
            x = _data(n, n * c, dtype, seed=vecs % 1000)
            want = orc.reducescatter(_bits(x))
            send = [x[r].clone().cuda() for r in range(n)]
            recv = [torch.zeros(c, dtype=dtype, device="cuda") for _ in range(n)]
            msx.reducescatter_ex(send, recv)
            msx.check_status()
            grid = msx.last_launch()[0]
            assert grid == n * blocks if blocks else (grid % n == 0 and 200 <= grid <= 256), (grid, n, blocks)
            for r in range(n):
                assert np.array_equal(_bits(recv[r]), want[r]), ("rs", n, blocks, vecs, r)
            buf = x.clone().cuda()
            msx.reducescatter(buf)
            msx.check_status()
            got, orig = _bits(buf), _bits(x)
            for r in range(n):
                assert np.array_equal(got[r, r * c:(r + 1) * c], want[r]), ("rs in place", n, blocks, vecs, r)
                mask = np.ones(n * c, bool)
                mask[r * c:(r + 1) * c] = False
                assert np.array_equal(got[r, mask], orig[r, mask])
            y = x[:, :c].contiguous()
            want_ag = orc.allgather(_bits(y))
            out = [torch.zeros(n * c, dtype=dtype, device="cuda") for _ in range(n)]
            msx.allgather_ex([y[r].clone().cuda() for r in range(n)], out)
            msx.check_status()
            grid = msx.last_launch()[0]
            assert grid == n * blocks if blocks else (grid % n == 0 and 200 <= grid <= 256), (grid, n, blocks)
            for r in range(n):
                assert np.array_equal(_bits(out[r]), want_ag[r]), ("ag", n, blocks, vecs, r)
            buf = torch.zeros((n, n * c), dtype=dtype)
            for r in range(n):
                buf[r, r * c:(r + 1) * c] = y[r]
            buf = buf.cuda()
            msx.allgather(buf)
            msx.check_status()
            assert np.array_equal(_bits(buf), want_ag), ("ag in place", n, blocks, vecs)
    finally:
        msx.set_option("hb_phased_min_bytes", old)
        msx.set_option("hb_blocks_per_rank", "0")
        msx.set_option("chaos", "0")


# ---------------------------------------------------------------- packet kernels, ragged sizes, many calls

def test_packet_kernels_with_a_one_lane_tail_never_stall(msx, orc):
    """Packet counts that leave a single lane with one more packet than the rest of its wave, every
    packet kernel, a few thousand calls each: a wave whose lanes leave the send loop at different
    iterations must not change what the receive loop polls (a wave-uniform condition kept as a lane
    mask once did, and a rank then waited on its own, never written, slot about once in 600 calls)."""
    n, calls = 8, 2500

    def hammer(name, fn):
        for it in range(calls):
            fn()
            rc, info = msx.status()
            assert rc == 0, (name, it, rc, info, msx.get_option("status_detail"))

    for c in [65544, 100]:
        msx.set_option("coll_algo", "ll")
        try:
            y = _tagged(n, c)
            buf = torch.full((n, n * c), 7.0)
            for r in range(n):
                buf[r, r * c:(r + 1) * c] = y[r]
            d = buf.cuda()
            hammer(f"allgather c={c}", lambda: msx.allgather(d))
            assert msx.last_launch()[2] == 1
            assert np.array_equal(_bits(d).view(np.uint8), orc.allgather(_bits(y)).view(np.uint8))
            x = _data(n, n * c, torch.float32, seed=c)
            send = [x[r].clone().cuda() for r in range(n)]
            recv = [torch.zeros(c, device="cuda") for _ in range(n)]
            hammer(f"reducescatter c={c}", lambda: msx.reducescatter_ex(send, recv))
            assert msx.last_launch()[2] == 2
            want = orc.reducescatter(_bits(x))
            for r in range(n):
                assert np.array_equal(_bits(recv[r]), want[r]), (c, r)
        finally:
            msx.set_option("coll_algo", "auto")
    for count in [2 * 32769, 14]:
        x = _data(n, count, torch.float32, seed=count)
        want = orc.allreduce_f32(x.numpy())
        for algo in [msx.ALGO_1PA_LL, msx.ALGO_2PA_LL]:
            send = [x[r].clone().cuda() for r in range(n)]
            recv = [torch.zeros(count, device="cuda") for _ in range(n)]
            hammer(f"allreduce algo={algo} count={count}", lambda: msx.allreduce_ex(send, recv, None, algo=algo))
            for r in range(n):
                assert np.array_equal(recv[r].cpu().numpy().view(np.uint8), want.view(np.uint8)), (algo, count, r)
