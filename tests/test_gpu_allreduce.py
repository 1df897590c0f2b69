"""GPU parity tests of AllReduce (1PA-LL, 2PA-LL, 2PA-HB fused and two-phase) against the
CPU oracle, element by element, through the C ABI.

Tolerances: the kernels add in fp32 in rank order 0..N-1 and round once, exactly like the
oracle, so every comparison here is BIT-EXACT (fp32 and bf16 alike); the looser bounds of
the benchmark spec (1 bf16 ulp vs fp64 for a fixed order) follow from the oracle's own pins.
"""
import numpy as np
import pytest
import torch

from paper_2504_09014_amd import synth

pytestmark = pytest.mark.gpu

ALGOS = {"1pa_ll": 1, "2pa_ll": 2, "2pa_hb": 3, "2pa_hb_2phase": 4}


@pytest.fixture(scope="module")
def msx():
    import paper_2504_09014_amd as m
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no fallback path")
    m.init()
    yield m
    m.set_option("chaos", "0")
    m.set_option("algo", "auto")


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.uint16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


def _oracle(orc, x):
    return orc.allreduce_bf16(_bits(x)) if x.dtype == torch.bfloat16 else orc.allreduce_f32(_bits(x))


def _run_ex(msx, x, algo, residual=None, inplace=False):
    """x: [n, count] CPU tensor.  Returns list of n output rows (numpy bit views)."""
    n = x.shape[0]
    send = [x[r].clone().cuda() for r in range(n)]            # separate allocations: any count is aligned
    recv = send if inplace else [torch.full_like(s, float("nan")) for s in send]
    res = None
    if residual is not None:
        if isinstance(residual, torch.Tensor) and residual.dim() == 1:
            shared = residual.cuda()
            res = [shared] * n
        else:
            res = [residual[r].clone().cuda() for r in range(n)]
    msx.allreduce_ex(send, recv, res, algo=algo)
    msx.check_status()
    return [_bits(r) for r in recv]


# ---------------------------------------------------------------- config 1

@pytest.mark.parametrize("algo", list(ALGOS))
def test_config1_integer_valued_fp32_bit_exact(msx, orc, algo):
    x = synth.int_valued_f32(8, 262144, seed=0)
    want = orc.allreduce_f32(x.numpy())
    assert np.array_equal(want.astype(np.int64), orc.allreduce_f32_as_i64(x.numpy()))
    outs = _run_ex(msx, x, ALGOS[algo])
    for r in range(8):
        assert np.array_equal(outs[r].view(np.uint32), want.view(np.uint32)), (algo, r)


def test_config1_in_place_contiguous_form_auto_algorithm(msx, orc):
    x = synth.int_valued_f32(8, 262144, seed=0)
    want = orc.allreduce_f32(x.numpy())
    buf = x.cuda()
    msx.allreduce(buf)
    msx.check_status()
    got = buf.cpu().numpy()
    for r in range(8):
        assert np.array_equal(got[r], want)


# ---------------------------------------------------------------- config 2: bf16 size sweep

@pytest.mark.parametrize("kib", [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_config2_bf16_sweep_all_algorithms_agree_with_oracle(msx, orc, kib):
    count = kib * 1024 // 2
    x = synth.normal(8, count, seed=kib)
    want = _oracle(orc, x)
    for name, algo in ALGOS.items():
        outs = _run_ex(msx, x, algo)
        for r in range(8):
            assert np.array_equal(outs[r], want), (name, kib, r)
    # automatic choice, in place, contiguous buffer
    buf = x.cuda()
    msx.allreduce(buf)
    msx.check_status()
    assert np.array_equal(_bits(buf), np.tile(want, (8, 1)))


# ---------------------------------------------------------------- ragged sizes, rank counts

@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_ragged_counts_and_rank_counts(msx, orc, n, dtype):
    for count in [1, 2, 3, 7, 8, 9, 15, 16, 17, 63, 64, 65, 1023, 1024, 1025, 4099, 70001]:
        x = synth.int_valued_f32(n, count, seed=count) if dtype == torch.float32 else synth.normal(n, count, seed=count)
        want = _oracle(orc, x)
        for name, algo in ALGOS.items():
            for inplace in (False, True):
                outs = _run_ex(msx, x, algo, inplace=inplace)
                for r in range(n):
                    assert np.array_equal(outs[r], want), (name, n, count, r, inplace)


def test_order_sensitive_inputs_follow_rank_order(msx):
    # (2^24 + 1) - 2^24 in fp32: 0 in rank order, 1 if the cancelling pair were added first
    x = torch.zeros(8, 64, dtype=torch.float32)
    x[0] = 2.0 ** 24
    x[1] = 1.0
    x[2] = -(2.0 ** 24)
    y = x[[0, 2, 1, 3, 4, 5, 6, 7]]
    for name, algo in ALGOS.items():
        assert all(np.all(o == 0.0) for o in _run_ex(msx, x, algo)), name
        assert all(np.all(o == 1.0) for o in _run_ex(msx, y, algo)), name


def test_ieee_special_values(msx, orc):
    x = torch.zeros(8, 16, dtype=torch.float32)
    x[:, 0] = -0.0
    x[0, 1] = float("inf")
    x[0, 2], x[1, 2] = float("inf"), float("-inf")
    x[3, 3] = float("nan")
    x[:, 4] = 1e-40                                          # fp32 subnormals must not be flushed
    want = orc.allreduce_f32(x.numpy())
    xb = x.bfloat16()
    wantb = orc.allreduce_bf16(_bits(xb))
    for name, algo in ALGOS.items():
        for o in _run_ex(msx, x, algo):
            assert np.array_equal(o.view(np.uint32)[[0, 1, 4]], want.view(np.uint32)[[0, 1, 4]]), name
            assert np.isnan(o[2]) and np.isnan(o[3])
        for o in _run_ex(msx, xb, algo):
            assert np.array_equal(o[[0, 1, 4]], wantb[[0, 1, 4]]), name


# ---------------------------------------------------------------- config 4: decode shape + residual

@pytest.mark.parametrize("T", [1, 8, 32, 128, 256])
def test_config4_decode_allreduce_with_fused_residual(msx, orc, T):
    x, res = synth.decode_activations(8, T, hidden=8192, seed=T)
    want = orc.allreduce_residual_bf16(_bits(x), _bits(res))
    one_phase_limit = int(msx.get_option("ll_max_bytes")) // 4      # 1PA keeps n full copies per rank
    for name, algo in ALGOS.items():
        if name == "1pa_ll" and T * 8192 * 2 > one_phase_limit:
            continue
        outs = _run_ex(msx, x, algo, residual=res)
        for r in range(8):
            assert np.array_equal(outs[r], want), (name, T, r)


def test_residual_per_rank_and_degenerate_cases(msx, orc):
    n, count = 8, 8192 + 24
    x = synth.normal(n, count, seed=3, std=0.5)
    res = synth.normal(n, count, seed=4)
    xb = _bits(x)
    for name, algo in ALGOS.items():
        if name == "2pa_hb_2phase":
            with pytest.raises(msx.MsxError):
                _run_ex(msx, x, algo, residual=res)
            continue
        outs = _run_ex(msx, x, algo, residual=res)
        for r in range(n):
            assert np.array_equal(outs[r], orc.allreduce_residual_bf16(xb, _bits(res[r]))), (name, r)
    zero = torch.zeros(count, dtype=torch.bfloat16)
    for name, algo in ALGOS.items():
        assert np.array_equal(_run_ex(msx, x, algo, residual=zero)[5], orc.allreduce_bf16(xb)), name
        outs = _run_ex(msx, torch.zeros_like(x), algo, residual=res[0].clone())
        assert np.array_equal(outs[2], _bits(res[0])), name
    xf = synth.int_valued_f32(n, 1000, seed=5)
    rf = synth.int_valued_f32(1, 1000, seed=6)[0]
    for name, algo in ALGOS.items():
        outs = _run_ex(msx, xf, algo, residual=rf)
        assert np.array_equal(outs[7], orc.allreduce_residual_f32(xf.numpy(), rf.numpy())), name


# ---------------------------------------------------------------- robustness of the flag layer

def test_back_to_back_calls_with_scrambled_timing(msx, orc):
    # rotating LL scratch and ever-growing semaphores: 150 calls in a row, sizes and algorithms
    # interleaved, workgroups delayed pseudo-randomly; every call checked
    sizes = [512, 4096, 3000, 65536, 1 << 17, 24, 100_000]
    xs = [synth.normal(8, c, seed=100 + i) for i, c in enumerate(sizes)]
    wants = [_oracle(orc, x) for x in xs]
    dev = [[x[r].clone().cuda() for r in range(8)] for x in xs]
    outs = [[torch.empty_like(t) for t in d] for d in dev]
    order = list(ALGOS.values())
    for it in range(150):
        i = it % len(sizes)
        msx.set_option("chaos", str(1 + it))
        msx.allreduce_ex(dev[i], outs[i], None, algo=order[it % 4])
        if it % 10 == 9:
            msx.check_status()
            for j in range(len(sizes)):
                if it >= j:
                    for r in (0, 7):
                        assert np.array_equal(_bits(outs[j][r]), wants[j]), (it, j, r)
    msx.set_option("chaos", "0")
    msx.check_status()


def test_flag_epoch_wraparound(msx, orc):
    x = synth.normal(8, 2048, seed=9)
    want = _oracle(orc, x)
    msx.set_option("epoch", str(2 ** 32 - 2))
    for k in range(6):                                        # flags ...FFFE, ...FFFF, 1, 2, 3, 4
        for algo in (1, 2):
            assert np.array_equal(_run_ex(msx, x, algo)[3], want), (k, algo)
    assert int(msx.get_option("epoch")) < 100


def test_dead_rank_times_out_and_context_recovers(msx, orc):
    x = synth.normal(8, 4096, seed=10)
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "5")
    try:
        for algo in list(ALGOS.values()) + [5]:
            send = [x[r].clone().cuda() for r in range(8)]
            recv = [torch.empty_like(s) for s in send]
            msx.allreduce_ex(send, recv, None, algo=algo)
            rc, info = msx.status()
            assert rc == -4, (algo, info)
            msx.reset()
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    assert np.array_equal(_run_ex(msx, x, 2)[0], _oracle(orc, x))


def test_ll_request_larger_than_scratch_is_refused(msx):
    limit = int(msx.get_option("ll_max_bytes"))
    count = limit // 2 + 4096
    send = [torch.zeros(count, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, None, algo=2)
    assert e.value.code == -5
    with pytest.raises(msx.MsxError):
        msx.allreduce_ex(send, send, None, algo=1)


def test_calls_captured_in_a_hip_graph_replay_correctly(msx, orc):
    # flags, scratch rotation and expected semaphore values live in device memory, so a captured
    # sequence of calls can be replayed; inputs change between replays, eager calls run in between
    n, count = 8, 6000
    xs = [synth.normal(n, count, seed=200 + i) for i in range(4)]
    send = [xs[0][r].clone().cuda() for r in range(n)]
    outs = {a: [torch.zeros(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)] for a in ALGOS.values()}
    for a in ALGOS.values():                                  # warm-up outside the capture
        msx.allreduce_ex(send, outs[a], None, algo=a)
    msx.check_status()
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            for _ in range(3):
                for a in ALGOS.values():
                    msx.allreduce_ex(send, outs[a], None, algo=a)
    torch.cuda.synchronize()
    for i, x in enumerate(xs):
        for r in range(n):
            send[r].copy_(x[r])
        for a in ALGOS.values():
            for t in outs[a]:
                t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        msx.check_status()
        want = _oracle(orc, x)
        for a in ALGOS.values():
            for r in (0, 4, 7):
                assert np.array_equal(_bits(outs[a][r]), want), (i, a, r)
        # eager calls between replays share the same device-side call state
        assert np.array_equal(_run_ex(msx, x, 2)[1], want)
        assert np.array_equal(_run_ex(msx, x, 1)[6], want)


# ---------------------------------------------------------------- two-phase ring

@pytest.mark.parametrize("n", [2, 3, 5, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_ring_allreduce_matches_ring_order_oracle(msx, orc, n, dtype):
    esz = 4 if dtype == torch.float32 else 2
    for vecs_per_chunk in [1, 3, 64, 1000, 16385]:
        count = vecs_per_chunk * n * 16 // esz
        if dtype == torch.float32:
            g = torch.Generator().manual_seed(count)
            x = torch.randn(n, count, generator=g) * torch.exp(torch.randn(n, count, generator=g) * 3)
        else:
            x = synth.normal(n, count, seed=count)
        want = orc.allreduce_ring(_bits(x))
        msx.set_option("chaos", str(3 + vecs_per_chunk))
        for inplace in (False, True):
            outs = _run_ex(msx, x, 5, inplace=inplace)
            for r in range(n):
                assert np.array_equal(outs[r].view(np.uint8), want.view(np.uint8)), (n, count, r, inplace)
        msx.set_option("chaos", "0")
        # and within the any-order tolerance of the fp64 sum (bf16: 2e-2 relative plus the spacing at
        # the largest partial sum, which covers sums that nearly cancel)
        if dtype == torch.bfloat16:
            ref = np.sum(x.double().numpy(), axis=0)
            got = orc.bf16_to_f32(outs[0]).astype(np.float64)
            absmax = np.abs(x.double().numpy()).max(axis=0)
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(n * absmax, 2.0 ** -126))) - 7)
            assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + n * ulp)


@pytest.mark.parametrize("n", [2, 3, 5, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_overlapped_ring_over_the_port_channel_matches_ring_order_oracle(msx, orc, n, dtype):
    """MSX_ALGO_2PR_PORT: every hop is a put + signal (+ flush) request to the port (FIFO, CPU proxy, runtime
    copies), chunks travel in two halves and the reduction of one half overlaps the copy of the other.  The
    halves change when an element is added, not the order or the rounding: the bits are the plain ring's."""
    esz = 4 if dtype == torch.float32 else 2
    for vecs_per_chunk, blocks in [(1, 0), (3, 0), (64, 0), (1001, 3), (16385, 0), (70000, 5)]:
        count = vecs_per_chunk * n * 16 // esz
        if dtype == torch.float32:
            g = torch.Generator().manual_seed(count)
            x = torch.randn(n, count, generator=g) * torch.exp(torch.randn(n, count, generator=g) * 3)
        else:
            x = synth.normal(n, count, seed=count)
        want = orc.allreduce_ring(_bits(x))
        msx.set_option("hb_blocks_per_rank", str(blocks))
        msx.set_option("chaos", str(3 + vecs_per_chunk))
        try:
            for inplace in (False, True):
                outs = _run_ex(msx, x, 10, inplace=inplace)
                for r in range(n):
                    assert np.array_equal(outs[r].view(np.uint8), want.view(np.uint8)), (n, count, r, inplace)
            assert np.array_equal(_run_ex(msx, x, 5)[n - 1].view(np.uint8), want.view(np.uint8))   # the thread-copy ring between
        finally:
            msx.set_option("chaos", "0")
            msx.set_option("hb_blocks_per_rank", "0")


def test_port_ring_refuses_what_it_cannot_serve_and_times_out_without_a_rank(msx, orc):
    send = [torch.zeros(100, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, None, algo=10)
    assert e.value.code == -2
    send = [torch.zeros(1024, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, send, algo=10)
    assert e.value.code == -2
    with pytest.raises(msx.MsxError) as e:
        msx.prepare_allreduce(send, send, None, algo=10)        # the proxy is told of every launch
    assert e.value.code == -2
    x = synth.normal(8, 8192, seed=12)
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "3")
    try:
        s_ = [x[r].clone().cuda() for r in range(8)]
        r_ = [torch.empty_like(t) for t in s_]
        msx.allreduce_ex(s_, r_, None, algo=10)
        rc, info = msx.status()
        assert rc == -4, info
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    assert np.array_equal(_run_ex(msx, x, 10)[0], orc.allreduce_ring(_bits(x)))


def test_ring_allreduce_integers_equal_the_other_algorithms(msx, orc):
    x = synth.int_valued_f32(8, 262144, seed=0)                 # config 1: every order is exact
    want = orc.allreduce_f32(x.numpy())
    for o in _run_ex(msx, x, 5):
        assert np.array_equal(o, want)


def test_ring_allreduce_refuses_unsupported_requests(msx):
    send = [torch.zeros(100, dtype=torch.bfloat16, device="cuda") for _ in range(8)]     # 200 B: not 16*8-divisible
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, None, algo=5)
    assert e.value.code == -2
    send = [torch.zeros(1024, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    with pytest.raises(msx.MsxError) as e:
        msx.allreduce_ex(send, send, send, algo=5)
    assert e.value.code == -2


# ---------------------------------------------------------------- plan interpreter

@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_plan_interpreter_runs_the_same_algorithms(msx, orc, n, dtype):
    esz = 4 if dtype == torch.float32 else 2
    for vecs_per_chunk in [1, 5, 64, 1000, 16385, 70001]:
        count = vecs_per_chunk * n * 16 // esz
        x = synth.int_valued_f32(n, count, seed=count) if dtype == torch.float32 else synth.normal(n, count, seed=count)
        want_pairs = _oracle(orc, x)
        want_ring = orc.allreduce_ring(_bits(x))
        msx.set_option("chaos", str(1 + vecs_per_chunk))
        for inplace in (False, True):
            for r, o in enumerate(_run_ex(msx, x, 6, inplace=inplace)):
                assert np.array_equal(o.view(np.uint8), want_pairs.view(np.uint8)), ("pairs", n, count, r, inplace)
            for r, o in enumerate(_run_ex(msx, x, 7, inplace=inplace)):
                assert np.array_equal(o.view(np.uint8), want_ring.view(np.uint8)), ("ring", n, count, r, inplace)
        msx.set_option("chaos", "0")


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_plan_interpreter_runs_the_packet_algorithms(msx, orc, n, dtype):
    """1PA-LL and 2PA-LL from packet operations: bit-identical to the oracle (and so to the hand kernels),
    scrambled timing, ragged sizes down to a single element, in place and out of place."""
    esz = 4 if dtype == torch.float32 else 2
    for count in [1 if esz == 4 else 2, 6, 510, 4096, 4098, 20000 + 2 * n, 131072 + 26]:
        x = synth.int_valued_f32(n, count, seed=count) if dtype == torch.float32 else synth.normal(n, count, seed=count)
        want = _oracle(orc, x)
        msx.set_option("chaos", str(3 + count))
        for algo in (8, 9):
            if algo == 8 and count * esz > 32768:
                continue
            for inplace in (False, True):
                for r, o in enumerate(_run_ex(msx, x, algo, inplace=inplace)):
                    assert np.array_equal(o.view(np.uint8), want.view(np.uint8)), (algo, n, count, r, inplace)
        msx.set_option("chaos", "0")
    # many calls in a row: the flag epoch and the scratch rotation advance as for the hand kernels, which may
    # be mixed in freely
    x = synth.normal(n, 3000, seed=77) if dtype == torch.bfloat16 else synth.int_valued_f32(n, 3000, seed=77)
    want = _oracle(orc, x)
    for k in range(12):
        algo = (8, 9, 1, 2)[k % 4]
        assert np.array_equal(_run_ex(msx, x, algo)[n - 1].view(np.uint8), want.view(np.uint8)), (k, algo)


def test_plan_interpreter_runs_the_phased_schedule(phased, orc):
    """MSX_ALGO_PLAN_2PA_HB at sizes where the hand kernel runs in chip-wide phases: lowered to the same
    schedule (reduce and hold, chip-wide barrier, put what is held), several rounds, partial last rounds."""
    msx = phased
    n = 8
    for blocks, vecs_per_chunk in [(1, 256 * 64 * 2 + 256 * 5 + 77), (2, 256 * 64 * 2 * 2 + 256 * 64 + 1), (1, 255),
                                   (2, 256 * 64 * 2), (0, 256 * 70 + 9)]:
        count = vecs_per_chunk * n * 8
        msx.set_option("hb_blocks_per_rank", str(blocks))
        msx.set_option("chaos", str(blocks * 5 + 1))
        x = synth.normal(n, count, seed=vecs_per_chunk)
        want = _oracle(orc, x)
        for inplace in (False, True):
            outs = _run_ex(msx, x, 6, inplace=inplace)
            for r in range(n):
                assert np.array_equal(outs[r], want), (blocks, vecs_per_chunk, r, inplace)
        assert np.array_equal(_run_ex(msx, x, 3)[5], want)           # the hand kernel on the same launch shape


def test_plan_interpreter_argument_checks_and_dead_rank(msx, orc):
    send = [torch.zeros(100, dtype=torch.bfloat16, device="cuda") for _ in range(8)]
    for algo in (6, 7):
        with pytest.raises(msx.MsxError) as e:
            msx.allreduce_ex(send, send, None, algo=algo)
        assert e.value.code == -2
    x = synth.normal(8, 4096, seed=10)
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "2")
    try:
        for algo in (6, 7, 8, 9):
            s_ = [x[r].clone().cuda() for r in range(8)]
            r_ = [torch.empty_like(t) for t in s_]
            msx.allreduce_ex(s_, r_, None, algo=algo)
            rc, info = msx.status()
            assert rc == -4, (algo, info)
            msx.reset()
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    assert np.array_equal(_run_ex(msx, x, 6)[0], _oracle(orc, x))


# ---------------------------------------------------------------- fused HB in chip-wide read / write phases

@pytest.fixture
def phased(msx):
    """Forces the phased form of the fused HB kernel at any size (by default it starts at 40 MiB per rank, 8 ranks)."""
    old = msx.get_option("hb_phased_min_bytes")
    msx.set_option("hb_phased_min_bytes", "0")
    yield msx
    msx.set_option("hb_phased_min_bytes", old)
    msx.set_option("hb_blocks_per_rank", "0")
    msx.set_option("chaos", "0")


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_phased_fused_hb_matches_oracle_over_rounds_and_ragged_ends(phased, orc, n, dtype):
    msx = phased
    epv = 4 if dtype == torch.float32 else 8
    # workgroups per rank 1 / 2 / all: a round is (workgroups x 64) tiles of 256 vectors per chunk, so the small
    # launches run several rounds (the last one partial, some workgroups idle in it) at sizes the oracle likes
    for blocks, vecs_per_chunk in [(1, 256 * 64 * 3 + 256 * 5 + 77), (2, 256 * 64 * 2 * 2 + 256 * 64 + 1),
                                   (1, 255), (1, 256), (2, 256 * 64 * 2), (0, 256 * 70 + 9), (0, 3)]:
        count = vecs_per_chunk * n * epv + (3 if vecs_per_chunk % 2 else 0)        # sometimes a few odd elements
        msx.set_option("hb_blocks_per_rank", str(blocks))
        msx.set_option("chaos", str(blocks * 7 + n))
        x = synth.normal(n, count, seed=300 + n + blocks, dtype=dtype)
        want = _oracle(orc, x)
        for inplace in (False, True):
            got = _run_ex(msx, x, 3, inplace=inplace)
            grid = msx.last_launch()[0]                          # the phased launch: what was asked for, else one workgroup per CU
            assert grid == n * blocks if blocks else (grid % n == 0 and 200 <= grid <= 256), (grid, n, blocks)
            for r in range(n):
                assert np.array_equal(got[r], want), (n, dtype, blocks, vecs_per_chunk, inplace, r)


def test_phased_fused_hb_with_shared_residual_and_back_to_back_calls(phased, orc):
    msx = phased
    n, count = 8, 8 * (256 * 64 * 2 + 300) * 8
    msx.set_option("hb_blocks_per_rank", "1")
    x = synth.normal(n, count, seed=310)
    res = synth.normal(1, count, seed=311)[0]
    want = orc.allreduce_residual_bf16(_bits(x), _bits(res))
    got = _run_ex(msx, x, 3, residual=res)
    for r in range(n):
        assert np.array_equal(got[r], want), r
    # the barrier counters carry over from call to call, also across other kernels and launch shapes
    plain = _oracle(orc, x)
    for i, blocks in enumerate([1, 3, 0, 2, 0, 1]):
        msx.set_option("hb_blocks_per_rank", str(blocks))
        msx.set_option("chaos", str(i))
        assert np.array_equal(_run_ex(msx, x, 3)[i % n], plain), (i, blocks)
        small = synth.normal(n, 512, seed=320 + i)
        assert np.array_equal(_run_ex(msx, small, 1)[0], _oracle(orc, small))        # a packet call in between
    # per-rank residuals are not phased: the ordinary fused kernel serves them
    per_rank = synth.normal(n, count, seed=312)
    got = _run_ex(msx, x, 3, residual=per_rank)
    for r in (0, 5):
        assert np.array_equal(got[r], orc.allreduce_residual_bf16(_bits(x), _bits(per_rank[r]))), r


def test_phased_fused_hb_replays_in_a_hip_graph(phased, orc):
    msx = phased
    n, count = 8, 8 * (256 * 64 * 3 + 40) * 8                     # three rounds with one workgroup per rank: paced
    msx.set_option("hb_blocks_per_rank", "1")
    xs = [synth.normal(n, count, seed=330 + i) for i in range(3)]
    send = [xs[0][r].clone().cuda() for r in range(n)]
    out = [torch.zeros(count, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.allreduce_ex(send, out, None, algo=3)
    msx.check_status()
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            for _ in range(3):
                msx.allreduce_ex(send, out, None, algo=3)
    torch.cuda.synchronize()
    for i, x in enumerate(xs):
        for r in range(n):
            send[r].copy_(x[r])
            out[r].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        msx.check_status()
        want = _oracle(orc, x)
        for r in (0, 3, 7):
            assert np.array_equal(_bits(out[r]), want), (i, r)
        assert np.array_equal(_run_ex(msx, x, 3)[2], want)        # an eager call between the replays


def test_phased_fused_hb_dead_rank_times_out_and_context_recovers(phased, orc):
    msx = phased
    x = synth.normal(8, 8 * (256 * 64 + 5) * 8, seed=340)
    msx.set_option("hb_blocks_per_rank", "1")
    msx.set_option("spin_limit", "2000")
    msx.set_option("drop_rank", "5")
    try:
        send = [x[r].clone().cuda() for r in range(8)]
        recv = [torch.empty_like(s) for s in send]
        msx.allreduce_ex(send, recv, None, algo=3)
        rc, info = msx.status()
        assert rc == -4, info
    finally:
        msx.set_option("drop_rank", "-1")
        msx.set_option("spin_limit", str(1 << 20))
        msx.reset()
    assert np.array_equal(_run_ex(msx, x, 3)[0], _oracle(orc, x))


def test_phased_fused_hb_survives_barrier_counter_wraparound(phased, orc):
    """The chip-wide barrier's counters only grow; here they start three short of 2^32, so the very first
    barrier of the first call wraps them (signed distances decide), and later calls continue from there."""
    msx = phased
    n, count = 8, 8 * (256 * 64 * 3 + 40) * 8
    msx.set_option("hb_blocks_per_rank", "1")
    msx.set_option("sem_base", str(2 ** 32 - 3))
    try:
        for i in range(3):
            x = synth.normal(n, count, seed=350 + i)
            got = _run_ex(msx, x, 3)
            assert np.array_equal(got[i], _oracle(orc, x)), i
    finally:
        msx.reset()


def test_paced_shapes_that_share_a_schedule_slot_evict_each_other_harmlessly(phased, orc):
    """The learnt schedules live in 31 direct-mapped slots tagged with the launch's shape.  34 shapes taken in
    turn, twice over, must collide (pigeonhole): a shape that finds another one's entry starts from scratch, and
    no schedule learnt for one shape may hold back, or corrupt, a launch of another."""
    msx = phased
    n = 8
    msx.set_option("hb_blocks_per_rank", "1")
    shapes = []
    for k in range(34):
        count = 8 * (256 * 64 * 3 + 9 * k + 1) * 8                  # 3 rounds and a ragged end with one workgroup per rank
        x = synth.normal(n, count, seed=400 + k)
        shapes.append((x, _oracle(orc, x)))
    for sweep in range(2):
        for k, (x, want) in enumerate(shapes):
            got = _run_ex(msx, x, 3)
            for r in (0, 3, 7):
                assert np.array_equal(got[r], want), (sweep, k, r)
    msx.check_status()


def test_phased_fused_hb_with_paced_write_phases(phased, orc):
    """Launches of two rounds or more hold their write phases to a wall-clock schedule derived from the rounds
    before; one workgroup per rank makes 13 rounds out of 27 MiB per rank.  Pacing must not change a bit."""
    msx = phased
    n, count = 8, 8 * (256 * 64 * 13 + 77) * 8
    msx.set_option("hb_blocks_per_rank", "1")
    x = synth.normal(n, count, seed=360)
    want = _oracle(orc, x)
    # six calls of one shape in a row: the schedule is learnt, tightened, missed, frozen, and carried from call
    # to call (it lives beside the barrier counters); then once without pacing
    for pace in ("1", "1", "1", "1", "1", "1", "0"):
        msx.set_option("hb_pace", pace)
        try:
            got = _run_ex(msx, x, 3)
        finally:
            msx.set_option("hb_pace", "1")
        for r in (0, 7):
            assert np.array_equal(got[r], want), (pace, r)
    # the all-gather paces the same way
    blk = (256 * 64 * 13 + 5) * 8
    y = synth.normal(n, blk, seed=361)
    out = [torch.zeros(n * blk, dtype=torch.bfloat16, device="cuda") for _ in range(n)]
    msx.allgather_ex([y[r].clone().cuda() for r in range(n)], out)
    msx.check_status()
    want_ag = orc.allgather(_bits(y))
    for r in (0, 5):
        assert np.array_equal(_bits(out[r]), want_ag[r]), r
