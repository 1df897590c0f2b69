"""ctypes binding of libmsx.so.  Same names as the C entry points, minus the msx_ prefix.

Tensors are torch CUDA tensors (device memory and streams are torch's job); this module
only extracts pointers, sizes and the current stream and checks return codes.
"""
import ctypes as C
import os

import torch

__all__ = [
    "F32", "BF16", "F16", "I32", "SUM", "MAX", "MIN", "ALGO_AUTO", "ALGO_1PA_LL", "ALGO_2PA_LL", "ALGO_2PA_HB", "ALGO_2PA_HB_2PHASE", "ALGO_2PR_HB", "ALGO_PLAN_2PA_HB", "ALGO_PLAN_2PR_HB", "ALGO_PLAN_1PA_LL", "ALGO_PLAN_2PA_LL", "ALGO_2PR_PORT",
    "MsxError", "lib", "lib_path", "init", "reset", "finalize", "set_option", "get_option", "status",
    "check_status", "last_launch", "version", "strerror",
    "allreduce", "reducescatter", "allgather", "alltoall",
    "allreduce_ex", "allreduce_ex_static", "reducescatter_ex", "allgather_ex", "alltoall_ex", "moe_dispatch", "moe_dispatch_fp8", "moe_combine",
    "ctx_create", "ctx_destroy", "ctx_reset", "ctx_use", "ctx_set_max_blocks", "last_status",
    "moe_plan_create", "moe_plan_destroy",
    "prepare_allreduce", "prepare_reducescatter", "prepare_allgather", "prepare_alltoall",
    "prepare_moe_dispatch", "prepare_moe_combine", "run", "release", "Prepared",
    "prim_pingpong", "prim_barrier", "prim_put_signal_wait", "prim_ll_encode", "prim_ll_roundtrip", "prim_port_put_signal_wait", "prim_stream",
    "EXPORTS",
]

F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, MAX, MIN = 0, 1, 2
ALGO_AUTO, ALGO_1PA_LL, ALGO_2PA_LL, ALGO_2PA_HB, ALGO_2PA_HB_2PHASE, ALGO_2PR_HB = 0, 1, 2, 3, 4, 5
ALGO_PLAN_2PA_HB, ALGO_PLAN_2PR_HB, ALGO_PLAN_1PA_LL, ALGO_PLAN_2PA_LL = 6, 7, 8, 9
ALGO_2PR_PORT = 10

EXPORTS = [
    "msx_allreduce", "msx_reducescatter", "msx_allgather", "msx_alltoall",
    "msx_allreduce_ex", "msx_allreduce_ex_static", "msx_reducescatter_ex", "msx_allgather_ex", "msx_alltoall_ex",
    "msx_moe_dispatch", "msx_moe_dispatch_fp8", "msx_moe_combine", "msx_moe_plan_create", "msx_moe_plan_destroy",
    "msx_prepare_allreduce", "msx_prepare_reducescatter", "msx_prepare_allgather", "msx_prepare_alltoall",
    "msx_prepare_moe_dispatch", "msx_prepare_moe_combine", "msx_run", "msx_release",
    "msx_ctx_create", "msx_ctx_destroy", "msx_ctx_reset", "msx_ctx_use", "msx_ctx_set_max_blocks", "msx_last_status",
    "msx_prim_pingpong", "msx_prim_barrier", "msx_prim_put_signal_wait", "msx_prim_ll_encode",
    "msx_prim_ll_roundtrip", "msx_prim_port_put_signal_wait", "msx_prim_stream",
    "msx_init", "msx_reset", "msx_finalize", "msx_set_option", "msx_get_option", "msx_status",
    "msx_last_launch", "msx_last_hip_error", "msx_strerror", "msx_version",
    "msx_debug_choose", "msx_debug_lower_plan", "msx_debug_lower_plan_ex", "msx_debug_pace_update", "msx_debug_owner_magic",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class MsxError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = lib().msx_strerror(code).decode()
        extra = f" (hip error {lib().msx_last_hip_error()})" if code == -3 else ""
        super().__init__(f"{where}: {msg} [{code}]{extra}")


def lib_path():
    return os.path.join(_HERE, "libmsx.so")


def lib():
    """Load libmsx.so (built in-tree by build.py).  Fails loudly when it is missing."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no fallback path)")
        L = C.CDLL(path)
        vp, sz, i, u32 = C.c_void_p, C.c_size_t, C.c_int, C.c_uint32
        pp = C.POINTER(C.c_void_p)
        for name in ("msx_allreduce", "msx_reducescatter", "msx_allgather", "msx_alltoall"):
            getattr(L, name).argtypes = [vp, sz, i, i, i, vp]
        L.msx_allreduce_ex.argtypes = [pp, pp, pp, sz, i, i, i, i, vp]
        L.msx_allreduce_ex_static.argtypes = [pp, pp, pp, sz, i, i, i, i, vp]
        L.msx_reducescatter_ex.argtypes = [pp, pp, sz, i, i, i, vp]
        L.msx_allgather_ex.argtypes = [pp, pp, sz, i, i, vp]
        L.msx_alltoall_ex.argtypes = [pp, pp, sz, i, i, vp]
        L.msx_moe_dispatch.argtypes = [pp, pp, i, i, i, i, i, i, pp, pp, vp, sz, vp, vp]
        L.msx_moe_dispatch_fp8.argtypes = [pp, pp, i, i, i, i, i, pp, pp, pp, vp, sz, vp, vp]
        L.msx_moe_combine.argtypes = [pp, pp, i, i, i, i, sz, vp, vp]
        L.msx_moe_plan_create.argtypes = [vp, i, pp]
        L.msx_moe_plan_destroy.argtypes = [vp]
        L.msx_prepare_allreduce.argtypes = [pp, pp, pp, sz, i, i, i, i, pp]
        L.msx_prepare_reducescatter.argtypes = [pp, pp, sz, i, i, i, pp]
        L.msx_prepare_allgather.argtypes = [pp, pp, sz, i, i, pp]
        L.msx_prepare_alltoall.argtypes = [pp, pp, sz, i, i, pp]
        L.msx_prepare_moe_dispatch.argtypes = [pp, pp, i, i, i, i, i, i, pp, pp, vp, sz, vp, pp]
        L.msx_prepare_moe_combine.argtypes = [pp, pp, i, i, i, i, sz, vp, pp]
        L.msx_run.argtypes = [vp, vp]
        L.msx_release.argtypes = [vp]
        L.msx_ctx_create.argtypes = [i, sz, pp]
        L.msx_ctx_destroy.argtypes = [vp]
        L.msx_ctx_reset.argtypes = [vp]
        L.msx_ctx_use.argtypes = [vp]
        L.msx_ctx_set_max_blocks.argtypes = [vp, i]
        L.msx_last_status.argtypes = [vp, C.POINTER(i), C.POINTER(i), C.POINTER(u32), C.POINTER(u32)]
        L.msx_prim_pingpong.argtypes = [i, i, i, i, vp, vp]
        L.msx_prim_barrier.argtypes = [i, i, i, vp, vp]
        L.msx_prim_put_signal_wait.argtypes = [vp, vp, vp, sz, i, vp]
        L.msx_prim_port_put_signal_wait.argtypes = [vp, vp, vp, sz, vp]
        L.msx_prim_ll_encode.argtypes = [vp, sz, u32, vp, vp]
        L.msx_prim_ll_roundtrip.argtypes = [vp, vp, sz, i, vp]
        L.msx_prim_stream.argtypes = [i, vp, vp, sz, i, vp]
        L.msx_set_option.argtypes = [C.c_char_p, C.c_char_p]
        L.msx_get_option.argtypes = [C.c_char_p, C.c_char_p, sz]
        L.msx_status.argtypes = [vp, C.POINTER(u32)]
        L.msx_last_launch.argtypes = [C.POINTER(i), C.POINTER(i), C.POINTER(i)]
        L.msx_debug_choose.argtypes = [sz, i, sz, C.POINTER(i), C.POINTER(i), C.POINTER(i)]
        L.msx_debug_lower_plan.argtypes = [i, i, i, sz, i, vp, sz, C.POINTER(u32), C.POINTER(sz)]
        L.msx_debug_lower_plan_ex.argtypes = [i, i, i, sz, i, i, vp, sz, C.POINTER(u32), C.POINTER(sz)]
        L.msx_debug_pace_update.argtypes = [C.POINTER(u32), C.c_uint64, u32]
        L.msx_debug_owner_magic.argtypes = [i, i, C.POINTER(u32)]
        L.msx_strerror.argtypes = [i]
        L.msx_strerror.restype = C.c_char_p
        L.msx_version.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("msx_strerror", "msx_version"):
                getattr(L, name).restype = i
        _lib = L
    return _lib


def _ck(rc, where):
    if rc != 0:
        raise MsxError(rc, where)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dtype(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.int32:
        return I32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, what):
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _table(tensors):
    if tensors is None:
        return None
    arr = (C.c_void_p * len(tensors))()
    for k, t in enumerate(tensors):
        arr[k] = t.data_ptr()
    return C.cast(arr, C.POINTER(C.c_void_p))


def version():
    return lib().msx_version().decode()


def strerror(code):
    return lib().msx_strerror(code).decode()


def init():
    _ck(lib().msx_init(), "msx_init")


def reset():
    _ck(lib().msx_reset(), "msx_reset")


def finalize():
    _ck(lib().msx_finalize(), "msx_finalize")


def set_option(key, value):
    _ck(lib().msx_set_option(str(key).encode(), str(value).encode()), f"msx_set_option({key}={value})")


def get_option(key):
    buf = C.create_string_buffer(64)
    _ck(lib().msx_get_option(str(key).encode(), buf, 64), f"msx_get_option({key})")
    return buf.value.decode()


def status(stream=None):
    """Synchronise the stream; return (code, info) with info = (code, rank, site, expected, seen, block)."""
    info = (C.c_uint32 * 6)()
    rc = lib().msx_status(_stream(stream), info)
    return rc, tuple(int(v) for v in info)


def check_status(stream=None):
    rc, info = status(stream)
    if rc != 0:
        raise MsxError(rc, f"device status {info}")


def last_launch():
    g, b, a = C.c_int(0), C.c_int(0), C.c_int(0)
    lib().msx_last_launch(C.byref(g), C.byref(b), C.byref(a))
    return g.value, b.value, a.value


# ---- in-place forms: buf is a [nranks, ...] tensor -------------------------------------------

def _inplace(fn, name, buf, count, nranks, stream, op=SUM):
    _dev(buf, "buf")
    _ck(fn(C.c_void_p(buf.data_ptr()), count, _dtype(buf), op, nranks, _stream(stream)), name)


def allreduce(buf, stream=None, op=SUM):
    """buf: [nranks, count]; every row becomes the sum (max, min) of the rows."""
    _inplace(lib().msx_allreduce, "msx_allreduce", buf, buf.shape[1], buf.shape[0], stream, op)


def reducescatter(buf, stream=None, op=SUM):
    """buf: [nranks, count]; row r's share r becomes the sum (max, min) over rows of that share."""
    _inplace(lib().msx_reducescatter, "msx_reducescatter", buf, buf.shape[1], buf.shape[0], stream, op)


def allgather(buf, stream=None):
    """buf: [nranks, nranks*count]; row r's slot r is broadcast into slot r of every row."""
    n = buf.shape[0]
    if buf.shape[1] % n:
        raise ValueError("row length must be nranks*count")
    _inplace(lib().msx_allgather, "msx_allgather", buf, buf.shape[1] // n, n, stream)


def alltoall(buf, stream=None):
    """buf: [nranks, count]; block s of row d <- block d of row s."""
    _inplace(lib().msx_alltoall, "msx_alltoall", buf, buf.shape[1], buf.shape[0], stream)


# ---- per-rank pointer forms ---------------------------------------------------------------------

def allreduce_ex(send, recv, residual=None, algo=ALGO_AUTO, stream=None, count=None, op=SUM):
    """send, recv (, residual): lists of nranks 1-D device tensors of equal length."""
    n = len(send)
    for t in list(send) + list(recv) + list(residual or []):
        _dev(t, "tensor")
    cnt = send[0].numel() if count is None else count
    _ck(lib().msx_allreduce_ex(_table(send), _table(recv), _table(residual), cnt, _dtype(send[0]), op, n,
                               algo, _stream(stream)), "msx_allreduce_ex")


def allreduce_ex_static(send, recv, residual=None, algo=ALGO_AUTO, stream=None, count=None, op=SUM):
    """allreduce_ex on the library's fixed scratch array: the call allocates nothing."""
    n = len(send)
    for t in list(send) + list(recv) + list(residual or []):
        _dev(t, "tensor")
    cnt = send[0].numel() if count is None else count
    _ck(lib().msx_allreduce_ex_static(_table(send), _table(recv), _table(residual), cnt, _dtype(send[0]), op, n,
                                      algo, _stream(stream)), "msx_allreduce_ex_static")


def reducescatter_ex(send, recv, stream=None, op=SUM):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    _ck(lib().msx_reducescatter_ex(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), op, n,
                                   _stream(stream)), "msx_reducescatter_ex")


def allgather_ex(send, recv, stream=None):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    _ck(lib().msx_allgather_ex(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), n,
                               _stream(stream)), "msx_allgather_ex")


def alltoall_ex(send, recv, stream=None):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    _ck(lib().msx_alltoall_ex(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), n,
                              _stream(stream)), "msx_alltoall_ex")


def moe_dispatch(tokens, topk_idx, n_experts, recv_tokens, recv_counts, recv_src_token=None, stream=None, plan=None):
    """tokens[s]: [T, H]; topk_idx[s]: [T, K] int32; recv_tokens[d]: [cap, H];
    recv_counts: [nranks, nranks] int32; recv_src_token[d]: [cap] int32 (optional)."""
    n = len(tokens)
    T, H = tokens[0].shape
    K = topk_idx[0].shape[1]
    cap = recv_tokens[0].shape[0]
    for t in list(tokens) + list(topk_idx) + list(recv_tokens) + list(recv_src_token or []) + [recv_counts]:
        _dev(t, "tensor")
    if any(t.dtype != torch.int32 for t in topk_idx) or recv_counts.dtype != torch.int32:
        raise TypeError("topk_idx and recv_counts must be int32")
    _ck(lib().msx_moe_dispatch(_table(tokens), _table(topk_idx), T, H, K, n_experts, _dtype(tokens[0]), n,
                               _table(recv_tokens), _table(recv_src_token), C.c_void_p(recv_counts.data_ptr()),
                               cap, plan, _stream(stream)), "msx_moe_dispatch")


def moe_dispatch_fp8(tokens, topk_idx, n_experts, recv_q, recv_scales, recv_counts, recv_src_token=None,
                     stream=None, plan=None):
    """tokens[s]: [T, H] bf16; recv_q[d]: [cap, H] uint8; recv_scales[d]: [cap, H/128] float32."""
    n = len(tokens)
    T, H = tokens[0].shape
    K = topk_idx[0].shape[1]
    cap = recv_q[0].shape[0]
    for t in (list(tokens) + list(topk_idx) + list(recv_q) + list(recv_scales) + list(recv_src_token or [])
              + [recv_counts]):
        _dev(t, "tensor")
    if tokens[0].dtype != torch.bfloat16 or recv_q[0].dtype != torch.uint8 or recv_scales[0].dtype != torch.float32:
        raise TypeError("tokens bf16, recv_q uint8, recv_scales float32")
    _ck(lib().msx_moe_dispatch_fp8(_table(tokens), _table(topk_idx), T, H, K, n_experts, n, _table(recv_q),
                                   _table(recv_scales), _table(recv_src_token),
                                   C.c_void_p(recv_counts.data_ptr()), cap, plan, _stream(stream)),
        "msx_moe_dispatch_fp8")


def moe_combine(expert_out, out_tokens, stream=None, plan=None):
    """expert_out[d]: [cap, H] processed rows in dispatch order; out_tokens[s]: [T, H].
    Uses the routing the last moe_dispatch through `plan` left there (None: the built-in plan)."""
    n = len(expert_out)
    cap, H = expert_out[0].shape
    T = out_tokens[0].shape[0]
    for t in list(expert_out) + list(out_tokens):
        _dev(t, "tensor")
    _ck(lib().msx_moe_combine(_table(expert_out), _table(out_tokens), T, H, _dtype(expert_out[0]), n, cap,
                              plan, _stream(stream)), "msx_moe_combine")


# ---- contexts, routing plans, prepared calls --------------------------------------------------------

def ctx_create(nranks=8, max_ll_bytes=0):
    h = C.c_void_p()
    _ck(lib().msx_ctx_create(nranks, max_ll_bytes, C.byref(h)), "msx_ctx_create")
    return h


def ctx_destroy(ctx):
    _ck(lib().msx_ctx_destroy(ctx), "msx_ctx_destroy")


def ctx_reset(ctx=None):
    _ck(lib().msx_ctx_reset(ctx), "msx_ctx_reset")


def ctx_use(ctx=None):
    _ck(lib().msx_ctx_use(ctx), "msx_ctx_use")


def ctx_set_max_blocks(ctx, max_blocks):
    _ck(lib().msx_ctx_set_max_blocks(ctx, max_blocks), "msx_ctx_set_max_blocks")


def last_status(ctx=None):
    """(code, rank, site, expected, seen) of ctx, read and cleared without waiting for the device."""
    r, s_, e, v = C.c_int(0), C.c_int(0), C.c_uint32(0), C.c_uint32(0)
    rc = lib().msx_last_status(ctx, C.byref(r), C.byref(s_), C.byref(e), C.byref(v))
    return rc, r.value, s_.value, e.value, v.value


def moe_plan_create(max_tokens_per_rank, ctx=None):
    h = C.c_void_p()
    _ck(lib().msx_moe_plan_create(ctx, max_tokens_per_rank, C.byref(h)), "msx_moe_plan_create")
    return h


def moe_plan_destroy(plan):
    _ck(lib().msx_moe_plan_destroy(plan), "msx_moe_plan_destroy")


class Prepared:
    """A prepared call: `run()` only enqueues its kernels.  Keeps the tensors alive."""

    def __init__(self, handle, keep):
        self.handle = handle
        self._keep = keep
        self._run = lib().msx_run

    def run(self, stream=None):
        rc = self._run(self.handle, _stream(stream) if stream is None or hasattr(stream, "cuda_stream") else stream)
        if rc != 0:
            raise MsxError(rc, "msx_run")

    def release(self):
        if self.handle is not None:
            _ck(lib().msx_release(self.handle), "msx_release")
            self.handle = None


def run(prepared, stream=None):
    prepared.run(stream)


def release(prepared):
    prepared.release()


def prepare_allreduce(send, recv, residual=None, algo=ALGO_AUTO, count=None, op=SUM):
    n = len(send)
    for t in list(send) + list(recv) + list(residual or []):
        _dev(t, "tensor")
    cnt = send[0].numel() if count is None else count
    h = C.c_void_p()
    _ck(lib().msx_prepare_allreduce(_table(send), _table(recv), _table(residual), cnt, _dtype(send[0]), op, n,
                                    algo, C.byref(h)), "msx_prepare_allreduce")
    return Prepared(h, (list(send), list(recv), list(residual or [])))


def prepare_reducescatter(send, recv, op=SUM):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    h = C.c_void_p()
    _ck(lib().msx_prepare_reducescatter(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), op, n,
                                        C.byref(h)), "msx_prepare_reducescatter")
    return Prepared(h, (list(send), list(recv)))


def prepare_allgather(send, recv):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    h = C.c_void_p()
    _ck(lib().msx_prepare_allgather(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), n, C.byref(h)),
        "msx_prepare_allgather")
    return Prepared(h, (list(send), list(recv)))


def prepare_alltoall(send, recv):
    n = len(send)
    for t in list(send) + list(recv):
        _dev(t, "tensor")
    h = C.c_void_p()
    _ck(lib().msx_prepare_alltoall(_table(send), _table(recv), send[0].numel(), _dtype(send[0]), n, C.byref(h)),
        "msx_prepare_alltoall")
    return Prepared(h, (list(send), list(recv)))


def prepare_moe_dispatch(tokens, topk_idx, n_experts, recv_tokens, recv_counts, plan, recv_src_token=None):
    n = len(tokens)
    T, H = tokens[0].shape
    K = topk_idx[0].shape[1]
    cap = recv_tokens[0].shape[0]
    for t in list(tokens) + list(topk_idx) + list(recv_tokens) + list(recv_src_token or []) + [recv_counts]:
        _dev(t, "tensor")
    h = C.c_void_p()
    _ck(lib().msx_prepare_moe_dispatch(_table(tokens), _table(topk_idx), T, H, K, n_experts, _dtype(tokens[0]), n,
                                       _table(recv_tokens), _table(recv_src_token),
                                       C.c_void_p(recv_counts.data_ptr()), cap, plan, C.byref(h)),
        "msx_prepare_moe_dispatch")
    return Prepared(h, (list(tokens), list(topk_idx), list(recv_tokens), list(recv_src_token or []), recv_counts))


def prepare_moe_combine(expert_out, out_tokens, plan):
    n = len(expert_out)
    cap, H = expert_out[0].shape
    T = out_tokens[0].shape[0]
    for t in list(expert_out) + list(out_tokens):
        _dev(t, "tensor")
    h = C.c_void_p()
    _ck(lib().msx_prepare_moe_combine(_table(expert_out), _table(out_tokens), T, H, _dtype(expert_out[0]), n, cap,
                                      plan, C.byref(h)), "msx_prepare_moe_combine")
    return Prepared(h, (list(expert_out), list(out_tokens)))


# ---- primitives ------------------------------------------------------------------------------------

def prim_pingpong(iters, grid_blocks, block_a, block_b, stream=None):
    """ns per signal/wait round trip between two workgroups (synchronises)."""
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    _ck(lib().msx_prim_pingpong(iters, grid_blocks, block_a, block_b, C.c_void_p(out.data_ptr()),
                                _stream(stream)), "msx_prim_pingpong")
    check_status(stream)
    return float(out.item())


def prim_barrier(rounds, nranks, blocks_per_rank, stream=None):
    """Run `rounds` rank barriers; returns channel-0 semaphore values [nranks, nranks] (synchronises)."""
    out = torch.zeros((nranks, nranks), dtype=torch.int32, device="cuda")
    _ck(lib().msx_prim_barrier(rounds, nranks, blocks_per_rank, C.c_void_p(out.data_ptr()), _stream(stream)),
        "msx_prim_barrier")
    check_status(stream)
    return out.cpu().numpy().astype("uint32")


def prim_put_signal_wait(src, staging, dst, blocks_per_rank=4, stream=None):
    nbytes = src.numel() * src.element_size()
    _ck(lib().msx_prim_put_signal_wait(C.c_void_p(src.data_ptr()), C.c_void_p(staging.data_ptr()),
                                       C.c_void_p(dst.data_ptr()), nbytes, blocks_per_rank, _stream(stream)),
        "msx_prim_put_signal_wait")


def prim_port_put_signal_wait(src, staging, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    _ck(lib().msx_prim_port_put_signal_wait(C.c_void_p(src.data_ptr()), C.c_void_p(staging.data_ptr()),
                                            C.c_void_p(dst.data_ptr()), nbytes, _stream(stream)),
        "msx_prim_port_put_signal_wait")


def prim_ll_encode(src, flag, stream=None):
    """src: uint8 device tensor -> uint8 device tensor of 16-byte packets."""
    nbytes = src.numel() * src.element_size()
    out = torch.zeros(16 * ((nbytes + 7) // 8), dtype=torch.uint8, device=src.device)
    _ck(lib().msx_prim_ll_encode(C.c_void_p(src.data_ptr()), nbytes, flag & 0xFFFFFFFF,
                                 C.c_void_p(out.data_ptr()), _stream(stream)), "msx_prim_ll_encode")
    return out


def prim_ll_roundtrip(src, dst, blocks_per_rank=1, stream=None):
    nbytes = src.numel() * src.element_size()
    _ck(lib().msx_prim_ll_roundtrip(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), nbytes,
                                    blocks_per_rank, _stream(stream)), "msx_prim_ll_roundtrip")


def prim_stream(mode, src, dst, blocks=2048, stream=None):
    """mode 0: read src, 1: write dst, 2: copy src -> dst (the unused tensor may be None)."""
    t = src if src is not None else dst
    nbytes = t.numel() * t.element_size()
    _ck(lib().msx_prim_stream(mode, C.c_void_p(src.data_ptr()) if src is not None else None,
                              C.c_void_p(dst.data_ptr()) if dst is not None else None, nbytes, blocks,
                              _stream(stream)), "msx_prim_stream")
