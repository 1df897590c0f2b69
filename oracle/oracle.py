"""ctypes front-end of the C oracle.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this module; only the tests, the smoke check and
the benchmark's CPU-baseline leg do.  Arrays are numpy, rank-major and contiguous.  bf16
values travel as uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        vp, sz, i32, u32, u64 = C.c_void_p, C.c_size_t, C.c_int, C.c_uint32, C.c_uint64
        L.orc_bf16_to_f32.restype = C.c_float
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [C.c_float]
        L.orc_bf16_to_f32_buf.argtypes = [vp, vp, sz]
        L.orc_bf16_to_f32_buf.restype = None
        L.orc_f32_to_bf16_buf.argtypes = [vp, vp, sz]
        L.orc_f32_to_bf16_buf.restype = None
        L.orc_allreduce_f32.argtypes = [vp, vp, i32, sz]
        L.orc_allreduce_f32.restype = None
        L.orc_allreduce_f32_as_i64.argtypes = [vp, vp, i32, sz]
        L.orc_allreduce_f32_as_i64.restype = i32
        L.orc_allreduce_bf16.argtypes = [vp, vp, vp, i32, sz]
        L.orc_allreduce_bf16.restype = None
        L.orc_allreduce_residual_bf16.argtypes = [vp, vp, vp, vp, i32, sz]
        L.orc_allreduce_residual_bf16.restype = None
        L.orc_allreduce_residual_f32.argtypes = [vp, vp, vp, i32, sz]
        L.orc_allreduce_residual_f32.restype = None
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        L.orc_f16_to_f32.restype = C.c_float
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_allreduce_any.argtypes = [vp, vp, i32, sz, i32, i32]
        L.orc_allreduce_any.restype = None
        L.orc_allreduce_ring_bf16.argtypes = [vp, vp, i32, sz]
        L.orc_allreduce_ring_bf16.restype = None
        L.orc_allreduce_ring_f32.argtypes = [vp, vp, i32, sz]
        L.orc_allreduce_ring_f32.restype = None
        L.orc_reducescatter_f32.argtypes = [vp, vp, i32, sz]
        L.orc_reducescatter_f32.restype = None
        L.orc_reducescatter_bf16.argtypes = [vp, vp, i32, sz]
        L.orc_reducescatter_bf16.restype = None
        L.orc_allgather.argtypes = [vp, vp, i32, sz]
        L.orc_allgather.restype = None
        L.orc_alltoall.argtypes = [vp, vp, i32, sz]
        L.orc_alltoall.restype = None
        L.orc_ll_encode.argtypes = [u32, u32]
        L.orc_ll_encode.restype = u64
        L.orc_ll_decode.argtypes = [u64, u32, C.POINTER(u32)]
        L.orc_ll_decode.restype = i32
        L.orc_ll_encode_buf.argtypes = [vp, sz, u32, vp]
        L.orc_ll_encode_buf.restype = sz
        L.orc_ll_decode_buf.argtypes = [vp, sz, u32, vp]
        L.orc_ll_decode_buf.restype = i32
        L.orc_moe_dispatch.argtypes = [vp, vp, i32, i32, i32, i32, sz, vp, vp, vp, sz]
        L.orc_moe_dispatch.restype = i32
        L.orc_e4m3_to_f32.argtypes = [C.c_uint8]
        L.orc_e4m3_to_f32.restype = C.c_float
        L.orc_f32_to_e4m3.argtypes = [C.c_float]
        L.orc_f32_to_e4m3.restype = C.c_uint8
        L.orc_fp8_quantize_rows.argtypes = [vp, vp, vp, sz, sz]
        L.orc_fp8_quantize_rows.restype = None
        L.orc_moe_combine_bf16.argtypes = [vp, vp, i32, i32, i32, i32, sz, sz, vp, vp, vp]
        L.orc_moe_combine_bf16.restype = i32
        L.orc_sem_reached.argtypes = [u32, u32]
        L.orc_sem_reached.restype = i32
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def bf16_to_f32(bits):
    """uint16 array of bf16 patterns -> float32 array (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, np.float32)
    lib().orc_bf16_to_f32_buf(_p(bits), _p(out), bits.size)
    return out


def f32_to_bf16(x):
    """float32 array -> uint16 bf16 patterns, round to nearest even, NaN kept quiet."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().orc_f32_to_bf16_buf(_p(x), _p(out), x.size)
    return out


def allreduce_f32(x):
    """x: [n, count] float32 -> [count] float32 (what every rank must hold)."""
    x = _c(x, np.float32)
    n, count = x.shape
    out = np.empty(count, np.float32)
    lib().orc_allreduce_f32(_p(x), _p(out), n, count)
    return out


def allreduce_f32_as_i64(x):
    x = _c(x, np.float32)
    n, count = x.shape
    out = np.empty(count, np.int64)
    bad = lib().orc_allreduce_f32_as_i64(_p(x), _p(out), n, count)
    if bad:
        raise ValueError("inputs are not all integer-valued")
    return out


def allreduce_bf16(x, want_ref64=False):
    """x: [n, count] uint16 (bf16 bits) -> [count] uint16 (, [count] float64)."""
    x = _c(x, np.uint16)
    n, count = x.shape
    out = np.empty(count, np.uint16)
    ref = np.empty(count, np.float64) if want_ref64 else None
    lib().orc_allreduce_bf16(_p(x), _p(out), _p(ref), n, count)
    return (out, ref) if want_ref64 else out


def allreduce_residual_bf16(x, res, want_ref64=False):
    """x: [n, count] uint16, res: [count] uint16 (one rank's residual) -> [count] uint16."""
    x = _c(x, np.uint16)
    res = _c(res, np.uint16)
    n, count = x.shape
    assert res.shape == (count,)
    out = np.empty(count, np.uint16)
    ref = np.empty(count, np.float64) if want_ref64 else None
    lib().orc_allreduce_residual_bf16(_p(x), _p(res), _p(out), _p(ref), n, count)
    return (out, ref) if want_ref64 else out


def allreduce_residual_f32(x, res):
    x = _c(x, np.float32)
    res = _c(res, np.float32)
    n, count = x.shape
    assert res.shape == (count,)
    out = np.empty(count, np.float32)
    lib().orc_allreduce_residual_f32(_p(x), _p(res), _p(out), n, count)
    return out


def f16_to_f32(code):
    return float(lib().orc_f16_to_f32(int(code) & 0xFFFF))


def f32_to_f16(x):
    return int(lib().orc_f32_to_f16(float(np.float32(x))))


def allreduce_any(x, dtype, op):
    """x: [n, count] float32 (dtype 0), uint16 bit patterns (1 = bf16, 2 = fp16) or int32 (3);
    op 0 sum (int32: modulo 2^32), 1 max, 2 min."""
    x = np.ascontiguousarray(x)
    assert x.dtype == (np.float32 if dtype == 0 else np.int32 if dtype == 3 else np.uint16)
    n, count = x.shape
    out = np.empty(count, x.dtype)
    lib().orc_allreduce_any(_p(x), _p(out), n, count, dtype, op)
    return out


def allreduce_ring(x):
    """Ring-order AllReduce (partial sums rounded to the element type at every hop).
    x: [n, count] float32 or uint16 (bf16 bits), count % n == 0 -> [count]."""
    x = np.ascontiguousarray(x)
    n, count = x.shape
    if count % n:
        raise ValueError("count must be divisible by the number of ranks")
    out = np.empty(count, x.dtype)
    if x.dtype == np.float32:
        lib().orc_allreduce_ring_f32(_p(x), _p(out), n, count)
    elif x.dtype == np.uint16:
        lib().orc_allreduce_ring_bf16(_p(x), _p(out), n, count)
    else:
        raise TypeError(x.dtype)
    return out


def reducescatter(x):
    """x: [n, count] (float32 or uint16 bf16 bits), count % n == 0 -> [n, count/n]."""
    x = np.ascontiguousarray(x)
    n, count = x.shape
    if count % n:
        raise ValueError("count must be divisible by the number of ranks")
    out = np.empty((n, count // n), x.dtype)
    if x.dtype == np.float32:
        lib().orc_reducescatter_f32(_p(x), _p(out), n, count)
    elif x.dtype == np.uint16:
        lib().orc_reducescatter_bf16(_p(x), _p(out), n, count)
    else:
        raise TypeError(x.dtype)
    return out


def allgather(x):
    """x: [n, c] any dtype -> [n, n*c]: every row is the concatenation of all rows of x."""
    x = np.ascontiguousarray(x)
    n, c = x.shape
    out = np.empty((n, n * c), x.dtype)
    lib().orc_allgather(_p(x), _p(out), n, c * x.dtype.itemsize)
    return out


def alltoall(x):
    """x: [n, n*c] any dtype -> [n, n*c] with out[d, s*c:(s+1)*c] = x[s, d*c:(d+1)*c]."""
    x = np.ascontiguousarray(x)
    n, total = x.shape
    if total % n:
        raise ValueError("row length must be divisible by the number of ranks")
    out = np.empty_like(x)
    lib().orc_alltoall(_p(x), _p(out), n, (total // n) * x.dtype.itemsize)
    return out


def ll_encode(data, flag):
    return int(lib().orc_ll_encode(int(data) & 0xFFFFFFFF, int(flag) & 0xFFFFFFFF))


def ll_decode(unit, expect):
    w = C.c_uint32(0)
    ok = lib().orc_ll_decode(int(unit), int(expect) & 0xFFFFFFFF, C.byref(w))
    return (bool(ok), int(w.value) if ok else None)


def ll_encode_buf(payload, flag):
    """payload: uint8 array -> uint64 units (two per 16-byte packet)."""
    payload = _c(np.asarray(payload).view(np.uint8).reshape(-1), np.uint8)
    npk = (payload.size + 7) // 8
    units = np.empty(2 * npk, np.uint64)
    wrote = lib().orc_ll_encode_buf(_p(payload), payload.size, int(flag) & 0xFFFFFFFF, _p(units))
    assert wrote == units.size
    return units


def ll_decode_buf(units, nbytes, flag):
    units = _c(units, np.uint64)
    out = np.zeros(nbytes, np.uint8)
    ok = lib().orc_ll_decode_buf(_p(units), nbytes, int(flag) & 0xFFFFFFFF, _p(out))
    return (bool(ok), out if ok else None)


def moe_dispatch(tokens, topk, n_experts, cap=None):
    """tokens: [n, T, H] any dtype; topk: [n, T, K] int32.

    Returns (recv [n, cap, H], recv_src [n, cap] int32 (-1 where unused),
    counts [n dst, n src] int32, rc)."""
    tokens = np.ascontiguousarray(tokens)
    topk = _c(topk, np.int32)
    n, T, H = tokens.shape
    K = topk.shape[2]
    assert topk.shape[:2] == (n, T)
    if cap is None:
        cap = n * T
    recv = np.zeros((n, cap, H), tokens.dtype)
    src = np.full((n, cap), -1, np.int32)
    counts = np.zeros((n, n), np.int32)
    rc = lib().orc_moe_dispatch(_p(tokens), _p(topk), n, T, K, n_experts,
                                H * tokens.dtype.itemsize, _p(recv), _p(src), _p(counts), cap)
    return recv, src, counts, rc


def e4m3_to_f32(code):
    return float(lib().orc_e4m3_to_f32(int(code) & 0xFF))


def f32_to_e4m3(x):
    return int(lib().orc_f32_to_e4m3(float(np.float32(x))))


def fp8_quantize_rows(x):
    """x: [rows, H] uint16 (bf16 bits), H % 128 == 0 -> (q [rows, H] uint8, scales [rows, H/128] float32)."""
    x = _c(x, np.uint16)
    rows, H = x.shape
    assert H % 128 == 0
    q = np.empty((rows, H), np.uint8)
    scales = np.empty((rows, H // 128), np.float32)
    lib().orc_fp8_quantize_rows(_p(x), _p(q), _p(scales), rows, H)
    return q, scales


def moe_combine_bf16(y, topk, n_experts, T=None):
    """y: [n, cap, H] uint16 (bf16 bits) rows in dispatch order; topk: [n, T, K] int32.
    Returns (out [n, T, H] uint16, rc)."""
    y = _c(y, np.uint16)
    topk = _c(topk, np.int32)
    n, cap, H = y.shape
    T = topk.shape[1]
    K = topk.shape[2]
    out = np.zeros((n, T, H), np.uint16)
    acc = np.zeros(n * T * H, np.float32)
    seen = np.zeros(n * T, np.uint8)
    rc = lib().orc_moe_combine_bf16(_p(y), _p(topk), n, T, K, n_experts, H, cap, _p(out), _p(acc), _p(seen))
    return out, rc


def sem_reached(sem, expected):
    return bool(lib().orc_sem_reached(int(sem) & 0xFFFFFFFF, int(expected) & 0xFFFFFFFF))
