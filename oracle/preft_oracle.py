"""ctypes front end of the fp64 CPU oracle (``preft_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the CPU-baseline leg of the benchmark may import
this module; the product path never does.  Argument marshalling only: all arithmetic is
in the C file, which states the paper's Eq. 1-4 as plain fp64 loops.

Tensors may be numpy arrays (float64 / float32) or CPU torch tensors (float64 / float32 /
bfloat16); they are handed to C in their storage type and widened exactly there.
Adapter weights use the paper's shapes: LoRA ``A:[r,m]``, ``B:[n,r]`` (Eq. 2); DiReFT
``A,B:[r,d]``, ``b:[r]`` (Eq. 3).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "preft_oracle.c")
_LIB = os.path.join(_HERE, "libpreft_oracle.so")

PROMPT_ONLY = 0      # P^PreFT = {1..p}            (Eq. 4)
ALL_POSITIONS = 1    # P^A     = {1..p+T}          (Sec. 3.2)

_F64, _F32, _BF16 = 0, 1, 2
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        dblp = ctypes.POINTER(ctypes.c_double)
        vpp = ctypes.POINTER(ctypes.c_void_p)
        lib.ora_positions.restype = ctypes.c_int
        lib.ora_positions.argtypes = [i32p, ctypes.c_int64, i32p, i32p, i32p,
                                      ctypes.c_int32, ctypes.c_int32, ctypes.c_int]
        lib.ora_lora_batch.restype = ctypes.c_int
        lib.ora_lora_batch.argtypes = [dblp, i64p, ctypes.c_int64,
                                       ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                       ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                       i32p, i32p, i32p, ctypes.c_int32,
                                       vpp, vpp, ctypes.c_int32,
                                       ctypes.c_int32, ctypes.c_double, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.ora_direft_batch.restype = ctypes.c_int
        lib.ora_direft_batch.argtypes = [dblp, i64p, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         i32p, i32p, i32p, ctypes.c_int32,
                                         vpp, vpp, vpp, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_double, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.ora_loreft_batch.restype = ctypes.c_int
        lib.ora_loreft_batch.argtypes = lib.ora_direft_batch.argtypes
        lib.ora_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().ora_threads())


# ----------------------------------------------------------------------------------------
# marshalling helpers
# ----------------------------------------------------------------------------------------
def _as_typed(a):
    """-> (numpy array sharing/holding the bits, dtype code).  bf16 is carried as uint16."""
    try:
        import torch
    except ImportError:  # pragma: no cover
        torch = None
    if torch is not None and isinstance(a, torch.Tensor):
        if a.device.type != "cpu":
            raise ValueError("the oracle takes CPU tensors only")
        a = a.contiguous()
        if a.dtype == torch.bfloat16:
            return a.view(torch.int16).numpy().view(np.uint16), _BF16
        if a.dtype == torch.float32:
            return a.numpy(), _F32
        if a.dtype == torch.float64:
            return a.numpy(), _F64
        raise ValueError(f"unsupported dtype {a.dtype}")
    a = np.ascontiguousarray(a)
    if a.dtype == np.float64:
        return a, _F64
    if a.dtype == np.float32:
        return a, _F32
    raise ValueError(f"unsupported dtype {a.dtype}")


def _i32(a):
    try:
        import torch
        if isinstance(a, torch.Tensor):
            a = a.cpu().numpy()
    except ImportError:  # pragma: no cover
        pass
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _pool(mats, shape):
    """list of per-adapter matrices (entries may be None = never dereferenced)."""
    keep, code = [], None
    arr = (ctypes.c_void_p * max(len(mats), 1))()
    for i, m in enumerate(mats):
        if m is None:
            arr[i] = None
            continue
        t, c = _as_typed(m)
        if tuple(t.shape) != tuple(shape):
            raise ValueError(f"adapter {i}: shape {tuple(t.shape)} != {tuple(shape)}")
        if code is not None and c != code:
            raise ValueError("mixed weight dtypes in one pool")
        code = c
        keep.append(t)
        arr[i] = t.ctypes.data
    return arr, (code if code is not None else _F64), keep


def positions(T, seg_start, seg_adapter, seg_prompt_len, N, position_set):
    """Per-row acting adapter id, -1 where Eq. 1 leaves the row alone."""
    lib = _load()
    ss, sa, sp = _i32(seg_start), _i32(seg_adapter), _i32(seg_prompt_len)
    S = len(sa)
    assert len(ss) == S + 1 and len(sp) == S
    out = np.empty(max(T, 1), dtype=np.int32)
    rc = lib.ora_positions(_ptr(out, ctypes.c_int32), T, _ptr(ss, ctypes.c_int32),
                           _ptr(sa, ctypes.c_int32), _ptr(sp, ctypes.c_int32), S, N, position_set)
    if rc:
        raise ValueError("malformed segment table")
    return out[:T]


def lora(y0, x, seg_start, seg_adapter, seg_prompt_len, A_pool, B_pool, r, alpha,
         position_set, rows=None, gathered=False):
    """Eq. 1/2/4 over a batch: fp64 array [T,n] (or [len(rows),n]).

    gathered=True (needs rows): y0 and x hold only the selected rows, in the order of `rows`."""
    lib = _load()
    y0a, dt_y = _as_typed(y0)
    xa, dt_x = _as_typed(x)
    if dt_y != dt_x:
        raise ValueError("x and y0 must share a dtype")
    ss, sa, sp = _i32(seg_start), _i32(seg_adapter), _i32(seg_prompt_len)
    S = len(sa)
    assert len(ss) == S + 1 and len(sp) == S
    n, m = y0a.shape[1], xa.shape[1]
    assert y0a.shape[0] == xa.shape[0]
    if gathered:
        assert rows is not None and len(rows) == y0a.shape[0]
        T = int(ss[-1])
    else:
        T = y0a.shape[0]
    N = len(A_pool)
    assert len(B_pool) == N
    Ap, dt_w, keepA = _pool(A_pool, (r, m))
    Bp, dt_w2, keepB = _pool(B_pool, (n, r))
    if keepA and keepB and dt_w != dt_w2:
        raise ValueError("A and B pools must share a dtype")
    if rows is None:
        rows_arr, rows_p, count = None, None, T
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        assert rows_arr.size == 0 or (rows_arr.min() >= 0 and rows_arr.max() < T)
        rows_p, count = _ptr(rows_arr, ctypes.c_int64), len(rows_arr)
    out = np.empty((count, n), dtype=np.float64)
    rc = lib.ora_lora_batch(_ptr(out, ctypes.c_double), rows_p, count,
                            y0a.ctypes.data, n, xa.ctypes.data, m, T, m, n,
                            _ptr(ss, ctypes.c_int32), _ptr(sa, ctypes.c_int32),
                            _ptr(sp, ctypes.c_int32), S,
                            Ap, Bp, N, r, float(alpha), position_set, dt_x, dt_w, int(bool(gathered)))
    if rc:
        raise ValueError("malformed segment table")
    return out


def direft(h, seg_start, seg_adapter, seg_prompt_len, A_pool, B_pool, b_pool, r, s,
           position_set, rows=None, gathered=False):
    """Eq. 1/3/4 (with the prefactor s of App. C.2) over a batch: fp64 [T,d] or [len(rows),d].

    gathered=True (needs rows): h holds only the selected rows, in the order of `rows`."""
    return _reft(_load().ora_direft_batch, h, seg_start, seg_adapter, seg_prompt_len, A_pool, B_pool, b_pool,
                 r, s, position_set, rows, gathered)


def loreft(h, seg_start, seg_adapter, seg_prompt_len, W_pool, R_pool, b_pool, r, s,
           position_set, rows=None, gathered=False):
    """LoReFT of App. C.2, h + s R^T (W h + b - R h), on the rows of Eq. 1/4; W, R are [r,d] each.
    Same conventions as `direft`."""
    return _reft(_load().ora_loreft_batch, h, seg_start, seg_adapter, seg_prompt_len, W_pool, R_pool, b_pool,
                 r, s, position_set, rows, gathered)


def _reft(entry, h, seg_start, seg_adapter, seg_prompt_len, A_pool, B_pool, b_pool, r, s,
          position_set, rows, gathered):
    ha, dt_h = _as_typed(h)
    d = ha.shape[1]
    ss, sa, sp = _i32(seg_start), _i32(seg_adapter), _i32(seg_prompt_len)
    S = len(sa)
    assert len(ss) == S + 1 and len(sp) == S
    if gathered:
        assert rows is not None and len(rows) == ha.shape[0]
        T = int(ss[-1])
    else:
        T = ha.shape[0]
    N = len(A_pool)
    assert len(B_pool) == N
    Ap, dt_w, keepA = _pool(A_pool, (r, d))
    Bp, dt_w2, keepB = _pool(B_pool, (r, d))
    if keepA and keepB and dt_w != dt_w2:
        raise ValueError("A and B pools must share a dtype")
    if b_pool is None:
        bp, keepb = None, []
    else:
        assert len(b_pool) == N
        bp, dt_b, keepb = _pool(b_pool, (r,))
        if keepb and keepA and dt_b != dt_w:
            raise ValueError("bias pool dtype differs from the weights'")
    if rows is None:
        rows_arr, rows_p, count = None, None, T
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        assert rows_arr.size == 0 or (rows_arr.min() >= 0 and rows_arr.max() < T)
        rows_p, count = _ptr(rows_arr, ctypes.c_int64), len(rows_arr)
    out = np.empty((count, d), dtype=np.float64)
    rc = entry(_ptr(out, ctypes.c_double), rows_p, count,
                              ha.ctypes.data, d, T, d,
                              _ptr(ss, ctypes.c_int32), _ptr(sa, ctypes.c_int32),
                              _ptr(sp, ctypes.c_int32), S,
                              Ap, Bp, bp, N, r, float(s), position_set, dt_h, dt_w, int(bool(gathered)))
    if rc:
        raise ValueError("malformed segment table")
    return out
