"""ctypes binding of libpreft.so: argument marshalling only, same names as the C ABI.

PyTorch supplies device memory and the current HIP stream; every step of the path runs in
the library's kernels.  There is no fallback: if the library is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpreft.so")

PREFT_PREFILL_ONLY = 0
PREFT_ALL_TOKENS = 1
PREFT_SCHEDULE_READY = 0x100
PREFT_F32 = 0
PREFT_BF16 = 1
PREFT_ECAPACITY = -6
PREFT_ESCHEDULE = -7
PREFT_ETOOLARGE = -8
PREFT_STATIC_SCRATCH_BYTES = 1 << 20


def PREFT_TEST_VARIANT(v: int) -> int:
    return (int(v) & 7) << 16


def PREFT_TEST_WAVES(w: int) -> int:
    return (int(w) & 15) << 19


def PREFT_TEST_ROWBLOCKS(b: int) -> int:
    return (int(b) & 3) << 23


def PREFT_TEST_COLSPLIT(c: int) -> int:
    return (int(c) & 15) << 25


def PREFT_TEST_RESIDENT(n: int) -> int:
    return (int(n) & 3) << 29


def test_flags(variant: int = 0, waves: int = 0, rowblocks: int = 0, colsplit: int = 0, resident: int = 0) -> int:
    """Test-only kernel selection bits of the C ABI's mode argument (PREFT_TEST_* in preft.h)."""
    return (PREFT_TEST_VARIANT(variant) | PREFT_TEST_WAVES(waves) | PREFT_TEST_ROWBLOCKS(rowblocks)
            | PREFT_TEST_COLSPLIT(colsplit) | PREFT_TEST_RESIDENT(resident))


# Tests and benchmarks only: bits OR-ed into the mode argument of every schedule and apply call
# made through this binding (see test_flags), so that a test can send its usual calls down a
# chosen kernel family.  The library itself keeps no such state; 0 leaves every call as written.
_extra_mode_bits = 0


def set_test_flags(bits: int = 0) -> int:
    """Sets the bits above (0: none) and returns the previous value."""
    global _extra_mode_bits
    prev, _extra_mode_bits = _extra_mode_bits, int(bits)
    return prev


def _mode(mode: int) -> int:
    return int(mode) | _extra_mode_bits

# every symbol include/preft.h declares
ABI_SYMBOLS = ("preft_workspace_bytes", "preft_workspace_bytes_z", "preft_schedule", "preft_lora_apply", "preft_lora_apply_packed",
               "preft_direft_apply", "preft_direft_apply_static", "preft_direft_apply_layers",
               "preft_loreft_prepare", "preft_loreft_apply", "preft_slots_create", "preft_slots_destroy",
               "preft_slots_store", "preft_slots_acquire", "preft_slots_pool", "preft_slots_resident",
               "preft_slots_stats", "preft_schedule_counts", "preft_strerror", "preft_version")

_lib = None


class PreftError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {preft_strerror(code)} (code {code})")


def load_library(path: Optional[str] = None):
    """Load libpreft.so (built in-tree by paper_2605_14217_amd.build; the environment variable
    PREFT_LIBRARY names another build of it) and declare its prototypes."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("PREFT_LIBRARY") or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build the HIP library first (python -m paper_2605_14217_amd.build); "
            "there is no CPU or PyTorch fallback for this path")
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, sz = c.c_void_p, c.c_int32, c.c_int64, c.c_size_t
    lib.preft_workspace_bytes.restype = sz
    lib.preft_workspace_bytes.argtypes = [i32, i32]
    lib.preft_workspace_bytes_z.restype = sz
    lib.preft_workspace_bytes_z.argtypes = [i32, i32, i32, i32]
    lib.preft_schedule.restype = c.c_int
    lib.preft_schedule.argtypes = [vp, sz, vp, vp, vp, i32, i32, i32, c.c_int, vp]
    lib.preft_lora_apply.restype = c.c_int
    lib.preft_lora_apply.argtypes = [vp, i64, vp, i64, i32, i32, i32, vp, vp, vp, i32, vp, vp, i32, i32,
                                     c.c_float, c.c_int, c.c_int, vp, sz, vp]
    lib.preft_lora_apply_packed.restype = c.c_int
    lib.preft_lora_apply_packed.argtypes = [i32, c.POINTER(vp), c.POINTER(i64), c.POINTER(i32), vp, i64, i32, i32,
                                            vp, vp, vp, i32, c.POINTER(vp), c.POINTER(vp), i32, i32,
                                            c.c_float, c.c_int, c.c_int, vp, sz, vp]
    lib.preft_direft_apply.restype = c.c_int
    lib.preft_direft_apply.argtypes = [vp, i64, i32, i32, vp, vp, vp, i32, vp, vp, vp, i32, i32,
                                       c.c_float, c.c_int, c.c_int, vp, sz, vp]
    lib.preft_direft_apply_static.restype = c.c_int
    lib.preft_direft_apply_static.argtypes = [vp, i64, i32, i32, vp, vp, vp, i32, vp, vp, vp, i32, i32,
                                              c.c_float, c.c_int, c.c_int, vp]
    lib.preft_direft_apply_layers.restype = c.c_int
    lib.preft_direft_apply_layers.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, i32, vp, vp, vp, i32, i32,
                                              c.c_float, c.c_int, c.c_int, vp, sz, vp]
    lib.preft_loreft_prepare.restype = c.c_int
    lib.preft_loreft_prepare.argtypes = [vp, vp, vp, vp, i32, i32, c.c_int, vp]
    lib.preft_loreft_apply.restype = c.c_int
    lib.preft_loreft_apply.argtypes = lib.preft_direft_apply.argtypes
    lib.preft_slots_create.restype = c.c_int
    lib.preft_slots_create.argtypes = [c.POINTER(vp), i32, i32, i32, c.POINTER(sz)]
    lib.preft_slots_destroy.restype = c.c_int
    lib.preft_slots_destroy.argtypes = [vp]
    lib.preft_slots_store.restype = c.c_int
    lib.preft_slots_store.argtypes = [vp, i32, i32, vp, vp]
    lib.preft_slots_acquire.restype = c.c_int
    lib.preft_slots_acquire.argtypes = [vp, c.POINTER(i32), i32, c.POINTER(i32), vp]
    lib.preft_slots_pool.restype = vp
    lib.preft_slots_pool.argtypes = [vp, i32]
    lib.preft_slots_resident.restype = i32
    lib.preft_slots_resident.argtypes = [vp, i32]
    lib.preft_slots_stats.restype = c.c_int
    lib.preft_slots_stats.argtypes = [vp, c.POINTER(i64)]
    lib.preft_schedule_counts.restype = c.c_int
    lib.preft_schedule_counts.argtypes = [vp, c.POINTER(i32), vp]
    lib.preft_strerror.restype = c.c_char_p
    lib.preft_strerror.argtypes = [c.c_int]
    lib.preft_version.restype = c.c_int
    lib.preft_version.argtypes = []
    _lib = lib
    return lib


# ----------------------------------------------------------------------------------------
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return PREFT_BF16
    if t.dtype == torch.float32:
        return PREFT_F32
    raise TypeError(f"unsupported activation dtype {t.dtype}")


def _matrix(t: torch.Tensor, name: str):
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise ValueError(f"{name}: need a 2-D device tensor with unit column stride")
    return t.data_ptr(), int(t.stride(0)), int(t.shape[0]), int(t.shape[1])


def _table(t: torch.Tensor, name: str, n: int):
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or t.numel() != n:
        raise ValueError(f"{name}: need a contiguous int32 device tensor of {n} entries")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise PreftError(rc, where)


def pointer_table(mats: Sequence[torch.Tensor]) -> torch.Tensor:
    """Device array of device pointers, one per adapter slot (the pool argument of the C ABI).
    The table only names the tensors: the caller keeps them alive while the table is in use."""
    dev = mats[0].device
    for m in mats:
        if not m.is_cuda or not m.is_contiguous():
            raise ValueError("pool slots must be contiguous device tensors")
    return torch.tensor([m.data_ptr() for m in mats], dtype=torch.int64, device=dev)


class PoolRef:
    """A pointer table that lives in library-owned device memory (the slot manager's): quacks like
    the int64 tensor of pointer_table as far as the apply calls need."""
    dtype = torch.int64

    def __init__(self, address: int, n: int):
        self._address, self._n = int(address), int(n)

    def data_ptr(self) -> int:
        return self._address

    def numel(self) -> int:
        return self._n


def preft_version() -> int:
    return int(load_library().preft_version())


def preft_strerror(code: int) -> str:
    return load_library().preft_strerror(int(code)).decode()


def preft_workspace_bytes(T: int, S: int) -> int:
    return int(load_library().preft_workspace_bytes(int(T), int(S)))


def preft_workspace_bytes_z(T: int, S: int, rank: int, n_proj: int = 1) -> int:
    return int(load_library().preft_workspace_bytes_z(int(T), int(S), int(rank), int(n_proj)))


def new_workspace(T: int, S: int, device="cuda", z_rank: int = 0, z_proj: int = 1) -> torch.Tensor:
    """Caller-owned workspace for a batch of T rows in S segments; with z_rank > 0 it also has room for
    the intermediate z of LoRA calls of up to that rank and z_proj outputs (preft_workspace_bytes_z)."""
    n = preft_workspace_bytes_z(T, S, z_rank, z_proj) if z_rank > 0 else preft_workspace_bytes(T, S)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def preft_schedule(workspace: torch.Tensor, seg_start, seg_adapter, seg_prefill_len, T: int, N: int,
                   mode: int, stream=None) -> None:
    S = int(seg_adapter.numel())
    rc = load_library().preft_schedule(
        workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S, int(T), int(N), int(mode), _stream(stream))
    _check(rc, "preft_schedule")


def preft_schedule_counts(workspace: torch.Tensor, stream=None):
    out = (ctypes.c_int32 * 3)()
    _check(load_library().preft_schedule_counts(workspace.data_ptr(), out, _stream(stream)),
           "preft_schedule_counts")          # raises PREFT_ESCHEDULE if an apply call refused the schedule
    return int(out[0]), int(out[1]), int(out[2])


def preft_lora_apply(y: torch.Tensor, x: torch.Tensor, seg_start, seg_adapter, seg_prefill_len,
                     A_pool: torch.Tensor, B_pool: torch.Tensor, rank: int, scale: float, mode: int,
                     workspace: torch.Tensor, stream=None) -> None:
    """y[t] += scale * B_i (A_i x[t]) on active rows, in place.  A_pool/B_pool: pointer tables
    (see pointer_table) of [rank, d_in] and [d_out, rank] matrices."""
    yp, ldy, T, d_out = _matrix(y, "y")
    xp, ldx, T2, d_in = _matrix(x, "x")
    if T != T2 or x.dtype != y.dtype:
        raise ValueError("x and y must agree in rows and dtype")
    S = int(seg_adapter.numel())
    N = int(A_pool.numel())
    if B_pool.numel() != N or A_pool.dtype != torch.int64 or B_pool.dtype != torch.int64:
        raise ValueError("A_pool and B_pool must be int64 pointer tables of equal length")
    rc = load_library().preft_lora_apply(
        yp, ldy, xp, ldx, T, d_in, d_out,
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S,
        A_pool.data_ptr(), B_pool.data_ptr(), N, int(rank), float(scale), _dtype_code(y), _mode(mode),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "preft_lora_apply")


def preft_lora_apply_packed(ys: Sequence[torch.Tensor], x: torch.Tensor, seg_start, seg_adapter, seg_prefill_len,
                            A_pools: Sequence, B_pools: Sequence, rank: int, scale: float, mode: int,
                            workspace: torch.Tensor, stream=None) -> None:
    """ys[p][t] += scale * B_{p,i} (A_{p,i} x[t]) for every projection p of the same x (q,k,v or
    gate,up); ys may be separate tensors or column slices of one tensor."""
    n = len(ys)
    if len(A_pools) != n or len(B_pools) != n:
        raise ValueError("one A pool and one B pool per output")
    xp, ldx, T, d_in = _matrix(x, "x")
    yp, ldy, d_out = (ctypes.c_void_p * n)(), (ctypes.c_int64 * n)(), (ctypes.c_int32 * n)()
    Ap, Bp = (ctypes.c_void_p * n)(), (ctypes.c_void_p * n)()
    N = int(A_pools[0].numel())
    for i, y in enumerate(ys):
        yp[i], ldy[i], T2, d_out[i] = _matrix(y, f"ys[{i}]")
        if T2 != T or y.dtype != x.dtype:
            raise ValueError("x and every y must agree in rows and dtype")
        if A_pools[i].numel() != N or B_pools[i].numel() != N or A_pools[i].dtype != torch.int64:
            raise ValueError("pools must be int64 pointer tables of equal length")
        Ap[i], Bp[i] = A_pools[i].data_ptr(), B_pools[i].data_ptr()
    S = int(seg_adapter.numel())
    rc = load_library().preft_lora_apply_packed(
        n, yp, ldy, d_out, xp, ldx, T, d_in,
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S, Ap, Bp, N, int(rank), float(scale), _dtype_code(x),
        _mode(mode), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "preft_lora_apply_packed")


def preft_loreft_prepare(D: torch.Tensor, Rt: torch.Tensor, W: torch.Tensor, R: torch.Tensor, stream=None) -> None:
    """Derived LoReFT factors of one adapter: D = W - R ([rank, d]) and Rt = R^T ([d, rank]),
    written into the caller's contiguous device tensors."""
    rank, d = int(W.shape[0]), int(W.shape[1])
    for t, shape, name in ((D, (rank, d), "D"), (Rt, (d, rank), "Rt"), (W, (rank, d), "W"), (R, (rank, d), "R")):
        if tuple(t.shape) != shape or not t.is_contiguous() or not t.is_cuda or t.dtype != W.dtype:
            raise ValueError(f"{name}: need a contiguous device tensor of shape {shape} and the dtype of W")
    rc = load_library().preft_loreft_prepare(D.data_ptr(), Rt.data_ptr(), W.data_ptr(), R.data_ptr(), d, rank,
                                             _dtype_code(W), _stream(stream))
    _check(rc, "preft_loreft_prepare")


def preft_loreft_apply(h: torch.Tensor, seg_start, seg_adapter, seg_prefill_len,
                       D_pool: torch.Tensor, Rt_pool: torch.Tensor, b_pool: Optional[torch.Tensor],
                       rank: int, scale: float, mode: int, workspace: torch.Tensor, stream=None) -> None:
    """h[t] += scale * R_i^T (W_i h[t] + b_i - R_i h[t]) on active rows, in place, from the derived
    factors of preft_loreft_prepare (pointer tables of D = W - R and of R^T)."""
    _reft_apply("preft_loreft_apply", h, seg_start, seg_adapter, seg_prefill_len, D_pool, Rt_pool, b_pool, rank,
                scale, mode, workspace, stream)


def preft_direft_apply(h: torch.Tensor, seg_start, seg_adapter, seg_prefill_len,
                       W1_pool: torch.Tensor, W2t_pool: torch.Tensor, b_pool: Optional[torch.Tensor],
                       rank: int, scale: float, mode: int, workspace: torch.Tensor, stream=None) -> None:
    """h[t] += scale * W2_i^T (W1_i h[t] + b_i) on active rows, in place.  W1_pool: [rank, d]
    matrices; W2t_pool: [d, rank] matrices (W2 transposed); b_pool: [rank] vectors or None."""
    _reft_apply("preft_direft_apply", h, seg_start, seg_adapter, seg_prefill_len, W1_pool, W2t_pool, b_pool, rank,
                scale, mode, workspace, stream)


def preft_direft_apply_static(h: torch.Tensor, seg_start, seg_adapter, seg_prefill_len,
                              W1_pool: torch.Tensor, W2t_pool: torch.Tensor, b_pool: Optional[torch.Tensor],
                              rank: int, scale: float, mode: int, stream=None) -> None:
    """preft_direft_apply without a workspace: the schedule lives in the library's static device area
    (for callers that cannot allocate).  The call itself allocates nothing."""
    hp, ldh, T, d = _matrix(h, "h")
    S = int(seg_adapter.numel())
    N = int(W1_pool.numel())
    if W2t_pool.numel() != N or (b_pool is not None and b_pool.numel() != N):
        raise ValueError("pools must be pointer tables of equal length")
    rc = load_library().preft_direft_apply_static(
        hp, ldh, T, d,
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S,
        W1_pool.data_ptr(), W2t_pool.data_ptr(), None if b_pool is None else b_pool.data_ptr(), N,
        int(rank), float(scale), _dtype_code(h), _mode(mode), _stream(stream))
    _check(rc, "preft_direft_apply_static")


def preft_direft_apply_layers(hs: Sequence[torch.Tensor], h_layers: torch.Tensor, seg_start, seg_adapter,
                              seg_prefill_len, W1_pools: torch.Tensor, W2t_pools: torch.Tensor,
                              b_pools: Optional[torch.Tensor], N: int, rank: int, scale: float, mode: int,
                              workspace: torch.Tensor, stream=None) -> None:
    """DiReFT on len(hs) residual streams in one launch.  hs: the [T, d] device tensors (equal shape,
    stride and dtype); h_layers = pointer_table(hs) made once by the caller; W1_pools / W2t_pools /
    b_pools: int64 device tensors of len(hs) entries, each the data_ptr() of that layer's pointer
    table of N slots (b_pools None: no bias; an entry 0: no bias in that layer)."""
    L = len(hs)
    hp, ldh, T, d = _matrix(hs[0], "hs[0]")
    for i, h in enumerate(hs):
        if _matrix(h, f"hs[{i}]")[1:] != (ldh, T, d) or h.dtype != hs[0].dtype:
            raise ValueError("the residual streams must agree in shape, row stride and dtype")
    for t, name in ((h_layers, "h_layers"), (W1_pools, "W1_pools"), (W2t_pools, "W2t_pools"), (b_pools, "b_pools")):
        if t is None and name == "b_pools":
            continue
        if t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous() or t.numel() != L:
            raise ValueError(f"{name}: need a contiguous int64 device tensor of {L} pointers")
    S = int(seg_adapter.numel())
    rc = load_library().preft_direft_apply_layers(
        h_layers.data_ptr(), ldh, L, T, d,
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S,
        W1_pools.data_ptr(), W2t_pools.data_ptr(), None if b_pools is None else b_pools.data_ptr(), int(N),
        int(rank), float(scale), _dtype_code(hs[0]), _mode(mode),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "preft_direft_apply_layers")


def _reft_apply(entry: str, h, seg_start, seg_adapter, seg_prefill_len, W1_pool, W2t_pool, b_pool, rank, scale,
                mode, workspace, stream) -> None:
    hp, ldh, T, d = _matrix(h, "h")
    S = int(seg_adapter.numel())
    N = int(W1_pool.numel())
    if W2t_pool.numel() != N or (b_pool is not None and b_pool.numel() != N):
        raise ValueError("pools must be pointer tables of equal length")
    rc = getattr(load_library(), entry)(
        hp, ldh, T, d,
        _table(seg_start, "seg_start", S + 1), _table(seg_adapter, "seg_adapter", S),
        _table(seg_prefill_len, "seg_prefill_len", S), S,
        W1_pool.data_ptr(), W2t_pool.data_ptr(), None if b_pool is None else b_pool.data_ptr(), N,
        int(rank), float(scale), _dtype_code(h), _mode(mode),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, entry)


# ----------------------------------------------------------------------------------------
# adapter slot manager (argument marshalling only; the handle is the library's opaque pointer)
# ----------------------------------------------------------------------------------------
def preft_slots_create(n_adapters: int, n_slots: int, part_bytes) -> int:
    """Returns the manager handle.  part_bytes: bytes of each matrix of one adapter ([] = bookkeeping only)."""
    handle = ctypes.c_void_p()
    arr = (ctypes.c_size_t * max(len(part_bytes), 1))(*[int(b) for b in part_bytes])
    _check(load_library().preft_slots_create(ctypes.byref(handle), int(n_adapters), int(n_slots), len(part_bytes), arr),
           "preft_slots_create")
    return handle.value


def preft_slots_destroy(handle: int) -> None:
    _check(load_library().preft_slots_destroy(handle), "preft_slots_destroy")


def preft_slots_store(handle: int, adapter: int, part: int, src: torch.Tensor, stream=None) -> None:
    """src: contiguous CPU tensor holding the matrix."""
    if src.is_cuda or not src.is_contiguous():
        raise ValueError("src: need a contiguous CPU tensor")
    _check(load_library().preft_slots_store(handle, int(adapter), int(part), src.data_ptr(),
                                            _stream(stream) if torch.cuda.is_available() else None),
           "preft_slots_store")


def preft_slots_acquire(handle: int, adapter_ids, stream=None):
    """adapter_ids: sequence of ints -> list of slot ids (-1 = no adapter)."""
    n = len(adapter_ids)
    ids = (ctypes.c_int32 * max(n, 1))(*[int(a) for a in adapter_ids])
    out = (ctypes.c_int32 * max(n, 1))()
    _check(load_library().preft_slots_acquire(handle, ids, n, out,
                                              _stream(stream) if torch.cuda.is_available() else None),
           "preft_slots_acquire")
    return [int(out[i]) for i in range(n)]


def preft_slots_pool(handle: int, part: int) -> PoolRef:
    """Pointer table of part `part` (n_slots entries), usable as a pool argument of the apply calls."""
    address = load_library().preft_slots_pool(handle, int(part))
    if not address:
        raise PreftError(-1, "preft_slots_pool")
    return PoolRef(address, preft_slots_stats(handle)["n_slots"])


def preft_slots_resident(handle: int, adapter: int) -> int:
    return int(load_library().preft_slots_resident(handle, int(adapter)))


def preft_slots_stats(handle: int) -> dict:
    out = (ctypes.c_int64 * 5)()
    _check(load_library().preft_slots_stats(handle, out), "preft_slots_stats")
    return dict(hits=int(out[0]), misses=int(out[1]), evictions=int(out[2]), bytes_copied=int(out[3]),
                n_slots=int(out[4]))
