"""ctypes binding with the same names as include/ptqtp.h.

Tensors are torch CUDA(HIP) tensors; the binding only checks dtype/device/
contiguity, allocates outputs, and passes raw pointers plus the current stream.
"""
from __future__ import annotations

import ctypes
import os
import weakref

import torch

PTQTP_F32, PTQTP_F16 = 0, 1
PTQTP_FUSED_PLANES = 16      # OR into ptqtp_gemm's y_dtype
PTQTP_GEMM_SMALL_MAX_M = 64

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libptqtp.so")
_lib = None


class PtqtpError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {ptqtp_status_string(status)} (status {status})")
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(_LIB_PATH)
        p, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        lib.ptqtp_version.restype = i32
        lib.ptqtp_version.argtypes = []
        lib.ptqtp_status_string.restype = ctypes.c_char_p
        lib.ptqtp_status_string.argtypes = [i32]
        lib.ptqtp_packed_bytes.restype = sz
        lib.ptqtp_packed_bytes.argtypes = [i64, i64, i64, i32]
        lib.ptqtp_workspace_bytes.restype = sz
        lib.ptqtp_workspace_bytes.argtypes = [i64, i64, i64, i32]
        lib.ptqtp_pack.restype = i32
        lib.ptqtp_pack.argtypes = [p, p, p, p, i64, i64, i64, i32, p, sz, p, p]
        lib.ptqtp_check_blob.restype = i32
        lib.ptqtp_check_blob.argtypes = [p, sz, i64, i64, i32, p, p]
        lib.ptqtp_unpack.restype = i32
        lib.ptqtp_unpack.argtypes = [p, i64, i64, i64, i32, p, p, p, p, p]
        lib.ptqtp_gemv.restype = i32
        lib.ptqtp_gemv.argtypes = [p, p, p, i32, i64, i64, i64, i32, p, sz, p]
        lib.ptqtp_gemm_small.restype = i32
        lib.ptqtp_gemm_small.argtypes = [p, p, p, i32, i64, i64, i64, i32, p, sz, p]
        lib.ptqtp_gemm.restype = i32
        lib.ptqtp_gemm.argtypes = [p, p, p, i32, i64, i64, i64, i32, p, sz, p]
        lib.ptqtp_chain_plan_bytes.restype = sz
        lib.ptqtp_chain_plan_bytes.argtypes = [p, i32, i32]
        lib.ptqtp_chain_plan.restype = i32
        lib.ptqtp_chain_plan.argtypes = [p, i32, i32, p, sz, p]
        lib.ptqtp_chain_run.restype = i32
        lib.ptqtp_chain_run.argtypes = [p, i32, i32, p, p]
        lib.ptqtp_chain_run_batch.restype = i32
        lib.ptqtp_chain_run_batch.argtypes = [p, i32, i32, i64, p]
        lib.ptqtp_batch_plan_bytes.restype = sz
        lib.ptqtp_batch_plan_bytes.argtypes = [p, i32, i32]
        lib.ptqtp_batch_items.restype = i64
        lib.ptqtp_batch_items.argtypes = [p, i32, i32]
        lib.ptqtp_gemv_batch_plan.restype = i32
        lib.ptqtp_gemv_batch_plan.argtypes = [p, i32, i32, i32, p, sz, p]
        lib.ptqtp_gemv_batch.restype = i32
        lib.ptqtp_gemv_batch.argtypes = [p, i64, p]
        lib.ptqtp_gemm_batch.restype = i32
        lib.ptqtp_gemm_batch.argtypes = [p, i64, i64, p]
        lib.ptqtp_gemm_batch_fused.restype = i32
        lib.ptqtp_gemm_batch_fused.argtypes = [p, i64, i64, p]
        lib.ptqtp_quantize_workspace_bytes.restype = sz
        lib.ptqtp_quantize_workspace_bytes.argtypes = [i64, i64, i32]
        lib.ptqtp_quantize.restype = i32
        lib.ptqtp_quantize.argtypes = [p, i64, i64, i32, i32, ctypes.c_double, p, p, p, p, p, p, sz, p]
        lib.ptqtp_quantize_static.restype = i32
        lib.ptqtp_quantize_static.argtypes = [p, i64, i64, i32, i32, ctypes.c_double, p, p, p, p, p, p]
        lib.ptqtp_tune.restype = i32
        lib.ptqtp_tune.argtypes = [ctypes.c_char_p, i32]
        lib.ptqtp_gemm_route.restype = i32
        lib.ptqtp_gemm_route.argtypes = [i64, i64, i64, i32, i32, p]
        _lib = lib
    return _lib


def raw():
    """The ctypes library handle (for tests of the C ABI itself)."""
    return _load()


def ptqtp_version() -> int:
    return int(_load().ptqtp_version())


def ptqtp_status_string(status: int) -> str:
    return _load().ptqtp_status_string(int(status)).decode()


def ptqtp_packed_bytes(M: int, N: int, K: int, group: int = 128) -> int:
    return int(_load().ptqtp_packed_bytes(M, N, K, group))


def ptqtp_workspace_bytes(M: int, N: int, K: int, group: int = 128) -> int:
    return int(_load().ptqtp_workspace_bytes(M, N, K, group))


def ptqtp_tune(key: str, value: int) -> None:
    st = _load().ptqtp_tune(key.encode(), int(value))
    if st:
        raise PtqtpError(st, "ptqtp_tune")


PTQTP_ROUTE_STREAM, PTQTP_ROUTE_SMALL, PTQTP_ROUTE_SMALL_CHUNKS, PTQTP_ROUTE_TILE = 0, 1, 2, 3
TILE_SHAPES = ((256, 256), (256, 128), (128, 128), (128, 64), (64, 64))   # rows x tokens per route tile index


def ptqtp_gemm_route(M: int, N: int, K: int, group: int = 128, y_dtype: int = PTQTP_F32):
    """(path, tile, split_row_tile, second_tile): which kernels ptqtp_gemm would run (host logic, no GPU)."""
    r = (ctypes.c_int32 * 4)()
    st = _load().ptqtp_gemm_route(int(M), int(N), int(K), int(group), int(y_dtype), r)
    if st:
        raise PtqtpError(st, "ptqtp_gemm_route")
    return tuple(int(v) for v in r)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU, got {t.dtype} on {t.device}")
    return t.data_ptr()


def ptqtp_pack(T1, T2, a1, a2, M: int = 1, group: int = 128, check: bool = True) -> torch.Tensor:
    """Pack int8 planes [N,K] and fp16 scales [N,K/group] -> opaque uint8 blob on the GPU."""
    N, K = T1.shape
    nbytes = ptqtp_packed_bytes(M, N, K, group)
    if nbytes == 0:
        raise PtqtpError(2 if group == 128 else 3, "ptqtp_packed_bytes")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=T1.device)
    status = torch.empty(1, dtype=torch.int32, device=T1.device)
    st = _load().ptqtp_pack(_dev(T1, torch.int8, "T1"), _dev(T2, torch.int8, "T2"),
                            _dev(a1, torch.float16, "a1"), _dev(a2, torch.float16, "a2"),
                            M, N, K, group, packed.data_ptr(), nbytes, status.data_ptr(), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_pack")
    if check and int(status.item()) != 0:
        raise ValueError("ptqtp_pack: a plane holds a value outside {-1, 0, +1}")
    _mark_checked(packed, N, K, group)          # written by the library for this very shape
    return packed


def ptqtp_unpack(packed: torch.Tensor, N: int, K: int, M: int = 1, group: int = 128):
    _check_blob(packed, N, K, group, "ptqtp_unpack")
    dev = packed.device
    T1 = torch.empty((N, K), dtype=torch.int8, device=dev)
    T2 = torch.empty((N, K), dtype=torch.int8, device=dev)
    a1 = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    a2 = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    st = _load().ptqtp_unpack(_dev(packed, torch.uint8, "packed"), M, N, K, group, T1.data_ptr(), T2.data_ptr(),
                              a1.data_ptr(), a2.data_ptr(), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_unpack")
    return T1, T2, a1, a2


PTQTP_BLOB_BAD_MAGIC, PTQTP_BLOB_BAD_LAYOUT, PTQTP_BLOB_BAD_GROUP, PTQTP_BLOB_BAD_N, PTQTP_BLOB_BAD_K = 1, 2, 4, 8, 16
_checked = {}      # id(blob tensor) -> (weak reference to it, set of (N, K, group, version) already found good)


def _good_shapes(packed: torch.Tensor):
    entry = _checked.get(id(packed))
    return entry[1] if entry is not None and entry[0]() is packed else None


def ptqtp_check_blob(packed: torch.Tensor, N: int, K: int, group: int = 128) -> int:
    """Header of `packed` against (N, K, group) on the device; returns the PTQTP_BLOB_BAD_* bits (0 = good).
    Synchronises to read the status word."""
    status = torch.empty(1, dtype=torch.int32, device=packed.device)
    st = _load().ptqtp_check_blob(_dev(packed, torch.uint8, "packed"), packed.numel(), int(N), int(K), int(group),
                                  status.data_ptr(), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_check_blob")
    return int(status.item())


def _mark_checked(packed: torch.Tensor, N: int, K: int, group: int) -> None:
    shapes = _good_shapes(packed)
    if shapes is None:
        key, shapes = id(packed), set()
        _checked[key] = (weakref.ref(packed, lambda _ref, key=key: _checked.pop(key, None)), shapes)
    shapes.add((int(N), int(K), int(group), packed._version))


def _check_blob(packed: torch.Tensor, N: int, K: int, group: int, where: str) -> None:
    """The kernels trust N and K: a blob shorter than those need would be read past its end, and one packed for
    another shape would be streamed as it is.  Size on the host at every call; the header on the device once per
    (blob, shape) -- not while the stream is being captured, where nothing can be read back."""
    need = ptqtp_packed_bytes(1, N, K, group)
    if need == 0:
        raise PtqtpError(2 if group == 128 else 3, where)
    if packed.numel() < need:
        raise PtqtpError(4, where)
    key = (int(N), int(K), int(group), packed._version)
    if not packed.is_cuda:                      # refused with a TypeError where its pointer is taken
        return
    if key in (_good_shapes(packed) or ()) or torch.cuda.is_current_stream_capturing():
        return
    bad = ptqtp_check_blob(packed, N, K, group)
    if bad:
        names = [n for b, n in ((1, "magic"), (2, "layout id"), (4, "group"), (8, "N"), (16, "K")) if bad & b]
        raise ValueError(f"{where}: the blob's header does not match N={N}, K={K}, group={group} ({', '.join(names)} differ)")
    _mark_checked(packed, N, K, group)


def _forward(fn, where, packed, x, N, K, M, group, y_dtype, out):
    ydt = torch.float32 if (y_dtype & ~PTQTP_FUSED_PLANES) == PTQTP_F32 else torch.float16
    _check_blob(packed, N, K, group, where)
    if out is None:
        out = torch.empty((M, N), dtype=ydt, device=x.device)
    elif out.numel() != M * N:
        raise PtqtpError(2, where)
    st = fn(_dev(packed, torch.uint8, "packed"), _dev(x, torch.float16, "x"), _dev(out, ydt, "y"), y_dtype,
            M, N, K, group, None, 0, _stream())
    if st:
        raise PtqtpError(st, where)
    return out


def ptqtp_gemv(packed, x, N: int, K: int, group: int = 128, y_dtype: int = PTQTP_F32, out=None):
    """y [1,N] = dual trit-plane layer applied to x (fp16, K elements)."""
    if x.numel() != K:
        raise PtqtpError(2, "ptqtp_gemv")
    return _forward(_load().ptqtp_gemv, "ptqtp_gemv", packed, x, N, K, 1, group, y_dtype, out)


def ptqtp_gemm_small(packed, x, N: int, K: int, group: int = 128, y_dtype: int = PTQTP_F32, out=None):
    """y [M,N] for x fp16 [M,K], 1 <= M <= 64."""
    if x.dim() != 2 or x.shape[1] != K:
        raise PtqtpError(2, "ptqtp_gemm_small")
    return _forward(_load().ptqtp_gemm_small, "ptqtp_gemm_small", packed, x, N, K, x.shape[0], group, y_dtype, out)


def ptqtp_gemm(packed, x, N: int, K: int, group: int = 128, y_dtype: int = PTQTP_F32, out=None):
    """y [M,N] for x fp16 [M,K], any M up to 65536 (prefill uses the MFMA tile; y_dtype | PTQTP_FUSED_PLANES
    sums the planes in fp16 before the matrix pipe from 256 tokens on)."""
    if x.dim() != 2 or x.shape[1] != K:
        raise PtqtpError(2, "ptqtp_gemm")
    return _forward(_load().ptqtp_gemm, "ptqtp_gemm", packed, x, N, K, x.shape[0], group, y_dtype, out)


class _Linear(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("x", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64)]


class BatchPlan:
    """Device-side table for ptqtp_gemv_batch; keeps the tensors it names alive."""

    def __init__(self, plan: torch.Tensor, items: int, keep, tokens: int):
        self.plan, self.items, self._keep, self.tokens = plan, items, keep, tokens


def ptqtp_gemv_batch_plan(linears, group: int = 128, y_dtype: int = PTQTP_F32) -> BatchPlan:
    """linears: sequence of (packed, x, y, N, K) with torch tensors; x [M,K] (or [K]), y [M,N] (or [N]) of y_dtype."""
    ydt = torch.float32 if y_dtype == PTQTP_F32 else torch.float16
    n = len(linears)
    arr = (_Linear * max(n, 1))()
    tokens = None
    for i, (packed, x, y, N, K) in enumerate(linears):
        if N <= 0 or K <= 0 or x.numel() == 0 or x.numel() % K or y.numel() % N or x.numel() // K != y.numel() // N:
            raise PtqtpError(2, "ptqtp_gemv_batch_plan")
        _check_blob(packed, N, K, group, "ptqtp_gemv_batch_plan")
        tokens = x.numel() // K if tokens is None else min(tokens, x.numel() // K)
        arr[i] = _Linear(_dev(packed, torch.uint8, "packed"), _dev(x, torch.float16, "x"), _dev(y, ydt, "y"), N, K)
    lib = _load()
    nbytes = int(lib.ptqtp_batch_plan_bytes(arr, n, group))
    items = int(lib.ptqtp_batch_items(arr, n, group))
    if nbytes == 0 or items == 0:
        raise PtqtpError(2, "ptqtp_batch_plan_bytes")
    plan = torch.empty(nbytes, dtype=torch.uint8, device=linears[0][0].device)
    st = lib.ptqtp_gemv_batch_plan(arr, n, y_dtype, group, plan.data_ptr(), nbytes, _stream())
    if st:
        raise PtqtpError(st, "ptqtp_gemv_batch_plan")
    return BatchPlan(plan, items, [t for lin in linears for t in lin[:3]], tokens)


def ptqtp_gemm_batch(plan: BatchPlan, M: int) -> None:
    """Run a plan whose x tensors are [M, K] and y tensors [M, N]."""
    if M > plan.tokens:
        raise PtqtpError(2, "ptqtp_gemm_batch")
    st = _load().ptqtp_gemm_batch(plan.plan.data_ptr(), plan.items, int(M), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_gemm_batch")


def ptqtp_gemm_batch_fused(plan: BatchPlan, M: int) -> None:
    """ptqtp_gemm_batch with the planes summed in fp16 before the matrix pipe from 33 tokens on."""
    if M > plan.tokens:
        raise PtqtpError(2, "ptqtp_gemm_batch_fused")
    st = _load().ptqtp_gemm_batch_fused(plan.plan.data_ptr(), plan.items, int(M), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_gemm_batch_fused")


def ptqtp_gemv_batch(plan: BatchPlan) -> None:
    st = _load().ptqtp_gemv_batch(plan.plan.data_ptr(), plan.items, _stream())
    if st:
        raise PtqtpError(st, "ptqtp_gemv_batch")


def ptqtp_quantize(W: torch.Tensor, group: int = 128, max_iters: int = 50, eps: float = 1e-4):
    """PTQTP decomposition of W (fp16 [N,K] on the GPU) -> (T1, T2 int8 [N,K], a1, a2 fp16 [N,K/group], iters int32[1])."""
    N, K = W.shape
    lib = _load()
    nbytes = int(lib.ptqtp_quantize_workspace_bytes(N, K, group))
    if nbytes == 0:
        raise PtqtpError(2 if group == 128 else 3, "ptqtp_quantize_workspace_bytes")
    dev = W.device
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    T1 = torch.empty((N, K), dtype=torch.int8, device=dev)
    T2 = torch.empty((N, K), dtype=torch.int8, device=dev)
    a1 = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    a2 = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    iters = torch.zeros(1, dtype=torch.int32, device=dev)
    st = lib.ptqtp_quantize(_dev(W, torch.float16, "W"), N, K, group, int(max_iters), float(eps), T1.data_ptr(),
                            T2.data_ptr(), a1.data_ptr(), a2.data_ptr(), iters.data_ptr(), ws.data_ptr(), nbytes, _stream())
    if st:
        raise PtqtpError(st, "ptqtp_quantize")
    return T1, T2, a1, a2, iters


PTQTP_QUANTIZE_STATIC_BYTES = 16 * 1024 * 1024 + 256


def ptqtp_quantize_static(W: torch.Tensor, T1, T2, a1, a2, iters, group: int = 128, max_iters: int = 50,
                          eps: float = 1e-4) -> None:
    """ptqtp_quantize with the workspace in the library's static device array: the caller brings every output
    (T1, T2 int8 [N,K]; a1, a2 fp16 [N,K/group]; iters int32[1]) and nothing is allocated, here or in the library."""
    N, K = W.shape
    st = _load().ptqtp_quantize_static(_dev(W, torch.float16, "W"), N, K, group, int(max_iters), float(eps),
                                       _dev(T1, torch.int8, "T1"), _dev(T2, torch.int8, "T2"),
                                       _dev(a1, torch.float16, "a1"), _dev(a2, torch.float16, "a2"),
                                       _dev(iters, torch.int32, "iters"), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_quantize_static")


PTQTP_EPI_NONE, PTQTP_EPI_SWIGLU = 0, 1


class _Stage(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("x", ctypes.c_void_p), ("y", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("epilogue", ctypes.c_int32), ("y_dtype", ctypes.c_int32),
                ("level", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class ChainPlan:
    """Device-side table for ptqtp_chain_run; keeps the host stage array and the tensors it names alive."""

    def __init__(self, plan: torch.Tensor, arr, count: int, group: int, keep, tokens: int):
        self.plan, self.arr, self.count, self.group, self._keep, self.tokens = plan, arr, count, group, keep, tokens


def ptqtp_chain_plan(stages, group: int = 128) -> ChainPlan:
    """stages: sequence of dicts with packed, x, y, N, K and optionally residual (tensor or None),
    epilogue (PTQTP_EPI_*), level (int), fused_planes (bool: honoured by ptqtp_chain_run_batch from 256 tokens on);
    y's torch dtype (float32 / float16) gives y_dtype."""
    n = len(stages)
    arr = (_Stage * max(n, 1))()
    keep = []
    tokens = None
    for i, s in enumerate(stages):
        y = s["y"]
        if y.dtype not in (torch.float32, torch.float16):
            raise PtqtpError(5, "ptqtp_chain_plan")
        res = s.get("residual")
        # the buffers must hold what the stage reads and writes: m tokens of K inputs, m x n_out outputs
        N, K = int(s["N"]), int(s["K"])
        n_out = N // 2 if int(s.get("epilogue", PTQTP_EPI_NONE)) == PTQTP_EPI_SWIGLU else N
        if N <= 0 or K <= 0 or n_out <= 0:
            raise PtqtpError(2, "ptqtp_chain_plan")
        m = min(s["x"].numel() // K, y.numel() // n_out, *([res.numel() // n_out] if res is not None else []))
        if m < 1:
            raise PtqtpError(2, "ptqtp_chain_plan")
        _check_blob(s["packed"], N, K, group, "ptqtp_chain_plan")
        tokens = m if tokens is None else min(tokens, m)
        arr[i] = _Stage(_dev(s["packed"], torch.uint8, "packed"), _dev(s["x"], torch.float16, "x"), _dev(y, y.dtype, "y"),
                        _dev(res, torch.float16, "residual") if res is not None else None,
                        int(s["N"]), int(s["K"]), int(s.get("epilogue", PTQTP_EPI_NONE)),
                        (PTQTP_F32 if y.dtype == torch.float32 else PTQTP_F16) | (PTQTP_FUSED_PLANES if s.get("fused_planes") else 0),
                        int(s.get("level", i)), 0)
        keep += [s["packed"], s["x"], y, res]
    lib = _load()
    nbytes = int(lib.ptqtp_chain_plan_bytes(arr, n, group))
    if nbytes == 0:
        raise PtqtpError(2, "ptqtp_chain_plan_bytes")
    plan = torch.empty(nbytes, dtype=torch.uint8, device=stages[0]["packed"].device)
    st = lib.ptqtp_chain_plan(arr, n, group, plan.data_ptr(), nbytes, _stream())
    if st:
        raise PtqtpError(st, "ptqtp_chain_plan")
    return ChainPlan(plan, arr, n, group, keep, tokens)


def ptqtp_chain_run(plan: ChainPlan) -> None:
    """One token: one launch per level on the current stream."""
    st = _load().ptqtp_chain_run(plan.arr, plan.count, plan.group, plan.plan.data_ptr(), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_chain_run")


def ptqtp_chain_run_batch(plan: ChainPlan, M: int) -> None:
    """The chain at M tokens per stage (x [M,K], y / residual [M,n_out]); one launch per stage.  M may not exceed
    what the smallest buffer named in the plan holds."""
    if M > plan.tokens:
        raise PtqtpError(2, "ptqtp_chain_run_batch")
    st = _load().ptqtp_chain_run_batch(plan.arr, plan.count, plan.group, int(M), _stream())
    if st:
        raise PtqtpError(st, "ptqtp_chain_run_batch")
