"""fp64 CPU oracle for the dual trit-plane linear layer -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the HIP library and never imports it.

Two independent evaluations of the layer (paper, Eq. 1-2 with the group-wise
scales of paragraph "Batch Processing"):

* forward()       -- C, scale-after-plane-product order of Eq. 1 (ptqtp_oracle.c)
* forward_dense() -- numpy, "dequantization" order: rebuild W^ then a library
                     matmul (Sec. "Inference Efficiency" names both orders)
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ptqtp_oracle.c")
_SRC_Q = os.path.join(_HERE, "ptqtp_quantizer_oracle.c")
_SRC_B = os.path.join(_HERE, "ptqtp_block_oracle.c")
_LIB = os.path.join(_HERE, "libptqtp_oracle.so")
_lib = None

OK, ERR_SHAPE, ERR_TRIT, ERR_CODE = 0, 1, 2, 3


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__({1: "bad shape", 2: "trit outside {-1,0,1}", 3: "unused 2-bit code"}.get(code, str(code)))
        self.code = code


def build(force: bool = False) -> str:
    """Compile ptqtp_oracle.c with gcc (-O2, OpenMP for the row loop)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_Q), os.path.getmtime(_SRC_B))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off", "-o", tmp, _SRC, _SRC_Q, _SRC_B, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(lib):
    """Declare the C signatures on a loaded library (the built one, or a deliberately broken copy in the mutation tests)."""
    p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.ptqtp_oracle_half_to_double.restype = ctypes.c_double
    lib.ptqtp_oracle_half_to_double.argtypes = [ctypes.c_uint16]
    lib.ptqtp_oracle_forward_f64x.restype = i32
    lib.ptqtp_oracle_forward_f64x.argtypes = [p, p, p, p, p, i64, i64, i64, i64, p, p, i32]
    lib.ptqtp_oracle_forward.restype = i32
    lib.ptqtp_oracle_forward.argtypes = [p, p, p, p, p, p, i64, i64, i64, i64, p, p, i32]
    lib.ptqtp_oracle_pack_canonical.restype = i32
    lib.ptqtp_oracle_pack_canonical.argtypes = [p, i64, i64, p]
    lib.ptqtp_oracle_unpack_canonical.restype = i32
    lib.ptqtp_oracle_unpack_canonical.argtypes = [p, i64, i64, p]
    lib.ptqtp_oracle_model_bits.restype = i64
    lib.ptqtp_oracle_model_bits.argtypes = [i64, i64, i64]
    lib.ptqtp_oracle_quantize.restype = i32
    lib.ptqtp_oracle_quantize.argtypes = [p, i64, i64, i64, i32, ctypes.c_double, p, p, p, p, p, p, p, p]
    lib.ptqtp_oracle_double_to_half_bits.restype = ctypes.c_uint16
    lib.ptqtp_oracle_double_to_half_bits.argtypes = [ctypes.c_double]
    lib.ptqtp_oracle_silu.restype = ctypes.c_double
    lib.ptqtp_oracle_silu.argtypes = [ctypes.c_double]
    lib.ptqtp_oracle_swiglu.restype = i32
    lib.ptqtp_oracle_swiglu.argtypes = [p, i64, i64, p]
    lib.ptqtp_oracle_residual_add.restype = i32
    lib.ptqtp_oracle_residual_add.argtypes = [p, p, i64, p]
    lib.ptqtp_oracle_round_half.restype = ctypes.c_double
    lib.ptqtp_oracle_round_half.argtypes = [ctypes.c_double]
    lib.ptqtp_oracle_round_half_array.restype = None
    lib.ptqtp_oracle_round_half_array.argtypes = [p, i64, p]
    return lib


_LIB_SAN = os.path.join(_HERE, "libptqtp_oracle_san.so")
SANITIZED_ENV = "PTQTP_ORACLE_SANITIZED"      # set to 1: load the AddressSanitizer/UBSan build (see build_sanitized)


def build_sanitized() -> str:
    """The same sources with -fsanitize=address,undefined (host code only, gcc): memory errors and undefined
    behaviour in the oracle abort the process that loads it.  The process must have the sanitizer runtime
    preloaded (sanitizer_preload()); tests/test_oracle_sanitized.py runs the pin tests that way."""
    tmp = _LIB_SAN + f".tmp{os.getpid()}"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                           "-o", tmp, _SRC, _SRC_Q, _SRC_B, "-lm"])
    os.replace(tmp, _LIB_SAN)
    return _LIB_SAN


def sanitizer_preload() -> str:
    """Path of gcc's AddressSanitizer runtime, for LD_PRELOAD of a process that loads the sanitized build."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


def _load():
    global _lib
    if _lib is None:
        if os.environ.get(SANITIZED_ENV) == "1":
            _lib = _bind(ctypes.CDLL(_LIB_SAN if os.path.exists(_LIB_SAN) else build_sanitized()))
        else:
            _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def half_to_double(bits: int) -> float:
    return _load().ptqtp_oracle_half_to_double(int(bits) & 0xFFFF)


def forward(T1, T2, a1, a2, x, group: int = 128, threads: int = 1, want_bound: bool = True):
    """y, B = forward(...).  T int8 [N,K]; a float16 [N,K/group]; x float16 [M,K]
    (or float64 [M,K] for linearity checks).  Returns float64 [M,N] arrays."""
    lib = _load()
    T1, pT1 = _c(T1, np.int8)
    T2, pT2 = _c(T2, np.int8)
    N, K = T1.shape
    if T2.shape != (N, K):
        raise OracleError(ERR_SHAPE)
    a1 = np.ascontiguousarray(a1)
    a2 = np.ascontiguousarray(a2)
    if a1.dtype != np.float16 or a2.dtype != np.float16:
        raise TypeError("scales must be float16")
    if K % group or a1.shape != (N, K // group) or a2.shape != (N, K // group):
        raise OracleError(ERR_SHAPE)
    x = np.ascontiguousarray(x)
    if x.ndim == 1:
        x = x[None, :]
    M = x.shape[0]
    if x.shape[1] != K:
        raise OracleError(ERR_SHAPE)
    y = np.empty((M, N), dtype=np.float64)
    b = np.empty((M, N), dtype=np.float64) if want_bound else None
    pb = b.ctypes.data_as(ctypes.c_void_p) if want_bound else None
    pa1 = a1.view(np.uint16).ctypes.data_as(ctypes.c_void_p)
    pa2 = a2.view(np.uint16).ctypes.data_as(ctypes.c_void_p)
    py = y.ctypes.data_as(ctypes.c_void_p)
    if x.dtype == np.float16:
        scratch = np.empty((M, K), dtype=np.float64)
        rc = lib.ptqtp_oracle_forward(pT1, pT2, pa1, pa2, x.view(np.uint16).ctypes.data_as(ctypes.c_void_p),
                                      scratch.ctypes.data_as(ctypes.c_void_p), M, N, K, group, py, pb, threads)
    elif x.dtype == np.float64:
        rc = lib.ptqtp_oracle_forward_f64x(pT1, pT2, pa1, pa2, x.ctypes.data_as(ctypes.c_void_p),
                                           M, N, K, group, py, pb, threads)
    else:
        raise TypeError("x must be float16 or float64")
    if rc != OK:
        raise OracleError(rc)
    return y, b


def reconstruct_dense(T1, T2, a1, a2, group: int = 128) -> np.ndarray:
    """W^ = alpha1 (.) T1 + alpha2 (.) T2 as float64 [N,K] (Eq. 2, group-wise scales).
    Exact: each entry is a sum of two binary16-valued numbers."""
    T1 = np.asarray(T1, dtype=np.float64)
    T2 = np.asarray(T2, dtype=np.float64)
    A1 = np.repeat(np.asarray(a1, dtype=np.float64), group, axis=1)
    A2 = np.repeat(np.asarray(a2, dtype=np.float64), group, axis=1)
    return A1 * T1 + A2 * T2


def forward_dense(T1, T2, a1, a2, x, group: int = 128) -> np.ndarray:
    """Second, independent evaluation: rebuild W^ and use the library matmul."""
    W = reconstruct_dense(T1, T2, a1, a2, group)
    x = np.asarray(x, dtype=np.float64)
    if x.ndim == 1:
        x = x[None, :]
    return x @ W.T


def forward_fused(T1, T2, a1, a2, x, group: int = 128):
    """The "dequantization" forward with the weight held in binary16 (Sec. "Inference Efficiency"
    names a dequantization forward beside the dequantization-free one): W16 = each entry of
    W^ = alpha1 T1 + alpha2 T2 rounded ONCE to binary16, then y = x W16^T in float64.
    Returns (y, B16) with B16 = |x| |W16|^T, both float64 [M, N]."""
    W16 = round_half(reconstruct_dense(T1, T2, a1, a2, group))
    x = np.asarray(x, dtype=np.float64)
    if x.ndim == 1:
        x = x[None, :]
    return x @ W16.T, np.abs(x) @ np.abs(W16).T


def pack_canonical(T) -> np.ndarray:
    T, pT = _c(T, np.int8)
    N, K = T.shape
    out = np.empty((N, K // 4), dtype=np.uint8)
    rc = _load().ptqtp_oracle_pack_canonical(pT, N, K, out.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise OracleError(rc)
    return out


def unpack_canonical(packed, K: int) -> np.ndarray:
    packed, pp = _c(packed, np.uint8)
    N = packed.shape[0]
    T = np.empty((N, K), dtype=np.int8)
    rc = _load().ptqtp_oracle_unpack_canonical(pp, N, K, T.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise OracleError(rc)
    return T


def model_bits(n: int, d: int, group: int = 128) -> int:
    return int(_load().ptqtp_oracle_model_bits(n, d, group))


def double_to_half_bits(f: float) -> int:
    return int(_load().ptqtp_oracle_double_to_half_bits(float(f)))


def quantize(W, group: int = 128, max_iters: int = 50, eps: float = 1e-4) -> dict:
    """PTQTP decomposition of W (float16 [N,K]) -> dict(T1, T2 int8 [N,K]; a1, a2 float16 [N,K/group];
    a1_f64, a2_f64 float64 (the iteration's alpha); lam float64; iters int).  See ptqtp_quantizer_oracle.c."""
    W = np.ascontiguousarray(W)
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a float16 matrix")
    N, K = W.shape
    if K % group:
        raise OracleError(ERR_SHAPE)
    ng = K // group
    out = {"T1": np.empty((N, K), np.int8), "T2": np.empty((N, K), np.int8),
           "a1_f64": np.empty((N, ng), np.float64), "a2_f64": np.empty((N, ng), np.float64),
           "a1": np.empty((N, ng), np.float16), "a2": np.empty((N, ng), np.float16),
           "lam": np.empty((N, ng), np.float64)}
    iters = ctypes.c_int(0)
    ptr = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    rc = _load().ptqtp_oracle_quantize(ptr(W.view(np.uint16)), N, K, group, int(max_iters), float(eps),
                                       ptr(out["T1"]), ptr(out["T2"]), ptr(out["a1_f64"]), ptr(out["a2_f64"]),
                                       ptr(out["a1"].view(np.uint16)), ptr(out["a2"].view(np.uint16)),
                                       ptr(out["lam"]), ctypes.byref(iters))
    if rc != OK:
        raise OracleError(rc)
    out["iters"] = iters.value
    return out


# ---------------------------------------------------------------- decoder-block steps around the linears
SILU_LIPSCHITZ = 1.1      # sup |silu'(z)| = 1.0998...


def silu(z: float) -> float:
    return _load().ptqtp_oracle_silu(float(z))


def swiglu(y, I: int) -> np.ndarray:
    """h[m,i] = silu(y[m,i]) * y[m,I+i] for y float64 [M, 2I] (gate rows first, then up rows)."""
    y, py = _c(y, np.float64)
    M = y.shape[0]
    if y.ndim != 2 or y.shape[1] != 2 * I:
        raise OracleError(ERR_SHAPE)
    h = np.empty((M, I), dtype=np.float64)
    rc = _load().ptqtp_oracle_swiglu(py, M, I, h.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise OracleError(rc)
    return h


def residual_add(y, r16) -> np.ndarray:
    """y + r with r float16 (widened exactly), float64 result of y's shape."""
    y, py = _c(y, np.float64)
    r16 = np.ascontiguousarray(r16)
    if r16.dtype != np.float16 or r16.shape != y.shape:
        raise OracleError(ERR_SHAPE)
    out = np.empty_like(y)
    rc = _load().ptqtp_oracle_residual_add(py, r16.view(np.uint16).ctypes.data_as(ctypes.c_void_p), y.size,
                                           out.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise OracleError(rc)
    return out


def round_half(v) -> np.ndarray:
    """Each float64 rounded once to the nearest binary16 (ties to even), returned as float64."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty_like(v)
    _load().ptqtp_oracle_round_half_array(v.ctypes.data_as(ctypes.c_void_p), v.size, out.ctypes.data_as(ctypes.c_void_p))
    return out


def stage(lin: dict, x, epilogue: str = "none", residual=None, threads: int = 1) -> dict:
    """One stage of a decode chain in float64: the linear, then the epilogue.

    epilogue "none":   out = y (+ residual)
             "swiglu": lin stacks gate rows over up rows (N = 2I); out = silu(gate) * up (+ residual)
    Returns {"out": exact float64 value, "err": E} where E[m,n] bounds the change of `out` when every
    entry of the linear's result moves by at most its L1 bound B (first order: for swiglu
    E = 1.1 * B_gate * |up| + |silu(gate)| * B_up).  A result with relative error tau in the
    linear is off by at most tau * E (+ tau^2 * 1.1 * B_gate * B_up for swiglu)."""
    y, B = forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, group=lin.get("group", 128), threads=threads)
    if epilogue == "none":
        out, err, err2 = y, B, np.zeros_like(B)
    elif epilogue == "swiglu":
        I = y.shape[1] // 2
        out = swiglu(y, I)
        g, u = y[:, :I], y[:, I:]
        sg = np.array([silu(t) for t in g.ravel()]).reshape(g.shape)
        err = SILU_LIPSCHITZ * B[:, :I] * np.abs(u) + np.abs(sg) * B[:, I:]
        err2 = SILU_LIPSCHITZ * B[:, :I] * B[:, I:]
    else:
        raise ValueError(epilogue)
    if residual is not None:
        out = residual_add(out, residual)
    return {"out": out, "err": err, "err2": err2}
