"""ctypes face of the CPU oracle (oracle/omc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "omc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
# tests/test_oracle_mutations.py points this at deliberately broken builds to show that the pins notice
_LIB_OVERRIDE = os.environ.get("OMC_ORACLE_LIBRARY")

GCC_FLAGS = ["-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when force, else when stale or missing)."""
    if _LIB_OVERRIDE and not force:
        return _LIB_OVERRIDE
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", *GCC_FLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Fmt(C.Structure):
    _fields_ = [("exp_bits", C.c_int32), ("man_bits", C.c_int32), ("bias", C.c_int32)]


class _Opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("one_minus_beta1", C.c_float), ("one_minus_beta2", C.c_float),
                ("bias_corr1", C.c_float), ("bias_corr2", C.c_float)]


class _Var(C.Structure):
    _fields_ = [("data_offset", C.c_uint64), ("aux_offset", C.c_uint64), ("n", C.c_uint64),
                ("fmt", _Fmt), ("quantized", C.c_int32), ("use_pvt", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.orc_format_bits.restype = C.c_int
        L.orc_format_bits.argtypes = [_Fmt]
        L.orc_format_max.restype = C.c_double
        L.orc_format_max.argtypes = [_Fmt]
        L.orc_decode_value.restype = C.c_double
        L.orc_decode_value.argtypes = [C.c_uint32, _Fmt]
        L.orc_decode.restype = C.c_float
        L.orc_decode.argtypes = [C.c_uint32, _Fmt]
        L.orc_encode.restype = C.c_uint32
        L.orc_encode.argtypes = [C.c_float, _Fmt]
        L.orc_encode_array.restype = None
        L.orc_encode_array.argtypes = [C.c_void_p, C.c_uint64, _Fmt, C.c_void_p]
        L.orc_decode_array.restype = None
        L.orc_decode_array.argtypes = [C.c_void_p, C.c_uint64, _Fmt, C.c_void_p]
        L.orc_packed_bytes.restype = C.c_uint64
        L.orc_packed_bytes.argtypes = [C.c_uint64, C.c_int]
        L.orc_pack.restype = None
        L.orc_pack.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.orc_unpack.restype = None
        L.orc_unpack.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.orc_exact_sum.restype = C.c_double
        L.orc_exact_sum.argtypes = [C.c_void_p, C.c_uint64]
        L.orc_pvt_fit.restype = None
        L.orc_pvt_fit.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.orc_compress.restype = C.c_int
        L.orc_compress.argtypes = [C.c_void_p, C.c_uint64, _Fmt, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_decompress.restype = C.c_int
        L.orc_decompress.argtypes = [C.c_void_p, C.c_uint64, _Fmt, C.c_void_p, C.c_void_p]
        L.orc_step_quantized.restype = C.c_int
        L.orc_step_quantized.argtypes = [C.c_void_p, C.c_uint64, _Fmt, C.c_int, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_Opt)]
        L.orc_step_fp32.restype = C.c_int
        L.orc_step_fp32.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.POINTER(_Opt)]
        L.orc_step_varset.restype = C.c_int
        L.orc_step_varset.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.POINTER(_Opt), C.c_int]
        L.orc_dequant_gemm_dx.restype = C.c_int
        L.orc_dequant_gemm_dx.argtypes = [C.c_void_p, C.c_void_p, _Fmt, C.c_void_p, C.c_void_p,
                                          C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                          C.c_int]
        L.orc_gemm_dw.restype = C.c_int
        L.orc_gemm_dw.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                                  C.c_uint32, C.c_uint32, C.c_int]
        L.orc_mean_f32.restype = C.c_int
        L.orc_mean_f32.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_void_p]
        L.orc_dequant_gemm.restype = C.c_int
        L.orc_dequant_gemm.argtypes = [C.c_void_p, C.c_void_p, _Fmt, C.c_void_p, C.c_void_p,
                                       C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                       C.c_int]
    return _lib


# --------------------------------------------------------------------------- formats
@dataclass(frozen=True)
class Format:
    """SxEyMz with x = 1.  bias None means 2^(E-1)-1."""
    exp_bits: int
    man_bits: int
    bias: int | None = None

    @property
    def resolved_bias(self) -> int:
        return (1 << (self.exp_bits - 1)) - 1 if self.bias is None else self.bias

    @property
    def bits(self) -> int:
        return 1 + self.exp_bits + self.man_bits

    def c(self) -> _Fmt:
        return _Fmt(self.exp_bits, self.man_bits, self.resolved_bias)

    @property
    def max(self) -> float:
        return lib().orc_format_max(self.c())


@dataclass
class Opt:
    """Optimizer hyper-parameters; the derived fp32 constants are rounded once from fp64."""
    kind: int = 0                 # 0 SGD, 1 momentum, 2 Adam
    lr: float = 0.01
    momentum: float = 0.9
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    t: int = 1                    # Adam step number (1-based)

    def c(self) -> _Opt:
        f32 = lambda x: float(np.float32(x))
        return _Opt(self.kind, f32(self.lr), f32(self.momentum), f32(self.beta1), f32(self.beta2),
                    f32(self.eps), f32(1.0 - self.beta1), f32(1.0 - self.beta2),
                    f32(1.0 - self.beta1 ** self.t), f32(1.0 - self.beta2 ** self.t))


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


# --------------------------------------------------------------------------- scalar / array codec
def encode(values, fmt: Format) -> np.ndarray:
    v = _f32(values).ravel()
    out = np.empty(v.size, dtype=np.uint32)
    lib().orc_encode_array(_p(v), v.size, fmt.c(), _p(out))
    return out


def decode(codes, fmt: Format) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint32).ravel()
    out = np.empty(c.size, dtype=np.float32)
    lib().orc_decode_array(_p(c), c.size, fmt.c(), _p(out))
    return out


def decode_value(code: int, fmt: Format) -> float:
    return lib().orc_decode_value(int(code), fmt.c())


def packed_bytes(n: int, bits: int) -> int:
    return int(lib().orc_packed_bytes(n, bits))


def pack(codes, bits: int) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint32).ravel()
    out = np.empty(packed_bytes(c.size, bits), dtype=np.uint8)
    lib().orc_pack(_p(c), c.size, bits, _p(out))
    return out


def unpack(packed, n: int, bits: int) -> np.ndarray:
    b = np.ascontiguousarray(packed, dtype=np.uint8)
    assert b.size >= packed_bytes(n, bits)
    out = np.empty(n, dtype=np.uint32)
    lib().orc_unpack(_p(b), n, bits, _p(out))
    return out


def exact_sum(x) -> float:
    x = np.ascontiguousarray(x, dtype=np.float64).ravel()
    return lib().orc_exact_sum(_p(x), x.size)


# --------------------------------------------------------------------------- per-variable ops
def pvt_fit(V, Vt):
    V = _f32(V).ravel()
    Vt = _f32(Vt).ravel()
    assert V.size == Vt.size and V.size > 0
    s = np.empty(1, dtype=np.float32)
    b = np.empty(1, dtype=np.float32)
    lib().orc_pvt_fit(_p(V), _p(Vt), V.size, _p(s), _p(b))
    return s[0], b[0]


def compress(V, fmt: Format, use_pvt: bool = True):
    """-> (packed uint8 array, sb float32[2])"""
    V = _f32(V).ravel()
    packed = np.empty(packed_bytes(V.size, fmt.bits), dtype=np.uint8)
    sb = np.empty(2, dtype=np.float32)
    rc = lib().orc_compress(_p(V), V.size, fmt.c(), int(use_pvt), _p(packed), _p(sb))
    if rc:
        raise ValueError(f"orc_compress failed ({rc})")
    return packed, sb


def decompress(packed, n: int, fmt: Format, sb=None) -> np.ndarray:
    b = np.ascontiguousarray(packed, dtype=np.uint8)
    assert b.size >= packed_bytes(n, fmt.bits)
    out = np.empty(n, dtype=np.float32)
    sbp = None if sb is None else np.ascontiguousarray(sb, dtype=np.float32)
    rc = lib().orc_decompress(_p(b), n, fmt.c(), _p(sbp), _p(out))
    if rc:
        raise ValueError(f"orc_decompress failed ({rc})")
    return out


def step_quantized(packed, n, fmt: Format, sb, g, st0, st1, opt: Opt, use_pvt=True):
    """In place on packed / sb / st0 / st1 (numpy arrays owned by the caller)."""
    assert packed.dtype == np.uint8 and packed.flags.c_contiguous
    assert sb.dtype == np.float32 and sb.size == 2
    g = _f32(g)
    o = opt.c()
    rc = lib().orc_step_quantized(_p(packed), n, fmt.c(), int(use_pvt), _p(sb), _p(g),
                                  _p(st0), _p(st1), C.byref(o))
    if rc:
        raise ValueError(f"orc_step_quantized failed ({rc})")


def step_fp32(W, g, st0, st1, opt: Opt):
    assert W.dtype == np.float32 and W.flags.c_contiguous
    g = _f32(g)
    o = opt.c()
    lib().orc_step_fp32(_p(W), W.size, _p(g), _p(st0), _p(st1), C.byref(o))


# --------------------------------------------------------------------------- variable sets
def make_var_table(vars_):
    """vars_: iterable of dicts(data_offset, aux_offset, n, fmt: Format|None, quantized, use_pvt)."""
    vars_ = list(vars_)
    tab = (_Var * len(vars_))()
    for i, v in enumerate(vars_):
        fmt = v["fmt"].c() if v.get("fmt") is not None else _Fmt(8, 23, 127)
        tab[i] = _Var(v["data_offset"], v["aux_offset"], v["n"], fmt,
                      int(v["quantized"]), int(v.get("use_pvt", True)))
    return tab


def step_varset(arena, var_table, sb_table, grads, state0, state1, opt: Opt, threads: int = 1):
    """One iteration over a whole variable set, in place (arena uint8, sb_table float32 [nvars,2])."""
    assert arena.dtype == np.uint8 and arena.flags.c_contiguous
    assert sb_table.dtype == np.float32 and sb_table.flags.c_contiguous
    assert grads.dtype == np.float32 and grads.flags.c_contiguous
    o = opt.c()
    rc = lib().orc_step_varset(_p(arena), C.cast(var_table, C.c_void_p), len(var_table),
                               _p(sb_table), _p(grads), _p(state0), _p(state1), C.byref(o),
                               int(threads))
    if rc:
        raise ValueError(f"orc_step_varset failed ({rc})")


# --------------------------------------------------------------------------- forward GEMM
def dequant_gemm(A_bf16_bits, packed, fmt: Format, sb, M, N, K, rows=None, threads: int = 1):
    """C[rows] = A[rows] @ decompress(packed) in double.  A as uint16 bf16 bit patterns [M, K]."""
    A = np.ascontiguousarray(A_bf16_bits, dtype=np.uint16)
    assert A.size == M * K
    r0, r1 = (0, M) if rows is None else rows
    out = np.empty((r1 - r0, N), dtype=np.float64)
    sbp = None if sb is None else np.ascontiguousarray(sb, dtype=np.float32)
    b = np.ascontiguousarray(packed, dtype=np.uint8)
    rc = lib().orc_dequant_gemm(_p(A), _p(b), fmt.c(), _p(sbp), _p(out), M, N, K, r0, r1,
                                int(threads))
    if rc:
        raise ValueError(f"orc_dequant_gemm failed ({rc})")
    return out


def dequant_gemm_dx(dY_bf16_bits, packed, fmt: Format, sb, M, N, K, rows=None, threads: int = 1):
    """dX[rows] = dY[rows] @ decompress(packed)^T in double; the weights are [K, N], dY is uint16 bf16 bits [M, N]."""
    dY = np.ascontiguousarray(dY_bf16_bits, dtype=np.uint16)
    assert dY.size == M * N
    r0, r1 = (0, M) if rows is None else rows
    out = np.empty((r1 - r0, K), dtype=np.float64)
    sbp = None if sb is None else np.ascontiguousarray(sb, dtype=np.float32)
    b = np.ascontiguousarray(packed, dtype=np.uint8)
    rc = lib().orc_dequant_gemm_dx(_p(dY), _p(b), fmt.c(), _p(sbp), _p(out), M, N, K, r0, r1, int(threads))
    if rc:
        raise ValueError(f"orc_dequant_gemm_dx failed ({rc})")
    return out


def gemm_dw(X_bf16_bits, dY_bf16_bits, M, N, K, rows=None, threads: int = 1):
    """dW[rows] = (X^T @ dY)[rows] in double; X is [M, K], dY is [M, N], both uint16 bf16 bits; rows index k."""
    X = np.ascontiguousarray(X_bf16_bits, dtype=np.uint16)
    dY = np.ascontiguousarray(dY_bf16_bits, dtype=np.uint16)
    assert X.size == M * K and dY.size == M * N
    r0, r1 = (0, K) if rows is None else rows
    out = np.empty((r1 - r0, N), dtype=np.float64)
    rc = lib().orc_gemm_dw(_p(X), _p(dY), _p(out), M, N, K, r0, r1, int(threads))
    if rc:
        raise ValueError(f"orc_gemm_dw failed ({rc})")
    return out


# --------------------------------------------------------------------------- server aggregation
def aggregate_mean(replica_values) -> np.ndarray:
    """Equal-weight federated average of R decompressed copies of one variable (fp32, clients in
    index order, one rounding per operation).  replica_values: sequence of R float32 arrays."""
    vs = [_f32(v) for v in replica_values]
    n = vs[0].size
    assert all(v.size == n for v in vs)
    ptrs = (C.c_void_p * len(vs))(*[v.ctypes.data for v in vs])
    out = np.empty(n, dtype=np.float32)
    rc = lib().orc_mean_f32(ptrs, len(vs), n, _p(out))
    if rc:
        raise ValueError(f"orc_mean_f32 failed ({rc})")
    return out
