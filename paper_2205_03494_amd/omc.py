"""Thin binding over libomc (include/omc.h): argument marshalling only.

Every step of the method runs inside the library's HIP kernels; PyTorch appears here only as the
owner of device memory and of the stream.  The functions carry the C names.  Tensors must be
contiguous and live on the GPU; nothing here falls back to a CPU path, and importing this module
fails loudly when the shared library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("OMC_LIBRARY_PATH", os.path.join(_HERE, "libomc.so"))  # override: another build of libomc

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `make -C paper_2205_03494_amd/csrc` "
        "(or __graft_entry__.build()); there is no fallback implementation")

_lib = C.CDLL(LIB_PATH)

OMC_OK = 0
OMC_VAR_QUANTIZED = 1
OMC_VAR_NO_PVT = 2
OMC_SGD, OMC_MOMENTUM, OMC_ADAM = 0, 1, 2
OMC_OPT_STREAM_CODES = 1
OMC_OPT_KEEP_CODES = 2
OMC_BIAS_DEFAULT = -1


class omc_format(C.Structure):
    _fields_ = [("exp_bits", C.c_uint8), ("man_bits", C.c_uint8), ("exp_bias", C.c_int16)]


class omc_var(C.Structure):
    _fields_ = [("data_offset", C.c_uint64), ("aux_offset", C.c_uint64), ("n", C.c_uint64),
                ("fmt", omc_format), ("flags", C.c_uint32)]


class omc_opt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("one_minus_beta1", C.c_float), ("one_minus_beta2", C.c_float),
                ("bias_corr1", C.c_float), ("bias_corr2", C.c_float), ("flags", C.c_uint32)]


def _sig(name, restype, *argtypes):
    fn = getattr(_lib, name)
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


_vp = C.c_void_p
_status_string = _sig("omc_status_string", C.c_char_p, C.c_int)
_format_validate = _sig("omc_format_validate", C.c_int, omc_format)
_format_bits = _sig("omc_format_bits", C.c_uint32, omc_format)
_format_max = _sig("omc_format_max", C.c_float, omc_format)
_packed_bytes = _sig("omc_packed_bytes", C.c_size_t, omc_format, C.c_uint64)
_compress_ws = _sig("omc_compress_workspace_bytes", C.c_size_t, C.c_uint64)
_compress = _sig("omc_compress", C.c_int, _vp, C.c_uint64, omc_format, C.c_int, _vp, _vp, _vp, C.c_size_t, _vp)
_compress_noalloc = _sig("omc_compress_noalloc", C.c_int, _vp, C.c_uint64, omc_format, C.c_int, _vp, _vp, _vp)
_compress_noalloc_max = _sig("omc_compress_noalloc_max_elems", C.c_uint64)
_decompress = _sig("omc_decompress", C.c_int, _vp, C.c_uint64, omc_format, _vp, _vp, _vp)
_plan_bytes = _sig("omc_plan_bytes", C.c_size_t, _vp, C.c_uint32)
_plan_build = _sig("omc_plan_build", C.c_int, _vp, C.c_uint32, _vp, C.c_size_t)
_plan_ws = _sig("omc_plan_workspace_bytes", C.c_size_t, _vp)
_workspace_bytes = _sig("omc_workspace_bytes", C.c_size_t, _vp, C.c_uint32)
_plan_arena = _sig("omc_plan_arena_bytes", C.c_size_t, _vp)
_plan_aux = _sig("omc_plan_aux_elems", C.c_uint64, _vp)
_step = _sig("omc_step_update_recompress", C.c_int, _vp, C.c_size_t, _vp, _vp, _vp, _vp, _vp, _vp,
             C.c_uint64, C.POINTER(omc_opt), _vp, C.c_size_t, _vp)
_plan_launches = _sig("omc_plan_launches", C.c_uint32, _vp)
_step_ev = _sig("omc_step_update_recompress_events", C.c_int, _vp, C.c_size_t, _vp, _vp, _vp, _vp, _vp,
                _vp, C.c_uint64, C.POINTER(omc_opt), _vp, C.c_size_t, _vp, _vp, C.c_uint32)
_compress_set = _sig("omc_compress_set", C.c_int, _vp, C.c_uint64, _vp, _vp, _vp, C.c_size_t, _vp, _vp, C.c_size_t, _vp)
_decompress_set = _sig("omc_decompress_set", C.c_int, _vp, C.c_size_t, _vp, _vp, _vp, _vp, C.c_uint64, _vp)
_plan_transport = _sig("omc_plan_transport_bytes", C.c_uint64, _vp)
_rs_bytes = _sig("omc_reselect_plan_bytes", C.c_size_t, _vp, _vp)
_rs_build = _sig("omc_reselect_plan_build", C.c_int, _vp, _vp, _vp, C.c_size_t)
_rs_ws = _sig("omc_reselect_workspace_bytes", C.c_size_t, _vp)
_rs_alg = _sig("omc_reselect_algorithmic_bytes", C.c_uint64, _vp)
_reselect = _sig("omc_reselect", C.c_int, _vp, _vp, _vp, C.c_size_t, _vp, _vp, C.c_size_t, _vp, _vp, C.c_size_t, _vp)
_tr_meta = _sig("omc_transport_meta_bytes", C.c_size_t, C.c_uint32)
_tr_bytes = _sig("omc_transport_bytes", C.c_uint64, _vp)
_tr_pack = _sig("omc_transport_pack", C.c_int, _vp, _vp, _vp, C.c_size_t, _vp, _vp, C.c_size_t, _vp)
_tr_open = _sig("omc_transport_open", C.c_int, _vp, C.c_size_t, C.c_uint64, _vp, C.c_uint32, C.POINTER(C.c_uint32),
                C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64))
_agg_bytes = _sig("omc_aggregate_plan_bytes", C.c_size_t, _vp, C.c_uint32)
_agg_build = _sig("omc_aggregate_plan_build", C.c_int, _vp, C.c_uint32, _vp, C.c_size_t)
_agg_mean = _sig("omc_aggregate_mean", C.c_int, _vp, _vp, _vp, _vp, _vp, _vp, C.c_uint64, _vp)
_gemm_ws = _sig("omc_dequant_gemm_workspace_bytes", C.c_size_t, C.c_uint32)
_gemm = _sig("omc_dequant_gemm", C.c_int, _vp, _vp, omc_format, _vp, _vp, C.c_uint32, C.c_uint32,
             C.c_uint32, _vp, C.c_size_t, _vp)
_dw_ws = _sig("omc_dw_update_workspace_bytes", C.c_size_t, omc_format, C.c_uint32, C.c_uint32, C.c_uint32)
_dw = _sig("omc_dw_update_recompress", C.c_int, _vp, _vp, _vp, omc_format, _vp, C.c_int, _vp, _vp, C.POINTER(omc_opt), _vp,
           C.c_uint32, C.c_uint32, C.c_uint32, _vp, C.c_size_t, _vp)
_gemm_dx = _sig("omc_dequant_gemm_dx", C.c_int, _vp, _vp, omc_format, _vp, _vp, C.c_uint32, C.c_uint32,
                C.c_uint32, _vp, C.c_size_t, _vp)

EXPORTED = ["omc_status_string", "omc_format_validate", "omc_format_bits", "omc_format_max",
            "omc_packed_bytes", "omc_compress_workspace_bytes", "omc_compress", "omc_decompress",
            "omc_compress_noalloc", "omc_compress_noalloc_max_elems",
            "omc_plan_bytes", "omc_plan_build", "omc_plan_workspace_bytes", "omc_workspace_bytes", "omc_plan_arena_bytes",
            "omc_plan_aux_elems", "omc_plan_launches", "omc_step_update_recompress",
            "omc_step_update_recompress_events", "omc_compress_set", "omc_decompress_set",
            "omc_plan_transport_bytes", "omc_reselect_plan_bytes", "omc_reselect_plan_build",
            "omc_reselect_workspace_bytes", "omc_reselect_algorithmic_bytes", "omc_reselect",
            "omc_transport_meta_bytes", "omc_transport_bytes", "omc_transport_pack", "omc_transport_open",
            "omc_aggregate_plan_bytes", "omc_aggregate_plan_build",
            "omc_aggregate_mean", "omc_dequant_gemm_workspace_bytes",
            "omc_dequant_gemm", "omc_dequant_gemm_dx", "omc_dw_update_workspace_bytes",
            "omc_dw_update_recompress"]


class OmcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({_status_string(status).decode()})")


def _check(status: int, where: str):
    if status != OMC_OK:
        raise OmcError(status, where)


def fmt(exp_bits: int, man_bits: int, bias: int = OMC_BIAS_DEFAULT) -> omc_format:
    return omc_format(exp_bits, man_bits, bias)


def opt(kind: int, lr: float, momentum: float = 0.9, beta1: float = 0.9, beta2: float = 0.999,
        eps: float = 1e-8, t: int = 1, flags: int = 0) -> omc_opt:
    """Hyper-parameters; the derived constants are computed in fp64 here and rounded once (omc.h)."""
    return omc_opt(kind, lr, momentum, beta1, beta2, eps, 1.0 - beta1, 1.0 - beta2,
                   1.0 - beta1 ** t, 1.0 - beta2 ** t, flags)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libomc takes contiguous device tensors")
    return t.data_ptr()


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


# ------------------------------------------------------------------ host-only helpers
def omc_format_validate(f: omc_format) -> int:
    return _format_validate(f)


def omc_format_bits(f: omc_format) -> int:
    return _format_bits(f)


def omc_format_max(f: omc_format) -> float:
    return _format_max(f)


def omc_packed_bytes(f: omc_format, n: int) -> int:
    return _packed_bytes(f, n)


def omc_compress_workspace_bytes(n: int) -> int:
    return _compress_ws(n)


def omc_dequant_gemm_workspace_bytes(M: int) -> int:
    return _gemm_ws(M)


# ------------------------------------------------------------------ single variable
def omc_compress(v: torch.Tensor, n: int, f: omc_format, use_pvt: bool, codes: torch.Tensor,
                 sb: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(_compress(_ptr(v), n, f, int(use_pvt), _ptr(codes), _ptr(sb), _ptr(ws),
                     ws.numel() * ws.element_size(), _stream(stream)), "omc_compress")


def omc_compress_noalloc_max_elems() -> int:
    return _compress_noalloc_max()


def omc_compress_noalloc(v: torch.Tensor, n: int, f: omc_format, use_pvt: bool, codes: torch.Tensor,
                         sb: torch.Tensor, stream=None) -> None:
    _check(_compress_noalloc(_ptr(v), n, f, int(use_pvt), _ptr(codes), _ptr(sb), _stream(stream)),
           "omc_compress_noalloc")


def omc_decompress(codes: torch.Tensor, n: int, f: omc_format, sb: Optional[torch.Tensor],
                   out: torch.Tensor, stream=None) -> None:
    _check(_decompress(_ptr(codes), n, f, _ptr(sb), _ptr(out), _stream(stream)), "omc_decompress")


# ------------------------------------------------------------------ variable sets
@dataclass
class Plan:
    """Host and device copies of a plan blob (omc_plan_build)."""
    host: np.ndarray            # uint8
    dev: torch.Tensor           # uint8, same bytes on the GPU
    nvars: int

    @property
    def workspace_bytes(self) -> int:
        return _plan_ws(self.host.ctypes.data)

    @property
    def transport_bytes(self) -> int:
        return _plan_transport(self.host.ctypes.data)

    @property
    def launches(self) -> int:
        return _plan_launches(self.host.ctypes.data)

    @property
    def arena_bytes(self) -> int:
        return _plan_arena(self.host.ctypes.data)

    @property
    def aux_elems(self) -> int:
        return _plan_aux(self.host.ctypes.data)


def make_var_table(vars_: Sequence[dict]):
    tab = (omc_var * len(vars_))()
    for i, v in enumerate(vars_):
        flags = (OMC_VAR_QUANTIZED if v["quantized"] else 0) | (0 if v.get("use_pvt", True) else OMC_VAR_NO_PVT)
        f = v.get("fmt") or omc_format(8, 23, OMC_BIAS_DEFAULT)
        tab[i] = omc_var(int(v["data_offset"]), int(v["aux_offset"]), int(v["n"]), f, flags)
    return tab


def omc_workspace_bytes(var_table) -> int:
    return _workspace_bytes(C.cast(var_table, _vp), len(var_table))


def omc_plan_build(var_table, device="cuda") -> Plan:
    nvars = len(var_table)
    size = _plan_bytes(C.cast(var_table, _vp), nvars)
    host = np.zeros(max(size, 1), dtype=np.uint8)
    _check(_plan_build(C.cast(var_table, _vp), nvars, host.ctypes.data, size), "omc_plan_build")
    dev = torch.from_numpy(host).to(device)
    return Plan(host, dev, nvars)


def omc_step_update_recompress(arena: torch.Tensor, plan: Plan, sb_table: torch.Tensor,
                               grads: torch.Tensor, state0: Optional[torch.Tensor],
                               state1: Optional[torch.Tensor], o: omc_opt, ws: torch.Tensor,
                               stream=None) -> None:
    _check(_step(_ptr(arena), arena.numel() * arena.element_size(), plan.host.ctypes.data,
                 _ptr(plan.dev), _ptr(sb_table), _ptr(grads), _ptr(state0), _ptr(state1),
                 grads.numel(), C.byref(o), _ptr(ws), ws.numel() * ws.element_size(),
                 _stream(stream)), "omc_step_update_recompress")


def omc_compress_set(values: torch.Tensor, plan: Plan, arena: torch.Tensor, sb_table: torch.Tensor,
                     ws: torch.Tensor, stream=None) -> None:
    _check(_compress_set(_ptr(values), values.numel(), plan.host.ctypes.data, _ptr(plan.dev), _ptr(arena),
                         arena.numel() * arena.element_size(), _ptr(sb_table), _ptr(ws),
                         ws.numel() * ws.element_size(), _stream(stream)), "omc_compress_set")


def omc_decompress_set(arena: torch.Tensor, plan: Plan, sb_table: torch.Tensor, out: torch.Tensor,
                       stream=None) -> None:
    _check(_decompress_set(_ptr(arena), arena.numel() * arena.element_size(), plan.host.ctypes.data,
                           _ptr(plan.dev), _ptr(sb_table), _ptr(out), out.numel(), _stream(stream)),
           "omc_decompress_set")


# ------------------------------------------------------------------ a new round's quantized subset
@dataclass
class ReselectPlan:
    host: np.ndarray
    dev: torch.Tensor

    @property
    def workspace_bytes(self) -> int:
        return _rs_ws(self.host.ctypes.data)

    @property
    def algorithmic_bytes(self) -> int:
        return _rs_alg(self.host.ctypes.data)


def omc_reselect_plan_build(plan_old: Plan, plan_new: Plan) -> ReselectPlan:
    size = _rs_bytes(plan_old.host.ctypes.data, plan_new.host.ctypes.data)
    buf = np.zeros(max(size, 16), dtype=np.uint8)
    _check(_rs_build(plan_old.host.ctypes.data, plan_new.host.ctypes.data, buf.ctypes.data, size),
           "omc_reselect_plan_build")
    return ReselectPlan(buf, torch.from_numpy(buf).cuda())


def omc_reselect(rs: ReselectPlan, arena_old: torch.Tensor, sb_old: torch.Tensor, arena_new: torch.Tensor,
                 sb_new: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(_reselect(rs.host.ctypes.data, _ptr(rs.dev), _ptr(arena_old), arena_old.numel() * arena_old.element_size(),
                     _ptr(sb_old), _ptr(arena_new), arena_new.numel() * arena_new.element_size(), _ptr(sb_new),
                     _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "omc_reselect")


# ------------------------------------------------------------------ transport / checkpoint message
def omc_transport_meta_bytes(nvars: int) -> int:
    return _tr_meta(nvars)


def omc_transport_bytes(plan: Plan) -> int:
    return _tr_bytes(plan.host.ctypes.data)


def omc_transport_pack(plan: Plan, arena: torch.Tensor, sb_table: torch.Tensor, msg: torch.Tensor, stream=None) -> None:
    _check(_tr_pack(plan.host.ctypes.data, _ptr(plan.dev), _ptr(arena), arena.numel() * arena.element_size(),
                    _ptr(sb_table), _ptr(msg), msg.numel() * msg.element_size(), _stream(stream)), "omc_transport_pack")


def omc_transport_open(prefix: np.ndarray, msg_bytes: int):
    """prefix: the first bytes of a message in host memory (uint8).  Returns (omc_var table or None when the
    prefix is shorter than header + table, nvars, sb_offset, arena_offset, arena_bytes, aux_elems)."""
    prefix = np.ascontiguousarray(prefix, dtype=np.uint8)
    nv, so, ao, ab, ae = C.c_uint32(), C.c_uint64(), C.c_uint64(), C.c_uint64(), C.c_uint64()
    _check(_tr_open(prefix.ctypes.data, prefix.size, msg_bytes, None, 0, C.byref(nv), C.byref(so), C.byref(ao),
                    C.byref(ab), C.byref(ae)), "omc_transport_open")
    table = None
    if prefix.size >= _tr_meta(nv.value):
        table = (omc_var * nv.value)()
        _check(_tr_open(prefix.ctypes.data, prefix.size, msg_bytes, C.cast(table, _vp), nv.value, C.byref(nv),
                        C.byref(so), C.byref(ao), C.byref(ab), C.byref(ae)), "omc_transport_open")
    return table, nv.value, so.value, ao.value, ab.value, ae.value


class HipEvents:
    """Caller-owned HIP events for omc_step_update_recompress_events (plain HIP runtime calls)."""

    def __init__(self, count: int):
        self._hip = C.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [C.POINTER(_vp)]
        self._hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), _vp, _vp]
        self._hip.hipEventSynchronize.argtypes = [_vp]
        self._hip.hipEventDestroy.argtypes = [_vp]
        self.handles = (_vp * count)()
        for i in range(count):
            h = _vp()
            if self._hip.hipEventCreate(C.byref(h)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.handles[i] = h

    def elapsed_ms(self, i: int, j: int) -> float:
        self._hip.hipEventSynchronize(self.handles[j])
        ms = C.c_float()
        if self._hip.hipEventElapsedTime(C.byref(ms), self.handles[i], self.handles[j]) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def __del__(self):
        for h in self.handles:
            if h:
                self._hip.hipEventDestroy(h)


def omc_step_update_recompress_events(arena, plan: Plan, sb_table, grads, state0, state1, o: omc_opt,
                                      ws, events: HipEvents, first: int = 0, stream=None) -> None:
    """`first`: index of the first event handle to use (2 * plan.launches handles are consumed)."""
    _check(_step_ev(_ptr(arena), arena.numel() * arena.element_size(), plan.host.ctypes.data,
                    _ptr(plan.dev), _ptr(sb_table), _ptr(grads), _ptr(state0), _ptr(state1),
                    grads.numel(), C.byref(o), _ptr(ws), ws.numel() * ws.element_size(),
                    _stream(stream), C.cast(C.byref(events.handles, first * C.sizeof(_vp)), _vp),
                    len(events.handles) - first),
           "omc_step_update_recompress_events")


# ------------------------------------------------------------------ forward path
def omc_dequant_gemm(A: torch.Tensor, codes: torch.Tensor, f: omc_format, sb: Optional[torch.Tensor],
                     Cout: torch.Tensor, M: int, N: int, K: int, ws: torch.Tensor, stream=None) -> None:
    _check(_gemm(_ptr(A), _ptr(codes), f, _ptr(sb), _ptr(Cout), M, N, K, _ptr(ws),
                 ws.numel() * ws.element_size(), _stream(stream)), "omc_dequant_gemm")


def omc_dequant_gemm_dx(dY: torch.Tensor, codes: torch.Tensor, f: omc_format, sb: Optional[torch.Tensor],
                        dX: torch.Tensor, M: int, N: int, K: int, ws: torch.Tensor, stream=None) -> None:
    _check(_gemm_dx(_ptr(dY), _ptr(codes), f, _ptr(sb), _ptr(dX), M, N, K, _ptr(ws),
                    ws.numel() * ws.element_size(), _stream(stream)), "omc_dequant_gemm_dx")


def omc_dw_update_workspace_bytes(f: omc_format, M: int, N: int, K: int) -> int:
    return _dw_ws(f, M, N, K)


def omc_dw_update_recompress(X: torch.Tensor, dY: torch.Tensor, codes: torch.Tensor, f: omc_format, sb: torch.Tensor,
                             use_pvt: bool, state0: Optional[torch.Tensor], state1: Optional[torch.Tensor], o: omc_opt,
                             dW_out: Optional[torch.Tensor], M: int, N: int, K: int, ws: torch.Tensor, stream=None) -> None:
    _check(_dw(_ptr(X), _ptr(dY), _ptr(codes), f, _ptr(sb), int(use_pvt), _ptr(state0), _ptr(state1), C.byref(o),
               _ptr(dW_out), M, N, K, _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "omc_dw_update_recompress")


# --------------------------------------------------------------------------- server aggregation
OMC_MAX_REPLICAS = 16


@dataclass
class AggregatePlan:
    host: np.ndarray                 # the blob (uint8)
    dev: torch.Tensor                # its device copy
    nreplicas: int


def omc_aggregate_plan_build(plans: Sequence["Plan"]) -> AggregatePlan:
    """Merge the clients' plans (same variable list, own quantized subsets) into an aggregation plan."""
    R = len(plans)
    ptrs = (C.c_void_p * R)(*[p.host.ctypes.data for p in plans])
    size = _agg_bytes(ptrs, R)
    buf = np.zeros(max(size, 16), dtype=np.uint8)
    _check(_agg_build(ptrs, R, buf.ctypes.data, buf.size), "omc_aggregate_plan_build")
    return AggregatePlan(buf, torch.from_numpy(buf).cuda(), R)


def omc_aggregate_mean(agg: AggregatePlan, arenas: Sequence[torch.Tensor], sb_tables: Sequence[torch.Tensor],
                       out: torch.Tensor, stream=None) -> None:
    R = agg.nreplicas
    assert len(arenas) == R and len(sb_tables) == R
    ap = (C.c_void_p * R)(*[_ptr(a) for a in arenas])
    ab = (C.c_size_t * R)(*[a.numel() * a.element_size() for a in arenas])
    sp = (C.c_void_p * R)(*[_ptr(s) for s in sb_tables])
    _check(_agg_mean(agg.host.ctypes.data, _ptr(agg.dev), ap, ab, sp, _ptr(out), out.numel(), _stream(stream)),
           "omc_aggregate_mean")
