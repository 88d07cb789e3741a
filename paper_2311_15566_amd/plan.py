"""ctypes binding of the host-side planning calls (include/spotshard_plan.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .binding import ModelDesc, Slice, _check, _desc, _slice, lib

i32, u64, i64 = C.c_int32, C.c_uint64, C.c_int64
lib.ss_context_overlap.argtypes = [C.POINTER(ModelDesc), i32, C.POINTER(Slice), C.POINTER(Slice), u64, C.POINTER(u64), C.POINTER(u64)]
lib.ss_match_devices.argtypes = [i32, C.POINTER(u64), C.POINTER(i32), C.POINTER(u64)]
lib.ss_migration_order.argtypes = [i32, i32, C.POINTER(i64), i64, C.POINTER(i32)]
lib.ss_progressive_plan.argtypes = [i32, C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32)]
lib.ss_rows_to_keep.argtypes = [i32, C.POINTER(i32), i32, i32, C.POINTER(i32)]
lib.ss_jit_iterations.argtypes = [i32, i32, C.POINTER(C.c_double), C.c_double, C.c_double]
lib.ss_jit_iterations.restype = i32


class CostSample(C.Structure):
    _fields_ = [("batch", i32), ("length", i32), ("ms", C.c_double)]


class CostModel(C.Structure):
    _fields_ = [("n_batches", i32), ("batch", i32 * 16), ("dec_base_ms", C.c_double * 16), ("dec_per_row_ms", C.c_double * 16),
                ("pre_base_ms", C.c_double * 16), ("pre_per_token_ms", C.c_double * 16)]


lib.ss_cost_fit.argtypes = [C.POINTER(CostSample), i32, C.POINTER(CostSample), i32, C.POINTER(CostModel)]
lib.ss_cost_l_exe.argtypes = [C.POINTER(CostModel), i32, i32, i32, C.POINTER(C.c_double)]
lib.ss_cost_fit.restype = lib.ss_cost_l_exe.restype = i32
for f in (lib.ss_context_overlap, lib.ss_match_devices, lib.ss_migration_order, lib.ss_progressive_plan, lib.ss_rows_to_keep):
    f.restype = i32


def context_overlap(desc: dict, tied: bool, a: dict, b: dict, kv_rows: int):
    d, sa, sb = _desc(desc), _slice(a), _slice(b)
    mb, cb = u64(), u64()
    _check(lib.ss_context_overlap(C.byref(d), int(tied), C.byref(sa), C.byref(sb), int(kv_rows), C.byref(mb), C.byref(cb)))
    return mb.value, cb.value


def match_devices(weight):
    w = np.ascontiguousarray(weight, dtype=np.uint64)
    n = w.shape[0]
    pos = (i32 * n)()
    total = u64()
    _check(lib.ss_match_devices(n, w.ctypes.data_as(C.POINTER(u64)), pos, C.byref(total)))
    return total.value, list(pos)


def migration_order(delta, u_max: int):
    dl = np.ascontiguousarray(delta, dtype=np.int64)
    L, N = dl.shape
    order = (i32 * L)()
    _check(lib.ss_migration_order(L, N, dl.ctypes.data_as(C.POINTER(i64)), int(u_max), order))
    return list(order)


def progressive_plan(order, stage_of_layer):
    L = len(order)
    n_stages = max(stage_of_layer) + 1
    o, s = (i32 * L)(*order), (i32 * L)(*stage_of_layer)
    kind, arg = (i32 * (1 + L + n_stages))(), (i32 * (1 + L + n_stages))()
    _check(lib.ss_progressive_plan(L, o, s, n_stages, kind, arg))
    names = ("migrate_cache", "migrate_layer", "start_stage")
    return [(names[k], a) for k, a in zip(kind, arg)]


def rows_to_keep(lens, keep: int, n_dst: int):
    ln = (i32 * len(lens))(*[int(v) for v in lens])
    out = (i32 * n_dst)()
    _check(lib.ss_rows_to_keep(len(lens), ln, keep, n_dst, out))
    return list(out)


def jit_iterations(acquisition: bool, l_exe, t_grace: float, t_mig: float) -> int:
    t = (C.c_double * len(l_exe))(*[float(v) for v in l_exe])
    return int(lib.ss_jit_iterations(int(acquisition), len(l_exe) - 1, t, float(t_grace), float(t_mig)))


def cost_fit(decode, prefill=()) -> CostModel:
    """decode / prefill: sequences of (batch, length, ms)."""
    d = (CostSample * len(decode))(*[CostSample(int(b), int(n), float(ms)) for b, n, ms in decode])
    p = (CostSample * max(len(prefill), 1))(*[CostSample(int(b), int(n), float(ms)) for b, n, ms in prefill])
    m = CostModel()
    _check(lib.ss_cost_fit(d, len(decode), p, len(prefill), C.byref(m)))
    return m


def cost_l_exe(model: CostModel, batch: int, s_in: int, s_out: int):
    out = (C.c_double * (s_out + 1))()
    _check(lib.ss_cost_l_exe(C.byref(model), batch, s_in, s_out, out))
    return list(out)
