"""ctypes binding of libthc (include/thc.h).  Argument marshalling only: every step of the path runs
in the HIP kernels.  PyTorch supplies device memory (`tensor.data_ptr()`) and the current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_LIB = None
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libthc.so")

THC_MAX_WORKERS = 64
THC_DTYPE_F32, THC_DTYPE_BF16 = 0, 1
THC_ORDER_ASCENDING, THC_ORDER_SPLIT = 0, 1

EXPORTS = ("thc_version", "thc_strerror", "thc_workspace_bytes", "thc_prepare_range", "thc_compress",
           "thc_compress_all", "thc_aggregate", "thc_decompress", "thc_decompress_noalloc",
           "thc_uniform_workspace_bytes",
           "thc_uniform_prepare_range", "thc_uniform_compress", "thc_uniform_decompress", "thc_threshold",
           "thc_solve_table", "thc_solve_table_bruteforce", "thc_describe_plan")


class thc_params(C.Structure):
    _fields_ = [("d", C.c_uint64), ("block", C.c_uint64), ("n", C.c_uint32), ("b", C.c_uint32),
                ("g", C.c_uint32), ("agg_bits", C.c_uint32), ("in_dtype", C.c_uint32), ("t_p", C.c_float),
                ("seed", C.c_uint64), ("table", C.c_uint8 * 256), ("stage_order", C.c_uint32),
                ("first_block", C.c_uint32), ("group_log2", C.c_uint32), ("single_launch", C.c_uint32)]


class ThcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {thc_strerror(status)} ({status})")


def lib():
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2302_08545_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
        pp = C.POINTER(thc_params)
        L.thc_version.restype = C.c_int
        L.thc_strerror.restype = C.c_char_p
        L.thc_strerror.argtypes = [C.c_int]
        L.thc_workspace_bytes.argtypes = [pp, C.c_int, C.POINTER(C.c_size_t)]
        L.thc_uniform_workspace_bytes.argtypes = [pp, C.c_int, C.POINTER(C.c_size_t)]
        L.thc_prepare_range.argtypes = [pp, C.POINTER(vp), C.POINTER(vp), vp, vp, vp]
        L.thc_compress.argtypes = [pp, u32, u64, vp, vp, vp, vp, vp, vp]
        L.thc_compress_all.argtypes = [pp, u64, C.POINTER(vp), C.POINTER(vp), vp, C.POINTER(vp), vp, vp]
        L.thc_aggregate.argtypes = [pp, C.POINTER(vp), vp, vp]
        L.thc_decompress.argtypes = [pp, u64, vp, vp, vp, vp, vp]
        L.thc_decompress_noalloc.argtypes = [pp, u64, vp, vp, vp, vp]
        L.thc_uniform_prepare_range.argtypes = [pp, u64, C.POINTER(vp), C.POINTER(vp), C.c_int, vp, vp, vp, vp]
        L.thc_uniform_compress.argtypes = [pp, u32, u64, vp, vp, C.c_int, vp, vp, vp, vp, vp]
        L.thc_uniform_decompress.argtypes = [pp, u64, vp, C.c_int, vp, vp, vp, vp, vp]
        L.thc_threshold.restype = C.c_double
        L.thc_threshold.argtypes = [C.c_double]
        L.thc_solve_table.argtypes = [u32, u32, C.c_double, C.POINTER(C.c_uint8), C.POINTER(C.c_double)]
        L.thc_solve_table_bruteforce.argtypes = [u32, u32, C.c_double, C.POINTER(C.c_uint8), C.POINTER(C.c_double),
                                                 C.POINTER(C.c_uint64)]
        L.thc_describe_plan.argtypes = [pp, C.POINTER(C.c_uint32), C.c_size_t]
        _LIB = L
    return _LIB


def make_params(d: int, block: int, n: int, b: int, g: int, t_p: float, seed: int, table: Sequence[int],
                agg_bits: int = 8, in_dtype: int = THC_DTYPE_F32, stage_order: int = THC_ORDER_ASCENDING,
                first_block: int = 0, group_log2: int = 0, single_launch: int = 0) -> thc_params:
    p = thc_params()
    p.stage_order = stage_order
    p.first_block = first_block
    p.group_log2 = group_log2
    p.single_launch = single_launch
    p.d, p.block, p.n, p.b, p.g = d, block, n, b, g
    p.agg_bits, p.in_dtype, p.t_p, p.seed = agg_bits, in_dtype, t_p, seed
    for i, v in enumerate(table):
        p.table[i] = int(v)
    return p


def _ptr(t) -> Optional[int]:
    return None if t is None else (t if isinstance(t, int) else t.data_ptr())


def _ptr_array(ts):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = _ptr(t)
    return arr


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise ThcError(rc, where)


def thc_version() -> int:
    return lib().thc_version()


def thc_strerror(status: int) -> str:
    return lib().thc_strerror(status).decode()


def thc_workspace_bytes(p: thc_params, ef_enabled: bool = False) -> int:
    out = C.c_size_t(0)
    _check(lib().thc_workspace_bytes(C.byref(p), int(ef_enabled), C.byref(out)), "thc_workspace_bytes")
    return out.value


def thc_uniform_workspace_bytes(p: thc_params, rotate: bool) -> int:
    out = C.c_size_t(0)
    _check(lib().thc_uniform_workspace_bytes(C.byref(p), int(rotate), C.byref(out)), "thc_uniform_workspace_bytes")
    return out.value


def thc_prepare_range(p: thc_params, grads, ef, range_M, ws, stream=None) -> None:
    _check(lib().thc_prepare_range(C.byref(p), _ptr_array(grads), _ptr_array(ef), _ptr(range_M), _ptr(ws),
                                   _stream(stream)), "thc_prepare_range")


def thc_compress_all(p: thc_params, rnd: int, grads, ef_inout, range_M, packed_out, ws, stream=None) -> None:
    _check(lib().thc_compress_all(C.byref(p), rnd, _ptr_array(grads), _ptr_array(ef_inout), _ptr(range_M),
                                  _ptr_array(packed_out), _ptr(ws), _stream(stream)), "thc_compress_all")


def thc_compress(p: thc_params, worker_id: int, rnd: int, grad, ef_inout, range_M, packed_out, ws,
                 stream=None) -> None:
    _check(lib().thc_compress(C.byref(p), worker_id, rnd, _ptr(grad), _ptr(ef_inout), _ptr(range_M),
                              _ptr(packed_out), _ptr(ws), _stream(stream)), "thc_compress")


def thc_aggregate(p: thc_params, packed, agg_out, stream=None) -> None:
    _check(lib().thc_aggregate(C.byref(p), _ptr_array(packed), _ptr(agg_out), _stream(stream)), "thc_aggregate")


def thc_decompress(p: thc_params, rnd: int, agg, range_M, out, ws, stream=None) -> None:
    _check(lib().thc_decompress(C.byref(p), rnd, _ptr(agg), _ptr(range_M), _ptr(out), _ptr(ws), _stream(stream)),
           "thc_decompress")


def thc_decompress_noalloc(p: thc_params, rnd: int, agg, range_M, out, stream=None) -> None:
    _check(lib().thc_decompress_noalloc(C.byref(p), rnd, _ptr(agg), _ptr(range_M), _ptr(out), _stream(stream)),
           "thc_decompress_noalloc")


def thc_uniform_prepare_range(p: thc_params, rnd: int, grads, ef, rotate: bool, range_m, range_M, ws,
                              stream=None) -> None:
    _check(lib().thc_uniform_prepare_range(C.byref(p), rnd, _ptr_array(grads), _ptr_array(ef), int(rotate),
                                           _ptr(range_m), _ptr(range_M), _ptr(ws), _stream(stream)),
           "thc_uniform_prepare_range")


def thc_uniform_compress(p: thc_params, worker_id: int, rnd: int, grad, ef_inout, rotate: bool, range_m, range_M,
                         packed_out, ws, stream=None) -> None:
    _check(lib().thc_uniform_compress(C.byref(p), worker_id, rnd, _ptr(grad), _ptr(ef_inout), int(rotate),
                                      _ptr(range_m), _ptr(range_M), _ptr(packed_out), _ptr(ws), _stream(stream)),
           "thc_uniform_compress")


def thc_uniform_decompress(p: thc_params, rnd: int, agg, rotate: bool, range_m, range_M, out, ws,
                           stream=None) -> None:
    _check(lib().thc_uniform_decompress(C.byref(p), rnd, _ptr(agg), int(rotate), _ptr(range_m), _ptr(range_M),
                                        _ptr(out), _ptr(ws), _stream(stream)), "thc_uniform_decompress")


def thc_threshold(p: float) -> float:
    return lib().thc_threshold(p)


def thc_solve_table(b: int, g: int, p: float):
    """Returns (table as a list of 2^b ints, cost in sigma^2 units)."""
    out = (C.c_uint8 * 256)()
    cost = C.c_double(0.0)
    _check(lib().thc_solve_table(b, g, p, out, C.byref(cost)), "thc_solve_table")
    return [int(out[i]) for i in range(2 ** b)], cost.value


def thc_solve_table_bruteforce(b: int, g: int, p: float):
    """Exhaustive search over Alg. 4's enumeration.  Returns (table, cost, number of candidates visited)."""
    out = (C.c_uint8 * 256)()
    cost = C.c_double(0.0)
    count = C.c_uint64(0)
    _check(lib().thc_solve_table_bruteforce(b, g, p, out, C.byref(cost), C.byref(count)), "thc_solve_table_bruteforce")
    return [int(out[i]) for i in range(2 ** b)], cost.value, count.value


THC_PLAN_RECORD_WORDS = 40


def thc_describe_plan(p: thc_params):
    """The passes of the transform for these parameters: a list of dicts (kind, bits, tiling fields)."""
    n = lib().thc_describe_plan(C.byref(p), None, 0)
    _check(min(n, 0), "thc_describe_plan")
    buf = (C.c_uint32 * (n * THC_PLAN_RECORD_WORDS))()
    _check(min(lib().thc_describe_plan(C.byref(p), buf, n), 0), "thc_describe_plan")
    names = ("L", "logw", "nrows", "nfixed", "n0", "sh0", "sh1")
    out = []
    for k in range(n):
        r = buf[k * THC_PLAN_RECORD_WORDS:(k + 1) * THC_PLAN_RECORD_WORDS]
        rec = {"kind": r[0], "bits": list(r[2:2 + r[1]])}
        rec.update(zip(names, r[18:25]))
        rec["fcum"], rec["fmask"], rec["fpos"] = list(r[25:29]), list(r[29:33]), list(r[33:37])
        out.append(rec)
    return out
