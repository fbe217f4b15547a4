"""ctypes binding of include/nitsum_kvmig.h: argument marshalling only.

Functions carry the C names and semantics; see the header for layouts,
ownership and errors.  Device buffers are passed as integer addresses
(``tensor.data_ptr()``) and HIP streams as ``torch.cuda.Stream.cuda_stream``
integers; torch is imported only so that both share one HIP runtime.  A non-zero status raises
``NtsError`` with the library's message.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnts_kvmig.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2605_05467_amd.build` "
        "(there is no fallback path)")

# PyTorch ships its own copy of the HIP runtime.  Loading it first makes this
# library bind to that same copy; the other order would put two runtimes in one
# process, and device pointers from one are unknown to the other.
try:
    import torch  # noqa: F401
except ImportError:  # the library also works without PyTorch in the process
    pass

_lib = ctypes.CDLL(LIB_PATH)

NTS_OK, NTS_EINVAL, NTS_ERANGE, NTS_EDUP, NTS_EALIAS, NTS_ENOMEM, NTS_EHIP = 0, -1, -2, -3, -4, -5, -6
NTS_MAX_LAYERS = 96
NTS_VALIDATE_UNIQUE_DST = 1
NTS_DETECT_RUNS = 2
NTS_ORDER_BY_DST = 4
NTS_DEFAULT_STAGING_BYTES = 64 << 20
NTS_STATIC_STAGING_BYTES = 32 << 20

EXPORTS = (
    "nts_init", "nts_free", "nts_last_error", "nts_strerror", "nts_route",
    "nts_plan_create", "nts_plan_free", "nts_plan_info", "nts_plan_slots", "nts_plan_runs",
    "nts_run_pack", "nts_run_pack_chunk", "nts_run_unpack", "nts_run_unpack_chunk",
    "nts_run_migrate", "nts_run_migrate_batch", "nts_run_migrate_direct", "nts_run_memcpy_baseline",
    "nts_batch_staging_bytes", "nts_run_migrate_static",
    "nts_shard_linear", "nts_shard_linear_workspace", "nts_shard_linear_launch", "nts_shard_linear_view",
    "nts_shard_linear_tune", "nts_shard_linear_tuned",
    "nts_shard_linear_candidates", "nts_shard_linear_with", "nts_shard_linear_remember",
    "nts_balanced_block", "nts_goodput_efficiency", "nts_plan_cluster",
)
NTS_TP_LEVELS = 4
NTS_SPLIT_OUT, NTS_SPLIT_IN = 0, 1
NTS_BF16, NTS_F16 = 0, 1


class nts_desc(ctypes.Structure):
    _fields_ = [
        ("L", ctypes.c_int32), ("D", ctypes.c_int32), ("elem_bytes", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("Hs", ctypes.c_int32), ("Hd", ctypes.c_int32),
        ("src_head_off", ctypes.c_int32), ("dst_head_off", ctypes.c_int32), ("w", ctypes.c_int32),
        ("n_req", ctypes.c_int32), ("S_src", ctypes.c_int64), ("S_dst", ctypes.c_int64),
        ("ctx_len", ctypes.c_void_p), ("src_pages", ctypes.c_void_p), ("dst_pages", ctypes.c_void_p),
        ("src_token_stride", ctypes.c_int64), ("dst_token_stride", ctypes.c_int64),
        ("staging_bytes", ctypes.c_int64), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32),
    ]


class nts_linear_desc(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int32), ("n_out", ctypes.c_int32), ("n_in", ctypes.c_int32), ("tp", ctypes.c_int32),
        ("rank", ctypes.c_int32), ("split", ctypes.c_int32), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("ldx", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldy", ctypes.c_int64),
    ]


class nts_linear_launch(ctypes.Structure):
    _fields_ = [
        ("tiled", ctypes.c_int32), ("tile_rows", ctypes.c_int32), ("tile_cols", ctypes.c_int32),
        ("k_splits", ctypes.c_int32), ("slabs_ahead", ctypes.c_int32), ("k_waves", ctypes.c_int32),
        ("reserved", ctypes.c_int32 * 2),
    ]


class nts_tier(ctypes.Structure):
    _fields_ = [("rps", ctypes.c_double), ("thp", ctypes.c_double * 4), ("thd", ctypes.c_double * 4)]


class nts_alloc(ctypes.Structure):
    _fields_ = [("tier", ctypes.c_int32), ("tp_prefill", ctypes.c_int32), ("tp_decode", ctypes.c_int32),
                ("P", ctypes.c_int32), ("D", ctypes.c_int32), ("gpus", ctypes.c_int32),
                ("served_rps", ctypes.c_double)]


class nts_info(ctypes.Structure):
    _fields_ = [
        ("T", ctypes.c_int64), ("F", ctypes.c_int64), ("frag_bytes", ctypes.c_int64),
        ("X", ctypes.c_int64), ("chunk_frags", ctypes.c_int64), ("chunk_bytes", ctypes.c_int64),
        ("n_chunks", ctypes.c_int64), ("vec_bytes", ctypes.c_int32), ("n_runs", ctypes.c_int32),
    ]


_vp, _i, _i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
_pi = ctypes.POINTER(ctypes.c_int)
_lib.nts_init.argtypes = [_i, ctypes.POINTER(_vp)]
_lib.nts_free.argtypes = [_vp]
_lib.nts_last_error.argtypes = [_vp]
_lib.nts_last_error.restype = ctypes.c_char_p
_lib.nts_strerror.argtypes = [_i]
_lib.nts_strerror.restype = ctypes.c_char_p
_lib.nts_route.argtypes = [_i, _i, _i, _i, _i, _pi, _pi, _pi]
_lib.nts_plan_create.argtypes = [_vp, ctypes.POINTER(nts_desc), ctypes.POINTER(_vp)]
_lib.nts_plan_free.argtypes = [_vp]
_lib.nts_plan_info.argtypes = [_vp, ctypes.POINTER(nts_info)]
_lib.nts_plan_slots.argtypes = [_vp, _vp, _vp]
_lib.nts_plan_runs.argtypes = [_vp, _vp]
_lib.nts_run_pack.argtypes = [_vp, _vp, _vp, _vp]
_lib.nts_run_pack_chunk.argtypes = [_vp, _vp, _i64, _vp, _vp]
_lib.nts_run_unpack.argtypes = [_vp, _vp, _vp, _vp]
_lib.nts_run_unpack_chunk.argtypes = [_vp, _vp, _i64, _vp, _vp]
_lib.nts_run_migrate.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.nts_run_migrate_batch.argtypes = [_i, _vp, _vp, _vp, _vp, _vp]
_lib.nts_run_migrate_direct.argtypes = [_vp, _vp, _vp, _vp]
_lib.nts_run_migrate_static.argtypes = [_vp, _vp, _vp, _vp]
_lib.nts_batch_staging_bytes.argtypes = [_i, _vp, ctypes.POINTER(_i64)]
_lib.nts_run_memcpy_baseline.argtypes = [_vp, _vp, _vp, _i, _vp, ctypes.POINTER(_i64)]
_lib.nts_shard_linear_workspace.argtypes = [ctypes.POINTER(nts_linear_desc), ctypes.POINTER(ctypes.c_size_t)]
_lib.nts_shard_linear_launch.argtypes = [ctypes.POINTER(nts_linear_desc), ctypes.POINTER(nts_linear_launch)]
_lib.nts_shard_linear_view.argtypes = [ctypes.POINTER(nts_linear_desc)] + [ctypes.POINTER(ctypes.c_int64)] * 4
_lib.nts_shard_linear.argtypes = [_vp, ctypes.POINTER(nts_linear_desc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.nts_shard_linear_tune.argtypes = [_vp, ctypes.POINTER(nts_linear_desc), _vp, _vp, _i, _vp, _vp, ctypes.c_size_t, _vp,
                                       ctypes.POINTER(nts_linear_launch)]
_lib.nts_shard_linear_tuned.argtypes = [_vp, ctypes.POINTER(nts_linear_desc), ctypes.POINTER(nts_linear_launch)]
_lib.nts_shard_linear_candidates.argtypes = [ctypes.POINTER(nts_linear_desc), ctypes.POINTER(nts_linear_launch), _i, _pi]
_lib.nts_shard_linear_with.argtypes = [_vp, ctypes.POINTER(nts_linear_desc), ctypes.POINTER(nts_linear_launch), _vp, _vp,
                                       _vp, _vp, ctypes.c_size_t, _vp]
_lib.nts_shard_linear_remember.argtypes = [_vp, ctypes.POINTER(nts_linear_desc), ctypes.POINTER(nts_linear_launch)]
_d = ctypes.c_double
_lib.nts_balanced_block.argtypes = [_d, _d, _i, _pi, _pi]
_lib.nts_goodput_efficiency.argtypes = [_d, _i, _d, _i, _i, _i, _d, ctypes.POINTER(_d)]
_lib.nts_plan_cluster.argtypes = [_i, _i, ctypes.POINTER(nts_tier), _i, ctypes.POINTER(nts_alloc), _i, _pi, _pi]
for _name in EXPORTS:
    if _name not in ("nts_last_error", "nts_strerror"):
        getattr(_lib, _name).restype = _i


class NtsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{nts_strerror(status)} ({status}): {message}")
        self.status = status


def nts_strerror(status: int) -> str:
    return _lib.nts_strerror(status).decode()


def nts_last_error(ctx: int) -> str:
    return _lib.nts_last_error(ctx).decode()


def _check(status: int, ctx: Optional[int]) -> None:
    if status != NTS_OK:
        raise NtsError(status, nts_last_error(ctx) if ctx else "")


def nts_init(device_id: int = 0) -> int:
    out = _vp()
    _check(_lib.nts_init(device_id, ctypes.byref(out)), None)
    return out.value


def nts_free(ctx: int) -> None:
    _check(_lib.nts_free(ctx), ctx)


def nts_route(H: int, Ns: int, rs: int, Nd: int, rd: int) -> Tuple[int, int, int]:
    so, do, w = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    st = _lib.nts_route(H, Ns, rs, Nd, rd, ctypes.byref(so), ctypes.byref(do), ctypes.byref(w))
    if st != NTS_OK:
        raise NtsError(st, "nts_route")
    return so.value, do.value, w.value


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def nts_plan_create(ctx: int, *, L: int, D: int, elem_bytes: int, page_size: int, Hs: int, Hd: int,
                    src_head_off: int, dst_head_off: int, w: int, S_src: int, S_dst: int,
                    ctx_len, src_pages, dst_pages, src_token_stride: int = 0,
                    dst_token_stride: int = 0, staging_bytes: int = 0, flags: int = 0) -> int:
    ctx_len, src_pages, dst_pages = _i32(ctx_len), _i32(src_pages), _i32(dst_pages)
    d = nts_desc(L=L, D=D, elem_bytes=elem_bytes, page_size=page_size, Hs=Hs, Hd=Hd,
                 src_head_off=src_head_off, dst_head_off=dst_head_off, w=w, n_req=len(ctx_len),
                 S_src=S_src, S_dst=S_dst, ctx_len=ctx_len.ctypes.data,
                 src_pages=src_pages.ctypes.data, dst_pages=dst_pages.ctypes.data,
                 src_token_stride=src_token_stride, dst_token_stride=dst_token_stride,
                 staging_bytes=staging_bytes, flags=flags)
    out = _vp()
    _check(_lib.nts_plan_create(ctx, ctypes.byref(d), ctypes.byref(out)), ctx)
    return out.value


def nts_plan_free(plan: int) -> None:
    st = _lib.nts_plan_free(plan)
    if st != NTS_OK:
        raise NtsError(st, "nts_plan_free")


def nts_plan_info(plan: int) -> nts_info:
    info = nts_info()
    st = _lib.nts_plan_info(plan, ctypes.byref(info))
    if st != NTS_OK:
        raise NtsError(st, "nts_plan_info")
    return info


def nts_plan_slots(plan: int) -> Tuple[np.ndarray, np.ndarray]:
    T = nts_plan_info(plan).T
    s, d = np.empty(T, np.int32), np.empty(T, np.int32)
    st = _lib.nts_plan_slots(plan, s.ctypes.data, d.ctypes.data)
    if st != NTS_OK:
        raise NtsError(st, "nts_plan_slots")
    return s, d


def nts_plan_runs(plan: int) -> np.ndarray:
    """First token of every run, then T (n_runs + 1 entries); the plan needs NTS_DETECT_RUNS."""
    r = np.empty(nts_plan_info(plan).n_runs + 1, np.int32)
    st = _lib.nts_plan_runs(plan, r.ctypes.data)
    if st != NTS_OK:
        raise NtsError(st, "nts_plan_runs")
    return r


def layer_ptrs(base_ptr: int, L: int, slab_bytes: int):
    """Host table of 2L device pointers for one allocation [L][2][S][H_local][D]."""
    return (ctypes.c_void_p * (2 * L))(*[base_ptr + i * slab_bytes for i in range(2 * L)])


def _tab(ptrs):
    if isinstance(ptrs, ctypes.Array):
        return ptrs
    return (ctypes.c_void_p * len(ptrs))(*[int(p) for p in ptrs])


def _run(status: int) -> None:
    if status != NTS_OK:
        raise NtsError(status, "run call rejected (see nts_last_error on the context)")


def nts_run_pack(plan: int, src_layer_ptrs, stream_out: int, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_pack(plan, _tab(src_layer_ptrs), stream_out, hip_stream))


def nts_run_pack_chunk(plan: int, src_layer_ptrs, k: int, chunk_out: int, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_pack_chunk(plan, _tab(src_layer_ptrs), k, chunk_out, hip_stream))


def nts_run_unpack(plan: int, stream_in: int, dst_layer_ptrs, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_unpack(plan, stream_in, _tab(dst_layer_ptrs), hip_stream))


def nts_run_unpack_chunk(plan: int, chunk_in: int, k: int, dst_layer_ptrs, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_unpack_chunk(plan, chunk_in, k, _tab(dst_layer_ptrs), hip_stream))


def nts_run_migrate(plan: int, src_layer_ptrs, dst_layer_ptrs, staging: int, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_migrate(plan, _tab(src_layer_ptrs), _tab(dst_layer_ptrs), staging, hip_stream))


def nts_run_migrate_batch(plans, src_layer_ptrs, dst_layer_ptrs, staging: int, hip_stream: int = 0) -> None:
    """plans: sequence of plan handles; src/dst_layer_ptrs: one pointer table per plan."""
    n = len(plans)
    if len(src_layer_ptrs) != n or len(dst_layer_ptrs) != n:
        raise ValueError("one source and one destination pointer table per plan")
    stabs = [_tab(t) for t in src_layer_ptrs]   # kept alive until the call returns
    dtabs = [_tab(t) for t in dst_layer_ptrs]
    arr = ctypes.c_void_p * n
    _run(_lib.nts_run_migrate_batch(n, arr(*[int(p) for p in plans]),
                                    arr(*[ctypes.addressof(t) for t in stabs]),
                                    arr(*[ctypes.addressof(t) for t in dtabs]), staging, hip_stream))


def nts_run_migrate_static(plan: int, src_layer_ptrs, dst_layer_ptrs, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_migrate_static(plan, _tab(src_layer_ptrs), _tab(dst_layer_ptrs), hip_stream))


def nts_batch_staging_bytes(plans) -> int:
    n = len(plans)
    out = _i64(0)
    st = _lib.nts_batch_staging_bytes(n, (ctypes.c_void_p * max(n, 1))(*[int(p) for p in plans]), ctypes.byref(out))
    if st != NTS_OK:
        raise NtsError(st, "nts_batch_staging_bytes")
    return out.value


def nts_run_migrate_direct(plan: int, src_layer_ptrs, dst_layer_ptrs, hip_stream: int = 0) -> None:
    _run(_lib.nts_run_migrate_direct(plan, _tab(src_layer_ptrs), _tab(dst_layer_ptrs), hip_stream))


def nts_run_memcpy_baseline(plan: int, src_layer_ptrs, dst_layer_ptrs, merge_runs: bool = False,
                            hip_stream: int = 0) -> int:
    n = _i64(0)
    _run(_lib.nts_run_memcpy_baseline(plan, _tab(src_layer_ptrs), _tab(dst_layer_ptrs),
                                      1 if merge_runs else 0, hip_stream, ctypes.byref(n)))
    return n.value


def _linear_desc(M, n_out, n_in, tp, rank, split, ldx=0, ldw=0, ldy=0, dtype=0) -> nts_linear_desc:
    return nts_linear_desc(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=rank, split=split, dtype=dtype,
                           ldx=ldx, ldw=ldw, ldy=ldy)


def nts_shard_linear_workspace(*, M: int, n_out: int, n_in: int, tp: int, rank: int, split: int,
                               ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0) -> int:
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    n = ctypes.c_size_t(0)
    st = _lib.nts_shard_linear_workspace(ctypes.byref(d), ctypes.byref(n))
    if st != NTS_OK:
        raise NtsError(st, "nts_shard_linear_workspace")
    return n.value


def nts_shard_linear_launch(*, M: int, n_out: int, n_in: int, tp: int, rank: int, split: int,
                            ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0) -> "nts_linear_launch":
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    out = nts_linear_launch()
    st = _lib.nts_shard_linear_launch(ctypes.byref(d), ctypes.byref(out))
    if st != NTS_OK:
        raise NtsError(st, "nts_shard_linear_launch")
    return out


def nts_shard_linear_view(*, M: int, n_out: int, n_in: int, tp: int, rank: int, split: int,
                          ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0):
    """(elem_offset, rows, cols, row_stride) of the shard inside the full weight matrix."""
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    v = [ctypes.c_int64(0) for _ in range(4)]
    st = _lib.nts_shard_linear_view(ctypes.byref(d), *[ctypes.byref(x) for x in v])
    if st != NTS_OK:
        raise NtsError(st, "nts_shard_linear_view")
    return tuple(x.value for x in v)


def nts_shard_linear(ctx: int, X: int, W_full: int, Y: int, *, M: int, n_out: int, n_in: int, tp: int,
                     rank: int, split: int, ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0,
                     workspace: int = 0, workspace_bytes: int = 0, hip_stream: int = 0) -> None:
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    _check(_lib.nts_shard_linear(ctx, ctypes.byref(d), X, W_full, Y, workspace, workspace_bytes, hip_stream), ctx)


def nts_shard_linear_tune(ctx: int, X: int, W_list, Y: int, *, M: int, n_out: int, n_in: int, tp: int,
                          rank: int, split: int, ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0,
                          workspace: int = 0, workspace_bytes: int = 0, hip_stream: int = 0) -> "nts_linear_launch":
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    out = nts_linear_launch()
    ws = [W_list] if isinstance(W_list, int) else list(W_list)
    tab = (ctypes.c_void_p * len(ws))(*[int(w) for w in ws])
    _check(_lib.nts_shard_linear_tune(ctx, ctypes.byref(d), X, tab, len(ws), Y, workspace, workspace_bytes, hip_stream,
                                      ctypes.byref(out)), ctx)
    return out


def nts_shard_linear_tuned(ctx: int, *, M: int, n_out: int, n_in: int, tp: int, rank: int, split: int,
                           ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0) -> Optional["nts_linear_launch"]:
    """The configuration remembered for this shape, or None when it has not been tuned."""
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    out = nts_linear_launch()
    st = _lib.nts_shard_linear_tuned(ctx, ctypes.byref(d), ctypes.byref(out))
    if st == NTS_ERANGE:
        return None
    if st != NTS_OK:
        raise NtsError(st, "nts_shard_linear_tuned")
    return out


def nts_shard_linear_candidates(*, M: int, n_out: int, n_in: int, tp: int, rank: int, split: int,
                                ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0, max_out: int = 16):
    """The configurations the tuner would try (host arithmetic), the default first."""
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    out = (nts_linear_launch * max_out)()
    n = ctypes.c_int(0)
    st = _lib.nts_shard_linear_candidates(ctypes.byref(d), out, max_out, ctypes.byref(n))
    if st != NTS_OK:
        raise NtsError(st, "nts_shard_linear_candidates")
    return [out[i] for i in range(n.value)]


def nts_shard_linear_with(ctx: int, how: "nts_linear_launch", X: int, W_full: int, Y: int, *, M: int, n_out: int,
                          n_in: int, tp: int, rank: int, split: int, ldx: int = 0, ldw: int = 0, ldy: int = 0,
                          dtype: int = 0, workspace: int = 0, workspace_bytes: int = 0, hip_stream: int = 0) -> None:
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    _check(_lib.nts_shard_linear_with(ctx, ctypes.byref(d), ctypes.byref(how), X, W_full, Y, workspace, workspace_bytes,
                                      hip_stream), ctx)


def nts_shard_linear_remember(ctx: int, how: Optional["nts_linear_launch"], *, M: int, n_out: int, n_in: int, tp: int,
                              rank: int, split: int, ldx: int = 0, ldw: int = 0, ldy: int = 0, dtype: int = 0) -> None:
    d = _linear_desc(M, n_out, n_in, tp, rank, split, ldx, ldw, ldy, dtype)
    _check(_lib.nts_shard_linear_remember(ctx, ctypes.byref(d), ctypes.byref(how) if how is not None else None), ctx)


def nts_balanced_block(thp: float, thd: float, max_inst: int = 8) -> Tuple[int, int]:
    P, D = ctypes.c_int(), ctypes.c_int()
    st = _lib.nts_balanced_block(thp, thd, max_inst, ctypes.byref(P), ctypes.byref(D))
    if st != NTS_OK:
        raise NtsError(st, "nts_balanced_block")
    return P.value, D.value


def nts_goodput_efficiency(thp: float, tpi: int, thd: float, tpj: int, P: int, D: int, rps: float) -> float:
    ge = ctypes.c_double()
    st = _lib.nts_goodput_efficiency(thp, tpi, thd, tpj, P, D, rps, ctypes.byref(ge))
    if st != NTS_OK:
        raise NtsError(st, "nts_goodput_efficiency")
    return ge.value


def nts_plan_cluster(n_gpus: int, tiers: Sequence[Tuple[float, Sequence[float], Sequence[float]]],
                     max_inst: int = 8, max_out: int = 4096):
    """tiers: (rps, thp[4], thd[4]) per tier.  Returns (list of nts_alloc, gpus_left)."""
    arr = (nts_tier * max(1, len(tiers)))()
    for k, (rps, thp, thd) in enumerate(tiers):
        arr[k].rps = rps
        for i in range(4):
            arr[k].thp[i] = thp[i]
            arr[k].thd[i] = thd[i]
    out = (nts_alloc * max_out)()
    n, left = ctypes.c_int(), ctypes.c_int()
    st = _lib.nts_plan_cluster(n_gpus, len(tiers), arr, max_inst, out, max_out, ctypes.byref(n), ctypes.byref(left))
    if st != NTS_OK:
        raise NtsError(st, "nts_plan_cluster")
    return [out[i] for i in range(n.value)], left.value
