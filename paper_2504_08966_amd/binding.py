"""ctypes binding of libpact.so: same entry-point names as include/pact.h, arguments are
torch tensors (device memory) and plain numbers.  No arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

PACT_F32, PACT_BF16 = 0, 1
PACT_FLAG_NO_MERGE = 1
PACT_FLAG_SCORE_NO_NORM = 2
PACT_FLAG_SCORE_NORM_ONLY = 4
PACT_FLAG_KEY_STATS = 8
REPORT_FIELDS = ("n_kept", "n_pruned", "n_centers", "n_reincorporated", "n_dropped", "rounds",
                 "dc_checked_pairs", "dc_near_ties", "refine_overflow", "zero_norm_seen", "max_key_distance",
                 "rho_rechecked", "rho_near_ties", "score_near_ties", "nonfinite_seen")
REPORT_INTS = 16
_REPORT_FLOAT = REPORT_FIELDS.index("max_key_distance")

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class PactError(RuntimeError):
    pass


class _Params(C.Structure):
    _fields_ = [("lambda_", C.c_float), ("d_c", C.c_float), ("d_n", C.c_float), ("alpha", C.c_float),
                ("fallback_T", C.c_int32), ("flags", C.c_uint32)]


@dataclass
class PactParams:
    lam: float
    d_c: float
    d_n: float = 2.0
    alpha: float = 1.5
    fallback_T: int = 10
    flags: int = 0

    def c(self) -> _Params:
        return _Params(self.lam, self.d_c, self.d_n, self.alpha, self.fallback_T, self.flags)


def lib_path() -> str:
    return os.path.join(_HERE, "libpact.so")


def load_library():
    """Loads libpact.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise PactError(f"{path} is missing: build it with `python -m paper_2504_08966_amd.build` "
                        "(or __graft_entry__.build()); there is no CPU or PyTorch fallback")
    lib = C.CDLL(path)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.pact_workspace_bytes.restype = sz
    lib.pact_workspace_bytes.argtypes = [i32, i32, i32, C.c_int, i32, i32]
    lib.pact_score.restype = C.c_int
    lib.pact_score.argtypes = [vp, C.c_int, i32, i32, vp, C.c_int, i32, i32, vp, C.c_int, i32, i32,
                               C.c_uint32, vp, vp, sz, vp]
    lib.pact_prune.restype = C.c_int
    lib.pact_prune.argtypes = [vp, i32, f32, vp, vp, vp, vp, sz, vp]
    lib.dbdpc_cluster.restype = C.c_int
    lib.dbdpc_cluster.argtypes = [vp, C.c_int, i32, i32, vp, vp, f32, f32, i32, vp, vp, vp, vp, vp,
                                  vp, sz, vp]
    lib.pact_reincorporate.restype = C.c_int
    lib.pact_reincorporate.argtypes = [vp, C.c_int, i32, i32, vp, vp, f32, f32, vp, vp, vp, sz, vp]
    lib.pact_merge.restype = C.c_int
    lib.pact_merge.argtypes = [vp, C.c_int, i32, i32, vp, vp, vp, C.c_uint32, vp, C.c_int, vp, vp, sz, vp]
    lib.pact_reduce.restype = C.c_int
    lib.pact_reduce.argtypes = [vp, C.c_int, i32, i32, vp, vp, C.c_int, i32, i32, vp, C.c_int, i32, i32,
                                C.POINTER(_Params), vp, vp, vp, vp, vp, vp, C.c_int, vp, vp, vp, sz, vp]
    lib.pact_reduce_static.restype = C.c_int
    lib.pact_reduce_static.argtypes = [vp, C.c_int, i32, i32, vp, vp, C.c_int, i32, i32, vp, C.c_int, i32, i32,
                                       C.POINTER(_Params), vp, vp, vp, vp, vp, vp, C.c_int, vp, vp, vp]
    lib.pact_reduce_varlen.restype = C.c_int
    lib.pact_reduce_varlen.argtypes = [vp, C.c_int, i32, vp, vp, C.c_int, i32, i32, vp, C.c_int, i32, i32,
                                       C.POINTER(i32), i32, C.POINTER(_Params), vp, vp, vp, vp, vp, vp,
                                       C.c_int, vp, vp, vp, sz, vp]
    lib.pact_attention_handoff.restype = C.c_int
    lib.pact_attention_handoff.argtypes = [vp, vp, vp, vp, C.POINTER(i32), i32, i32, vp, vp, vp]
    lib.pact_calibration_copy.restype = C.c_int
    lib.pact_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.pact_plan_workgroups.restype = C.c_int
    lib.pact_plan_workgroups.argtypes = [C.POINTER(i32), i32, C.POINTER(C.c_uint16), C.POINTER(C.c_uint16)]
    lib.pact_profile_enable.restype = C.c_int
    lib.pact_profile_enable.argtypes = [C.c_int]
    lib.pact_profile_reset.restype = C.c_int
    lib.pact_profile_reset.argtypes = []
    lib.pact_profile_read.restype = C.c_int
    lib.pact_profile_read.argtypes = [C.POINTER(C.c_char_p), C.POINTER(C.c_float), i32]
    lib.pact_strerror.restype = C.c_char_p
    lib.pact_strerror.argtypes = [C.c_int]
    _LIB = lib
    return lib


def pact_strerror(status: int) -> str:
    return load_library().pact_strerror(status).decode()


def _check(status: int, what: str):
    if status != 0:
        raise PactError(f"{what} failed with status {status}: {pact_strerror(status)}")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PACT_F32
    if t.dtype == torch.bfloat16:
        return PACT_BF16
    raise PactError(f"unsupported dtype {t.dtype}")


def _out_dt(dtype) -> int:
    return PACT_BF16 if dtype == torch.bfloat16 else PACT_F32


def _p(t):
    """Device address of a tensor (None -> NULL).  The library reads rows back to back: a view with
    other strides would be read as if it were contiguous, so it is refused here."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise PactError("tensor arguments must be contiguous (row-major)")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def pact_workspace_bytes(n_max: int, batch: int, dk: int, n_q: int, d_h: int, key_dtype=PACT_F32) -> int:
    """key_dtype: PACT_F32 / PACT_BF16 or a torch dtype (fp32 keys, the default, need the larger workspace)."""
    if not isinstance(key_dtype, int):
        key_dtype = PACT_BF16 if key_dtype == torch.bfloat16 else PACT_F32
    return int(load_library().pact_workspace_bytes(n_max, batch, dk, key_dtype, n_q, d_h))


def alloc_workspace(n_max: int, batch: int, dk: int, n_q: int, d_h: int, device="cuda", key_dtype=PACT_F32) -> torch.Tensor:
    nbytes = pact_workspace_bytes(n_max, batch, dk, n_q, d_h, key_dtype)
    if nbytes == 0:
        raise PactError("pact_workspace_bytes: arguments out of range")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def new_report(batch: int = 1, device="cuda") -> torch.Tensor:
    return torch.zeros(batch, REPORT_INTS, dtype=torch.int32, device=device)


def read_report(rep: torch.Tensor):
    """Host copy of the device-side report(s) (synchronises the current stream)."""
    hc = rep.cpu()
    h = hc.tolist()
    out = [dict(zip(REPORT_FIELDS, row)) for row in h]
    fl = hc.view(torch.float32)
    for b, d in enumerate(out):
        d["max_key_distance"] = float(fl[b, _REPORT_FLOAT])
    return out[0] if len(out) == 1 else out


def pact_score(hidden, keys_pre, q, n_kv: int, d_h: int, n_q: int, ws=None, flags: int = 0):
    n, h = hidden.shape
    ws = ws if ws is not None else alloc_workspace(n, 1, n_kv * d_h, n_q, d_h, hidden.device)
    scores = torch.empty(n, dtype=torch.float32, device=hidden.device)
    _check(load_library().pact_score(_p(hidden), _dt(hidden), n, h, _p(keys_pre), _dt(keys_pre), n_kv, d_h,
                                     _p(q), _dt(q), q.shape[0], n_q, flags, _p(scores), _p(ws), ws.numel(),
                                     _stream()), "pact_score")
    return scores


def pact_prune(scores, lam: float, rep=None, ws=None):
    n = scores.shape[0]
    dev = scores.device
    kept = torch.empty(n, dtype=torch.int32, device=dev)
    pruned = torch.empty(n, dtype=torch.int32, device=dev)
    rep = rep if rep is not None else new_report(1, dev)
    _check(load_library().pact_prune(_p(scores), n, lam, _p(kept), _p(pruned), _p(rep), _p(ws),
                                     0 if ws is None else ws.numel(), _stream()), "pact_prune")
    return kept, pruned, rep


def dbdpc_cluster(keys, d_c: float, d_n: float = 2.0, fallback_T: int = 10, idx=None, n_idx_dev=None,
                  rep=None, ws=None, want_rho=False, want_rank=False):
    n, dk = keys.shape
    dev = keys.device
    ws = ws if ws is not None else alloc_workspace(n, 1, dk, 1, 1, dev, keys.dtype)
    center_idx = torch.empty(n, dtype=torch.int32, device=dev)
    cluster_id = torch.empty(n, dtype=torch.int32, device=dev)
    rep = rep if rep is not None else new_report(1, dev)
    rho = torch.zeros(n, dtype=torch.float64, device=dev) if want_rho else None
    rank = torch.zeros(n, dtype=torch.int32, device=dev) if want_rank else None
    _check(load_library().dbdpc_cluster(_p(keys), _dt(keys), n, dk, _p(idx), _p(n_idx_dev), d_c, d_n,
                                        fallback_T, _p(center_idx), _p(cluster_id), _p(rep), _p(rho),
                                        _p(rank), _p(ws), ws.numel(), _stream()), "dbdpc_cluster")
    return dict(center_idx=center_idx, cluster_id=cluster_id, rep=rep, rho=rho, rank=rank)


def pact_reincorporate(keys, pruned_idx, center_idx, d_c: float, alpha: float, cluster_id, rep, ws=None):
    n, dk = keys.shape
    ws = ws if ws is not None else alloc_workspace(n, 1, dk, 1, 1, keys.device, keys.dtype)
    _check(load_library().pact_reincorporate(_p(keys), _dt(keys), n, dk, _p(pruned_idx), _p(center_idx), d_c,
                                             alpha, _p(cluster_id), _p(rep), _p(ws), ws.numel(), _stream()),
           "pact_reincorporate")
    return cluster_id, rep


def pact_merge(hidden, cluster_id, rep, center_idx=None, flags: int = 0, out_dtype=torch.float32, ws=None):
    n, h = hidden.shape
    dev = hidden.device
    ws = ws if ws is not None else alloc_workspace(n, 1, 8, 1, 1, dev)
    merged = torch.empty(n, h, dtype=out_dtype, device=dev)
    counts = torch.empty(n, dtype=torch.int32, device=dev)
    _check(load_library().pact_merge(_p(hidden), _dt(hidden), n, h, _p(cluster_id), _p(center_idx), _p(rep),
                                     flags, _p(merged), _out_dt(out_dtype), _p(counts), _p(ws), ws.numel(),
                                     _stream()), "pact_merge")
    return merged, counts


def _alloc_outputs(total, h, batch, out_dtype, dev):
    i32 = dict(dtype=torch.int32, device=dev)
    return dict(scores=torch.empty(total, dtype=torch.float32, device=dev),
                kept_idx=torch.empty(total, **i32), pruned_idx=torch.empty(total, **i32),
                center_idx=torch.empty(total, **i32), cluster_id=torch.empty(total, **i32),
                merged=torch.empty(total, h, dtype=out_dtype, device=dev),
                cluster_counts=torch.empty(total, **i32), rep=new_report(batch, dev))


def pact_reduce(hidden, keys_pre, keys, q, n_kv: int, d_h: int, n_q: int, params: PactParams,
                out_dtype=torch.float32, ws=None, out=None):
    """Alg. 3 for one sample.  Returns the dict of output tensors (worst-case sized; the
    valid lengths are in out['rep'], on the device)."""
    n, h = hidden.shape
    dev = hidden.device
    ws = ws if ws is not None else alloc_workspace(n, 1, n_kv * d_h, n_q, d_h, dev, keys.dtype)
    o = out if out is not None else _alloc_outputs(n, h, 1, out_dtype, dev)
    pc = params.c()
    _check(load_library().pact_reduce(
        _p(hidden), _dt(hidden), n, h, _p(keys_pre), _p(keys), _dt(keys), n_kv, d_h, _p(q), _dt(q),
        q.shape[0], n_q, C.byref(pc), _p(o["scores"]), _p(o["kept_idx"]), _p(o["pruned_idx"]),
        _p(o["center_idx"]), _p(o["cluster_id"]), _p(o["merged"]), _out_dt(o["merged"].dtype),
        _p(o["cluster_counts"]), _p(o["rep"]), _p(ws), ws.numel(), _stream()), "pact_reduce")
    return o


def pact_reduce_static(hidden, keys_pre, keys, q, n_kv: int, d_h: int, n_q: int, params: PactParams, out):
    """pact_reduce on the library's own scratch array: no workspace argument, and nothing is
    allocated here either - `out` is a dict of output tensors as pact_reduce returns it."""
    n, h = hidden.shape
    pc = params.c()
    _check(load_library().pact_reduce_static(
        _p(hidden), _dt(hidden), n, h, _p(keys_pre), _p(keys), _dt(keys), n_kv, d_h, _p(q), _dt(q),
        q.shape[0], n_q, C.byref(pc), _p(out["scores"]), _p(out["kept_idx"]), _p(out["pruned_idx"]),
        _p(out["center_idx"]), _p(out["cluster_id"]), _p(out["merged"]), _out_dt(out["merged"].dtype),
        _p(out["cluster_counts"]), _p(out["rep"]), _stream()), "pact_reduce_static")
    return out


def new_outputs(total: int, h: int, batch: int = 1, out_dtype=torch.float32, device="cuda"):
    """Output tensors of pact_reduce / pact_reduce_varlen, sized for the worst case."""
    return _alloc_outputs(total, h, batch, out_dtype, device)


def pact_reduce_varlen(hidden, keys_pre, keys, q, n_kv: int, d_h: int, n_q: int, cu_seqlens, params,
                       out_dtype=torch.float32, ws=None, out=None):
    """Alg. 3 for a ragged batch; cu_seqlens is a host list of batch+1 ints, params a list of
    PactParams (one per sample)."""
    total, h = hidden.shape
    batch = len(cu_seqlens) - 1
    dev = hidden.device
    n_max = max(cu_seqlens[b + 1] - cu_seqlens[b] for b in range(batch))
    ws = ws if ws is not None else alloc_workspace(n_max, batch, n_kv * d_h, n_q, d_h, dev, keys.dtype)
    o = out if out is not None else _alloc_outputs(total, h, batch, out_dtype, dev)
    cu = (C.c_int32 * (batch + 1))(*cu_seqlens)
    pa = (_Params * batch)(*[p.c() for p in params])
    _check(load_library().pact_reduce_varlen(
        _p(hidden), _dt(hidden), h, _p(keys_pre), _p(keys), _dt(keys), n_kv, d_h, _p(q), _dt(q),
        q.shape[0], n_q, cu, batch, pa, _p(o["scores"]), _p(o["kept_idx"]), _p(o["pruned_idx"]),
        _p(o["center_idx"]), _p(o["cluster_id"]), _p(o["merged"]), _out_dt(o["merged"].dtype),
        _p(o["cluster_counts"]), _p(o["rep"]), _p(ws), ws.numel(), _stream()), "pact_reduce_varlen")
    return o


def pact_attention_handoff(center_idx, cluster_counts, rep, positions=None, cu_seqlens=None):
    """Positions of the merged tokens (their centres') and log cluster sizes (Eq. 11); entries
    0..n_centers-1 of each sample are written."""
    total = center_idx.numel()
    dev = center_idx.device
    pos_out = torch.zeros(total, dtype=torch.int32, device=dev)
    logw = torch.zeros(total, dtype=torch.float32, device=dev)
    if cu_seqlens is None:
        cu, batch = None, 1
    else:
        batch = len(cu_seqlens) - 1
        cu = (C.c_int32 * (batch + 1))(*cu_seqlens)
    _check(load_library().pact_attention_handoff(_p(center_idx), _p(cluster_counts), _p(rep), _p(positions), cu,
                                                 batch, total, _p(pos_out), _p(logw), _stream()),
           "pact_attention_handoff")
    return pos_out, logw


def pact_calibration_copy(dst, src):
    """Copy src into dst (same byte size) with the library's plain copy kernel."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load_library().pact_calibration_copy(_p(dst), _p(src), nbytes, _stream()), "pact_calibration_copy")


def pact_plan_workgroups(tiles):
    """Diagnostic (host only): (wg_map [256], wg_count [batch]) for samples expected to have `tiles` tiles each."""
    batch = len(tiles)
    arr = (C.c_int32 * batch)(*[int(x) for x in tiles])
    wg_map = (C.c_uint16 * 256)()
    wg_count = (C.c_uint16 * batch)()
    _check(load_library().pact_plan_workgroups(arr, batch, wg_map, wg_count), "pact_plan_workgroups")
    return list(wg_map), list(wg_count)


def pact_profile_enable(on: bool):
    load_library().pact_profile_enable(1 if on else 0)


def pact_profile_reset():
    load_library().pact_profile_reset()


def pact_profile_read(max_records: int = 4096):
    names = (C.c_char_p * max_records)()
    ms = (C.c_float * max_records)()
    n = load_library().pact_profile_read(names, ms, max_records)
    if n < 0:
        raise PactError("pact_profile_read failed")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]
