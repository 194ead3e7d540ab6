"""ctypes binding of the fp64 CPU oracle (oracle/ta_oracle.c).

Test infrastructure only.  Arrays are numpy: bf16 data is passed as uint16 bit
patterns, fp32 as float32, fp64 as float64; `as_oracle_array` converts a CPU
torch tensor without changing a bit.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_DT = {np.dtype(np.uint16): 0, np.dtype(np.float32): 1, np.dtype(np.float64): 2}
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if os.environ.get("TA_ORACLE_SANITIZED") == "1":   # the sanitizer run of the pins (tests/test_sanitized_oracle.py)
        path = _build.SAN_LIB
    elif not os.path.exists(_build.LIB) or \
            os.path.getmtime(_build.LIB) < os.path.getmtime(_build.SRC):
        _build.build()
    lib = ctypes.CDLL(path)
    c_int, c_i64, c_dbl, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    lib.ta_oracle_decode.argtypes = [c_int, c_int, c_int, c_int, c_i64, vp, vp, vp, c_int,
                                     c_dbl, vp, vp, vp, c_int]
    lib.ta_oracle_decode.restype = c_int
    lib.ta_oracle_max_threads.restype = c_int
    lib.ta_oracle_decode_causal.argtypes = [c_int, c_int, c_int, c_int, c_int, c_i64, vp, vp, vp, c_int,
                                            c_dbl, vp, vp, vp, c_int]
    lib.ta_oracle_decode_causal.restype = c_int
    lib.ta_oracle_energy_causal.argtypes = [c_int, c_i64, c_int, vp, vp, vp, c_int, c_dbl, vp]
    lib.ta_oracle_energy_causal.restype = c_dbl
    lib.ta_oracle_partial.argtypes = [c_int, vp, vp, vp, c_int, c_dbl, c_i64, c_i64, vp, vp, vp]
    lib.ta_oracle_partial.restype = c_int
    lib.ta_oracle_combine.argtypes = [c_int, c_int, vp, vp, vp, c_int, vp, c_int, vp, vp]
    lib.ta_oracle_combine.restype = c_int
    lib.ta_oracle_combine_alg3.argtypes = [c_int, c_int, vp, vp, vp, vp]
    lib.ta_oracle_combine_alg3.restype = c_int
    lib.ta_oracle_energy.argtypes = [c_int, c_i64, vp, vp, vp, c_int, c_dbl, vp]
    lib.ta_oracle_energy.restype = c_dbl
    lib.ta_oracle_recurrence.argtypes = [c_int, c_i64, vp, vp, vp, c_int, c_dbl, vp]
    lib.ta_oracle_recurrence.restype = c_int
    lib.ta_oracle_two_pass.argtypes = [c_int, vp, vp, vp, c_int, c_dbl, c_int, vp, vp, vp]
    lib.ta_oracle_two_pass.restype = c_int
    _lib = lib
    return lib


def as_oracle_array(x):
    """numpy view of a CPU torch tensor (bf16 -> uint16 bits) or numpy passthrough."""
    if isinstance(x, np.ndarray):
        return np.ascontiguousarray(x)
    import torch
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _same_dtype(*arrs):
    dts = {a.dtype for a in arrs}
    if len(dts) != 1 or arrs[0].dtype not in _DT:
        raise TypeError(f"q, K, V must share one of uint16(bf16)/float32/float64, got {dts}")
    return _DT[arrs[0].dtype]


def max_threads():
    return int(_load().ta_oracle_max_threads())


def decode(q, K, V, scale, valid_len=None, nthreads=None):
    """q [B,Hq,d], K,V [B,Hkv,N,d] -> (out [B,Hq,d] f64, lse [B,Hq] f64)."""
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    B, Hq, d = q.shape
    Bk, Hkv, N, dk = K.shape
    if (Bk, dk) != (B, d) or V.shape != K.shape or Hq % Hkv:
        raise ValueError("shape mismatch")
    vl = None
    if valid_len is not None:
        vl = np.ascontiguousarray(np.asarray(valid_len, dtype=np.int32))
        if vl.shape != (B,):
            raise ValueError("valid_len must be [B]")
    out = np.empty((B, Hq, d), np.float64)
    lse = np.empty((B, Hq), np.float64)
    nt = nthreads if nthreads is not None else max_threads()
    rc = lib.ta_oracle_decode(B, Hq, Hkv, d, N, _ptr(q), _ptr(K), _ptr(V), dt, float(scale),
                              _ptr(vl) if vl is not None else None, _ptr(out), _ptr(lse), int(nt))
    if rc:
        raise RuntimeError("ta_oracle_decode failed")
    return out, lse


def decode_causal(q, K, V, scale, valid_len=None, nthreads=None):
    """q [B,Sq,Hq,d], K,V [B,Hkv,N,d]; the last Sq cached keys are the query tokens' own,
    token t sees keys 0..L-Sq+t -> (out [B,Sq,Hq,d] f64, lse [B,Sq,Hq] f64)."""
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    B, Sq, Hq, d = q.shape
    Bk, Hkv, N, dk = K.shape
    if (Bk, dk) != (B, d) or V.shape != K.shape or Hq % Hkv:
        raise ValueError("shape mismatch")
    vl = None
    if valid_len is not None:
        vl = np.ascontiguousarray(np.asarray(valid_len, dtype=np.int32))
        if vl.shape != (B,):
            raise ValueError("valid_len must be [B]")
    out = np.empty((B, Sq, Hq, d), np.float64)
    lse = np.empty((B, Sq, Hq), np.float64)
    nt = nthreads if nthreads is not None else max_threads()
    rc = lib.ta_oracle_decode_causal(B, Sq, Hq, Hkv, d, N, _ptr(q), _ptr(K), _ptr(V), dt, float(scale),
                                     _ptr(vl) if vl is not None else None, _ptr(out), _ptr(lse), int(nt))
    if rc:
        raise RuntimeError("ta_oracle_decode_causal failed")
    return out, lse


def energy_causal(q, K, V, scale, zeta):
    """F_tot of Appendix C.1 for one head: q [Sq,d], K,V [L,d], zeta [Sq,d] f64."""
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    L, d = K.shape
    Sq = q.shape[0]
    zeta = np.ascontiguousarray(np.asarray(zeta, dtype=np.float64))
    if zeta.shape != (Sq, d):
        raise ValueError("zeta must be [Sq,d]")
    return float(lib.ta_oracle_energy_causal(d, L, Sq, _ptr(q), _ptr(K), _ptr(V), dt, float(scale), _ptr(zeta)))


def partial(q, K, V, scale, lo, hi):
    """One head: q [d], K,V [N,d]; chunk [lo,hi) -> (m, l, o[d])."""
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    N, d = K.shape
    if not (0 <= lo and hi <= N) or q.shape != (d,) or V.shape != K.shape:
        raise ValueError("bad chunk or shapes")
    m = np.empty(1, np.float64)
    l = np.empty(1, np.float64)
    o = np.empty(d, np.float64)
    rc = lib.ta_oracle_partial(d, _ptr(q), _ptr(K), _ptr(V), dt, float(scale), int(lo), int(hi),
                               _ptr(m), _ptr(l), _ptr(o))
    if rc:
        raise RuntimeError("ta_oracle_partial failed")
    return float(m[0]), float(l[0]), o


def flat_merges(P):
    """Merge list of the flat left-to-right P-way reduction into node 0."""
    return [(0, j) for j in range(1, P)], 0


def combine(m, l, o, merges=None, root=0):
    """m,l [P], o [P,d] (any float dtype, widened exactly) -> (out [d], lse)."""
    lib = _load()
    m = np.ascontiguousarray(np.asarray(m, dtype=np.float64))
    l = np.ascontiguousarray(np.asarray(l, dtype=np.float64))
    o = np.ascontiguousarray(np.asarray(o, dtype=np.float64))
    P, d = o.shape
    if merges is None:
        merges, root = flat_merges(P)
    mg = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    out = np.empty(d, np.float64)
    lse = np.empty(1, np.float64)
    rc = lib.ta_oracle_combine(P, d, _ptr(m), _ptr(l), _ptr(o), int(mg.shape[0]),
                               _ptr(mg) if mg.size else None, int(root), _ptr(out), _ptr(lse))
    if rc:
        raise RuntimeError("ta_oracle_combine failed")
    return out, float(lse[0])


def combine_alg3(o_norm, lse_j):
    lib = _load()
    o_norm = np.ascontiguousarray(np.asarray(o_norm, dtype=np.float64))
    lse_j = np.ascontiguousarray(np.asarray(lse_j, dtype=np.float64))
    P, d = o_norm.shape
    out = np.empty(d, np.float64)
    lse = np.empty(1, np.float64)
    rc = lib.ta_oracle_combine_alg3(P, d, _ptr(o_norm), _ptr(lse_j), _ptr(out), _ptr(lse))
    if rc:
        raise RuntimeError("ta_oracle_combine_alg3 failed")
    return out, float(lse[0])


def energy(q, K, V, scale, zeta):
    """F(zeta) of Observation 1 for one head: q [d], K,V [L,d], zeta [d] f64."""
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    L, d = K.shape
    zeta = np.ascontiguousarray(np.asarray(zeta, dtype=np.float64))
    if zeta.shape != (d,):
        raise ValueError("zeta must be [d]")
    return float(lib.ta_oracle_energy(d, L, _ptr(q), _ptr(K), _ptr(V), dt, float(scale), _ptr(zeta)))


def recurrence(q, K, V, scale):
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    L, d = K.shape
    out = np.empty(d, np.float64)
    rc = lib.ta_oracle_recurrence(d, L, _ptr(q), _ptr(K), _ptr(V), dt, float(scale), _ptr(out))
    if rc:
        raise RuntimeError("ta_oracle_recurrence failed")
    return out


def two_pass(q, K, V, scale, bounds):
    lib = _load()
    q, K, V = (as_oracle_array(a) for a in (q, K, V))
    dt = _same_dtype(q, K, V)
    L, d = K.shape
    bounds = np.ascontiguousarray(np.asarray(bounds, dtype=np.int64))
    p = bounds.shape[0] - 1
    out = np.empty(d, np.float64)
    lse = np.empty(1, np.float64)
    rc = lib.ta_oracle_two_pass(d, _ptr(q), _ptr(K), _ptr(V), dt, float(scale), p, _ptr(bounds),
                                _ptr(out), _ptr(lse))
    if rc:
        raise RuntimeError("ta_oracle_two_pass failed")
    return out, float(lse[0])
