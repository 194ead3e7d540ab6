"""ctypes binding of libtree_attn.so (declarations: include/tree_attn.h).

The `ta_*` functions mirror the C entry points one to one (raw pointers in,
status out).  `decode`, `decode_partial` and `tree_combine` are conveniences
that take torch tensors, allocate the outputs with torch and pass the current
torch stream; they add no arithmetic.
"""
import ctypes
import os

TA_BF16, TA_F32 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtree_attn.so")
_lib = None


class TAError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__(f"{where}: {ta_status_string(code)} (status {int(code)})")


class Problem(ctypes.Structure):
    """struct ta_problem"""
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("N", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_n", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_n", ctypes.c_int64),
        ("qkv_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("valid_len", ctypes.c_void_p),
        ("Sq", ctypes.c_int32),
    ]


def lib_path():
    return _LIB_PATH


def load():
    """Load the HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2408_04093_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    pp = ctypes.POINTER(Problem)
    lib.ta_status_string.argtypes = [ctypes.c_int]
    lib.ta_status_string.restype = ctypes.c_char_p
    lib.ta_suggest_chunks.argtypes = [pp]
    lib.ta_suggest_chunks.restype = i32
    lib.ta_workspace_bytes.argtypes = [pp, i32]
    lib.ta_workspace_bytes.restype = ctypes.c_size_t
    lib.ta_decode_partial.argtypes = [pp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.ta_decode_partial.restype = ctypes.c_int
    lib.ta_tree_combine.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp]
    lib.ta_tree_combine.restype = ctypes.c_int
    lib.ta_decode.argtypes = [pp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    lib.ta_decode.restype = ctypes.c_int
    lib.ta_decode_noalloc.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.ta_decode_noalloc.restype = ctypes.c_int
    lib.ta_energy.argtypes = [pp, vp, vp, vp, ctypes.c_size_t, vp, vp]
    lib.ta_energy.restype = ctypes.c_int
    lib.ta_decode_two_pass.argtypes = [pp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    lib.ta_decode_two_pass.restype = ctypes.c_int
    _lib = lib
    return lib


# ------------------------------------------------------------------ raw C ABI
def ta_status_string(code):
    return load().ta_status_string(int(code)).decode()


def ta_suggest_chunks(problem):
    return int(load().ta_suggest_chunks(ctypes.byref(problem)))


def ta_workspace_bytes(problem, P):
    return int(load().ta_workspace_bytes(ctypes.byref(problem), int(P)))


def ta_decode_partial(problem, q, K, V, P, chunk_bounds, part_m, part_l, part_o, stream):
    """All of q..part_o are integer device addresses (chunk_bounds may be None/0)."""
    return int(load().ta_decode_partial(ctypes.byref(problem), q, K, V, int(P), chunk_bounds or None,
                                        part_m, part_l, part_o, stream or None))


def ta_tree_combine(B, Hq, d, P, part_m, part_l, part_o, out, out_dtype, lse, stream):
    return int(load().ta_tree_combine(int(B), int(Hq), int(d), int(P), part_m, part_l, part_o,
                                      out, int(out_dtype), lse, stream or None))


def ta_decode(problem, q, K, V, workspace, workspace_bytes, out, lse, stream):
    return int(load().ta_decode(ctypes.byref(problem), q, K, V, workspace, int(workspace_bytes),
                                out, lse, stream or None))


def ta_decode_noalloc(problem, q, K, V, out, lse, stream):
    return int(load().ta_decode_noalloc(ctypes.byref(problem), q, K, V, out, lse, stream or None))


def ta_energy(problem, q, K, workspace, workspace_bytes, lse, stream):
    return int(load().ta_energy(ctypes.byref(problem), q, K, workspace, int(workspace_bytes), lse, stream or None))


def ta_decode_two_pass(problem, q, K, V, workspace, workspace_bytes, out, lse, stream):
    return int(load().ta_decode_two_pass(ctypes.byref(problem), q, K, V, workspace, int(workspace_bytes),
                                         out, lse, stream or None))


# ------------------------------------------------------------------ torch conveniences
def _dt(t):
    import torch
    if t.dtype == torch.bfloat16:
        return TA_BF16
    if t.dtype == torch.float32:
        return TA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_problem(q, K, V, scale, valid_len=None, out_dtype=None):
    """Describe torch tensors q [B,Hq,d] or [B,Sq,Hq,d], K,V [B,Hkv,N,d] (last dim contiguous)."""
    Sq = q.shape[1] if q.dim() == 4 else 1
    B, Hq, d = q.shape[0], q.shape[-2], q.shape[-1]
    _, Hkv, N, _ = K.shape
    if not q.is_contiguous() or K.stride(3) != 1 or V.stride(3) != 1:
        raise ValueError("q must be contiguous and K, V must have unit innermost stride")
    if K.shape != V.shape or K.shape[0] != B or K.shape[3] != d or not (q.dtype == K.dtype == V.dtype):
        raise ValueError("q, K, V shapes or dtypes disagree")
    if valid_len is not None:
        import torch
        if valid_len.dtype != torch.int32 or tuple(valid_len.shape) != (B,) or not valid_len.is_contiguous():
            raise ValueError("valid_len must be a contiguous int32 tensor of shape [B]")
    if not (q.is_cuda and K.is_cuda and V.is_cuda) or not (q.device == K.device == V.device) or \
            (valid_len is not None and valid_len.device != q.device):
        raise ValueError("q, K, V (and valid_len) must be device tensors on one GPU: their addresses are "
                         "dereferenced there")
    p = Problem()
    p.B, p.Hq, p.Hkv, p.d, p.N = B, Hq, Hkv, d, N
    p.k_stride_b, p.k_stride_h, p.k_stride_n = K.stride(0), K.stride(1), K.stride(2)
    p.v_stride_b, p.v_stride_h, p.v_stride_n = V.stride(0), V.stride(1), V.stride(2)
    p.qkv_dtype = _dt(q)
    p.out_dtype = p.qkv_dtype if out_dtype is None else out_dtype
    p.scale = float(scale)
    p.valid_len = valid_len.data_ptr() if valid_len is not None else None
    p.Sq = Sq
    return p


def decode_partial(q, K, V, scale, P, valid_len=None, chunk_bounds=None):
    """-> (part_m [B,Hq,P], part_l [B,Hq,P], part_o [B,Hq,P,d]) fp32 device tensors."""
    import torch
    p = make_problem(q, K, V, scale, valid_len)
    lead, d = tuple(q.shape[:-1]), q.shape[-1]          # (B,Hq) or (B,Sq,Hq)
    part_m = torch.empty(lead + (P,), dtype=torch.float32, device=q.device)
    part_l = torch.empty_like(part_m)
    part_o = torch.empty(lead + (P, d), dtype=torch.float32, device=q.device)
    rc = ta_decode_partial(p, q.data_ptr(), K.data_ptr(), V.data_ptr(), P,
                           chunk_bounds.data_ptr() if chunk_bounds is not None else None,
                           part_m.data_ptr(), part_l.data_ptr(), part_o.data_ptr(), _stream())
    if rc:
        raise TAError(rc, "ta_decode_partial")
    return part_m, part_l, part_o


def tree_combine(part_m, part_l, part_o, out_dtype=TA_F32):
    """part_o [B,Hq,P,d] or [B,Sq,Hq,P,d] -> (out [..,d], lse [..]) with the same leading axes."""
    import torch
    lead, P, d = tuple(part_o.shape[:-2]), part_o.shape[-2], part_o.shape[-1]
    B, Hq = lead[0], int(torch.Size(lead[1:]).numel())
    out = torch.empty(lead + (d,), dtype=torch.bfloat16 if out_dtype == TA_BF16 else torch.float32,
                      device=part_o.device)
    lse = torch.empty(lead, dtype=torch.float32, device=part_o.device)
    rc = ta_tree_combine(B, Hq, d, P, part_m.data_ptr(), part_l.data_ptr(), part_o.data_ptr(),
                         out.data_ptr(), out_dtype, lse.data_ptr(), _stream())
    if rc:
        raise TAError(rc, "ta_tree_combine")
    return out, lse


def decode(q, K, V, scale, valid_len=None, out_dtype=None, workspace=None):
    """-> (out [B,Hq,d], lse [B,Hq]); `workspace` (uint8 device tensor) is reused if given."""
    import torch
    p = make_problem(q, K, V, scale, valid_len, out_dtype)
    lead, d = tuple(q.shape[:-1]), q.shape[-1]
    need = ta_workspace_bytes(p, ta_suggest_chunks(p))
    if need == 0:
        raise TAError(load().ta_decode(ctypes.byref(p), None, None, None, None, 0, None, None, None),
                      "ta_decode")
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    out = torch.empty(lead + (d,), dtype=torch.bfloat16 if p.out_dtype == TA_BF16 else torch.float32,
                      device=q.device)
    lse = torch.empty(lead, dtype=torch.float32, device=q.device)
    rc = ta_decode(p, q.data_ptr(), K.data_ptr(), V.data_ptr(), workspace.data_ptr(), workspace.numel(),
                   out.data_ptr(), lse.data_ptr(), _stream())
    if rc:
        raise TAError(rc, "ta_decode")
    return out, lse


def energy(q, K, scale, valid_len=None):
    """lse [B,Hq] (or [B,Sq,Hq]) = logsumexp of the scaled scores; reads K only."""
    import torch
    p = make_problem(q, K, K, scale, valid_len)
    need = ta_workspace_bytes(p, ta_suggest_chunks(p))
    workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    lse = torch.empty(tuple(q.shape[:-1]), dtype=torch.float32, device=q.device)
    rc = ta_energy(p, q.data_ptr(), K.data_ptr(), workspace.data_ptr(), workspace.numel(), lse.data_ptr(), _stream())
    if rc:
        raise TAError(rc, "ta_energy")
    return lse


def decode_two_pass(q, K, V, scale, valid_len=None, out_dtype=None):
    """Energy pass then gradient pass (Algorithms 1 and 2) -> (out, lse), same shapes as decode()."""
    import torch
    p = make_problem(q, K, V, scale, valid_len, out_dtype)
    need = ta_workspace_bytes(p, ta_suggest_chunks(p))
    workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    out = torch.empty(tuple(q.shape), dtype=torch.bfloat16 if p.out_dtype == TA_BF16 else torch.float32,
                      device=q.device)
    lse = torch.empty(tuple(q.shape[:-1]), dtype=torch.float32, device=q.device)
    rc = ta_decode_two_pass(p, q.data_ptr(), K.data_ptr(), V.data_ptr(), workspace.data_ptr(), workspace.numel(),
                            out.data_ptr(), lse.data_ptr(), _stream())
    if rc:
        raise TAError(rc, "ta_decode_two_pass")
    return out, lse
