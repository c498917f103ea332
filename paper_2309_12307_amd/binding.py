"""ctypes binding of libs2attn.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (or raw device
pointers), passes their addresses and the current HIP stream to the C ABI of
include/s2attn.h, and raises on a non-zero return code.  There is no fallback of
any kind: if the shared library has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("S2ATTN_LIB", os.path.join(_HERE, "libs2attn.so"))

BF16, F32 = 0, 1
SHIFT_SECOND_HALF, SHIFT_NONE, SHIFT_ALL = 0, 1, 2
WRAP_JOINT, WRAP_SPLIT = 0, 2
BWD_AUTO, BWD_RECOMPUTE, BWD_STORED_DS = 0, 1, 2

EXPORTS = [
    "s2attn_check_args", "s2attn_bwd_workspace_bytes", "s2attn_fwd", "s2attn_bwd",
    "s2attn_fwd_f32", "s2attn_bwd_f32", "s2attn_fwd_ex", "s2attn_bwd_ex",
    "s2attn_strerror", "s2attn_effective_flops", "s2attn_bwd_ex_marked",
    "s2attn_bwd_workspace_bytes_ex", "s2attn_bwd_ex_static",
]


class S2AttnParams(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("o", ctypes.c_void_p), ("lse", ctypes.c_void_p), ("dout", ctypes.c_void_p),
        ("dq", ctypes.c_void_p), ("dk", ctypes.c_void_p), ("dv", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("B", ctypes.c_int), ("N", ctypes.c_int), ("H", ctypes.c_int),
        ("Hkv", ctypes.c_int), ("D", ctypes.c_int), ("G", ctypes.c_int),
        ("dtype", ctypes.c_int), ("shift", ctypes.c_int), ("shift_rule", ctypes.c_int),
        ("wrap_variant", ctypes.c_int), ("scale", ctypes.c_float),
        ("q_strides", ctypes.c_longlong * 3), ("k_strides", ctypes.c_longlong * 3),
        ("v_strides", ctypes.c_longlong * 3), ("dq_strides", ctypes.c_longlong * 3),
        ("dk_strides", ctypes.c_longlong * 3), ("dv_strides", ctypes.c_longlong * 3),
        ("heads_total", ctypes.c_int), ("head_offset", ctypes.c_int), ("bwd_algo", ctypes.c_int),
    ]


class S2AttnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"s2attn error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Opens libs2attn.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2309_12307_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.s2attn_check_args.argtypes = [ctypes.POINTER(S2AttnParams), i]
        L.s2attn_check_args.restype = i
        L.s2attn_bwd_workspace_bytes.argtypes = [i] * 7
        L.s2attn_bwd_workspace_bytes.restype = sz
        L.s2attn_bwd_workspace_bytes_ex.argtypes = [ctypes.POINTER(S2AttnParams)]
        L.s2attn_bwd_workspace_bytes_ex.restype = sz
        for name in ("s2attn_fwd", "s2attn_fwd_f32"):
            f = getattr(L, name)
            f.argtypes = [vp] * 5 + [i] * 6 + [vp]
            f.restype = i
        for name in ("s2attn_bwd", "s2attn_bwd_f32"):
            f = getattr(L, name)
            f.argtypes = [vp] * 9 + [vp, sz] + [i] * 6 + [vp]
            f.restype = i
        for name in ("s2attn_fwd_ex", "s2attn_bwd_ex", "s2attn_bwd_ex_static"):
            f = getattr(L, name)
            f.argtypes = [ctypes.POINTER(S2AttnParams), vp]
            f.restype = i
        L.s2attn_bwd_ex_marked.argtypes = [ctypes.POINTER(S2AttnParams), vp, ctypes.POINTER(vp)]
        L.s2attn_bwd_ex_marked.restype = i
        L.s2attn_strerror.argtypes = [i]
        L.s2attn_strerror.restype = ctypes.c_char_p
        L.s2attn_effective_flops.argtypes = [i] * 6
        L.s2attn_effective_flops.restype = ctypes.c_double
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().s2attn_strerror(code).decode()


def _check(code: int) -> None:
    if code != 0:
        raise S2AttnError(code, strerror(code))


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dims(q, k):
    B, N, H, D = q.shape
    Hkv = k.shape[2]
    return B, N, H, Hkv, D


def _require_contiguous(*ts):
    for t in ts:
        if t is not None and not t.is_contiguous():
            raise ValueError("s2attn tensors must be contiguous")


def bwd_workspace_bytes(B, N, H, Hkv, D, G, dtype=BF16) -> int:
    return int(lib().s2attn_bwd_workspace_bytes(B, N, H, Hkv, D, G, dtype))


def bwd_workspace_bytes_ex(p: "S2AttnParams") -> int:
    """Workspace size for a parameter block (accounts for its shift rule and head sharding)."""
    return int(lib().s2attn_bwd_workspace_bytes_ex(ctypes.byref(p)))


def effective_flops(B, N, H, D, G, which: int = 2) -> float:
    return float(lib().s2attn_effective_flops(B, N, H, D, G, which))


def make_params(q, k, v, o, lse, G, dout=None, dq=None, dk=None, dv=None, workspace=None,
                shift=-1, shift_rule=SHIFT_SECOND_HALF, wrap_variant=WRAP_JOINT, scale=0.0,
                dtype=None, dims=None, strided=False, heads_total=0, head_offset=0,
                bwd_algo=BWD_AUTO) -> S2AttnParams:
    """strided=True takes the {batch, token, head} strides of q, k, v (and dq, dk, dv) from
    the tensors themselves, so views into a packed (B, N, 3, H, D) tensor can be passed."""
    if dims is None:
        B, N, H, Hkv, D = _dims(q, k)
    else:
        B, N, H, Hkv, D = dims
    p = S2AttnParams()
    p.q, p.k, p.v, p.o, p.lse = _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse)
    p.dout, p.dq, p.dk, p.dv = _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv)
    p.workspace = _ptr(workspace)
    p.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    p.B, p.N, p.H, p.Hkv, p.D, p.G = B, N, H, Hkv, D, G
    p.dtype = _dtype_code(q) if dtype is None else dtype
    p.shift, p.shift_rule, p.wrap_variant, p.scale = shift, shift_rule, wrap_variant, scale
    p.heads_total, p.head_offset, p.bwd_algo = heads_total, head_offset, bwd_algo
    if strided:
        for name, t in (("q", q), ("k", k), ("v", v), ("dq", dq), ("dk", dk), ("dv", dv)):
            if t is None or isinstance(t, int):
                continue
            if t.stride(3) != 1:
                raise ValueError("the head-dim axis must be contiguous")
            setattr(p, name + "_strides", (ctypes.c_longlong * 3)(t.stride(0), t.stride(1), t.stride(2)))
    return p


def check_args(p: S2AttnParams, backward: bool) -> int:
    return int(lib().s2attn_check_args(ctypes.byref(p), 1 if backward else 0))


def s2attn_fwd(q, k, v, o, lse, G, stream=None) -> None:
    """o, lse <- S2-Attn(q, k, v) with the published defaults.  bf16 or fp32 tensors."""
    _require_contiguous(q, k, v, o, lse)
    B, N, H, Hkv, D = _dims(q, k)
    f = lib().s2attn_fwd if _dtype_code(q) == BF16 else lib().s2attn_fwd_f32
    _check(f(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, N, H, Hkv, D, G, _stream(stream)))


def s2attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, workspace, G, stream=None) -> None:
    """dq, dk, dv <- gradients of sum(o * dout); workspace is a uint8 device tensor."""
    _require_contiguous(q, k, v, o, dout, lse, dq, dk, dv, workspace)
    B, N, H, Hkv, D = _dims(q, k)
    f = lib().s2attn_bwd if _dtype_code(q) == BF16 else lib().s2attn_bwd_f32
    _check(f(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv),
             _ptr(workspace), workspace.numel() * workspace.element_size(),
             B, N, H, Hkv, D, G, _stream(stream)))


def s2attn_fwd_ex(p: S2AttnParams, stream=None) -> None:
    _check(lib().s2attn_fwd_ex(ctypes.byref(p), _stream(stream)))


def s2attn_bwd_ex(p: S2AttnParams, stream=None) -> None:
    _check(lib().s2attn_bwd_ex(ctypes.byref(p), _stream(stream)))


STATIC_SCRATCH_BYTES = 16 << 20


def s2attn_bwd_ex_static(p: S2AttnParams, stream=None) -> None:
    """s2attn_bwd_ex on the library's static scratch array: no workspace, no allocation."""
    _check(lib().s2attn_bwd_ex_static(ctypes.byref(p), _stream(stream)))


def s2attn_bwd_ex_marked(p: S2AttnParams, events, stream=None) -> None:
    """events: sequence of four raw hipEvent_t handles (ints) or None entries."""
    arr = (ctypes.c_void_p * 4)(*[e if e else None for e in events])
    _check(lib().s2attn_bwd_ex_marked(ctypes.byref(p), _stream(stream), arr))
