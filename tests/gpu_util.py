"""Helpers for the GPU parity tests: move seeded inputs to the device, run the HIP
path through the C ABI (via the ctypes binding) and bring the results back."""
import numpy as np
import torch

from paper_2309_12307_amd import binding


def to_dev(x: np.ndarray, bits: np.ndarray | None = None):
    if bits is not None:
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def run_hip(inp: dict, G: int, dtype: str, backward=True, ws_bytes=None, **ex):
    """inp: dict from inputs.make_inputs.  Returns dict of numpy float32 arrays
    o, lse, dq, dk, dv (gradients only when backward).  Extra keyword arguments
    (shift, shift_rule, wrap_variant, scale, bwd_algo) go through the *_ex entry points.
    ws_bytes: workspace size to pass instead of what the library asks for; a callable gets
    the library's size for the recomputing backward (the row terms) and the size it asks for."""
    bf = dtype == "bf16"
    q = to_dev(inp["q"], inp.get("q_bits") if bf else None)
    k = to_dev(inp["k"], inp.get("k_bits") if bf else None)
    v = to_dev(inp["v"], inp.get("v_bits") if bf else None)
    do = to_dev(inp["do"], inp.get("do_bits") if bf else None)
    B, N, H, D = q.shape
    Hkv = k.shape[2]
    o = torch.full_like(q, float("nan"))
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    if ex:
        p = binding.make_params(q, k, v, o, lse, G, **ex)
        binding.s2attn_fwd_ex(p)
    else:
        binding.s2attn_fwd(q, k, v, o, lse, G)
    out = {}
    if backward:
        dq = torch.full_like(q, float("nan"))
        dk = torch.full_like(k, float("nan"))
        dv = torch.full_like(v, float("nan"))
        if ex or ws_bytes is not None:
            p = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, **ex)
            nbytes = binding.bwd_workspace_bytes_ex(p)
            if ws_bytes is not None:
                p_min = binding.make_params(q, k, v, o, lse, G, **{**ex, "bwd_algo": binding.BWD_RECOMPUTE})
                nbytes = ws_bytes(binding.bwd_workspace_bytes_ex(p_min), nbytes) if callable(ws_bytes) else ws_bytes
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            p = binding.make_params(q, k, v, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, workspace=ws, **ex)
            binding.s2attn_bwd_ex(p)
        else:
            nbytes = binding.bwd_workspace_bytes(B, N, H, Hkv, D, G, binding.BF16 if bf else binding.F32)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            binding.s2attn_bwd(q, k, v, o, do, lse, dq, dk, dv, ws, G)
        torch.cuda.synchronize()
        out.update(dq=to_np(dq), dk=to_np(dk), dv=to_np(dv))
    torch.cuda.synchronize()
    out.update(o=to_np(o), lse=to_np(lse))
    return out


TOL_BF16 = 2e-2      # stated bound on o, dq, dk, dv in bf16 mode, against the fp32 oracle
TOL_LSE = 2e-3


def half_ulp_bf16(ref):
    """Half the spacing of bf16 numbers at |ref|: what rounding the exact value to the bf16
    output costs at most (2^-9 |ref| .. 2^-8 |ref|)."""
    _, ex = np.frexp(np.abs(np.asarray(ref, dtype=np.float32)))     # |ref| = m * 2^ex, m in [0.5, 1)
    return np.ldexp(np.float32(1.0), ex - 9).astype(np.float64)


def bf16_tol(ref):
    """Per-element bound for a bf16 output tensor: the stated 2e-2 on the value the kernel
    holds in fp32, plus the rounding of that value to the bf16 it has to be stored as.
    No allowance for the number of heads or terms summed."""
    return TOL_BF16 + half_ulp_bf16(ref)


def check_bf16_tensor(name, got, ref):
    """Asserts |got - ref| <= bf16_tol(ref) element-wise; returns (max error, max error beyond
    the output rounding)."""
    assert np.all(np.isfinite(got)), name
    err = np.abs(got.astype(np.float64) - ref)
    tol = bf16_tol(ref)
    if (err > tol).any():
        idx = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{name}: {(err > tol).sum()} elements over tolerance; worst at {idx}: "
                             f"got {got[idx]}, ref {ref[idx]}, err {err[idx]}, tol {tol[idx]}")
    return float(err.max()), float((err - half_ulp_bf16(ref)).max())


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))))


def run_hip_packed(inp: dict, G: int, dtype: str, **ex):
    """Same as run_hip, but q, k, v are non-contiguous views into one packed
    (B, N, H + 2*Hkv, D) tensor and dq, dk, dv views into one packed gradient tensor,
    passed through the stride fields of the parameter block (no split copy)."""
    bf = dtype == "bf16"
    q = to_dev(inp["q"], inp.get("q_bits") if bf else None)
    k = to_dev(inp["k"], inp.get("k_bits") if bf else None)
    v = to_dev(inp["v"], inp.get("v_bits") if bf else None)
    do = to_dev(inp["do"], inp.get("do_bits") if bf else None)
    B, N, H, D = q.shape
    Hkv = k.shape[2]
    packed = torch.cat([q, k, v], dim=2).contiguous()
    qv, kv, vv = packed[:, :, :H], packed[:, :, H:H + Hkv], packed[:, :, H + Hkv:]
    assert not qv.is_contiguous()
    o = torch.full_like(q, float("nan"))
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    p = binding.make_params(qv, kv, vv, o, lse, G, strided=True, **ex)
    binding.s2attn_fwd_ex(p)
    dpacked = torch.full_like(packed, float("nan"))
    dq, dk, dv = dpacked[:, :, :H], dpacked[:, :, H:H + Hkv], dpacked[:, :, H + Hkv:]
    nbytes = binding.bwd_workspace_bytes(B, N, H, Hkv, D, G, binding.BF16 if bf else binding.F32)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    p = binding.make_params(qv, kv, vv, o, lse, G, dout=do, dq=dq, dk=dk, dv=dv, workspace=ws, strided=True, **ex)
    binding.s2attn_bwd_ex(p)
    torch.cuda.synchronize()
    return dict(o=to_np(o), lse=to_np(lse), dq=to_np(dq), dk=to_np(dk), dv=to_np(dv))


def run_hip_head_shard(inp: dict, G: int, dtype: str, h0: int, h1: int, **ex):
    """Runs heads [h0, h1) of the layer in `inp` as one head shard: q, k, v are strided views
    of the layer's tensors (kv heads [h0/r, h1/r)), the shard's position in the layer goes
    through heads_total / head_offset.  Returns the shard's o, lse, dq, dk, dv."""
    bf = dtype == "bf16"
    q = to_dev(inp["q"], inp.get("q_bits") if bf else None)
    k = to_dev(inp["k"], inp.get("k_bits") if bf else None)
    v = to_dev(inp["v"], inp.get("v_bits") if bf else None)
    do = to_dev(inp["do"], inp.get("do_bits") if bf else None)
    B, N, H, D = q.shape
    r = H // k.shape[2]
    assert h0 % r == 0 and h1 % r == 0
    qv, kv, vv = q[:, :, h0:h1], k[:, :, h0 // r:h1 // r], v[:, :, h0 // r:h1 // r]
    dov = do[:, :, h0:h1].contiguous()
    Hs, Hkvs = h1 - h0, (h1 - h0) // r
    o = torch.full((B, N, Hs, D), float("nan"), dtype=q.dtype, device="cuda")
    lse = torch.full((B, Hs, N), float("nan"), dtype=torch.float32, device="cuda")
    dq = torch.full_like(o, float("nan"))
    dk = torch.full((B, N, Hkvs, D), float("nan"), dtype=q.dtype, device="cuda")
    dv = torch.full_like(dk, float("nan"))
    kw = dict(strided=True, heads_total=H, head_offset=h0, dims=(B, N, Hs, Hkvs, D), **ex)
    p = binding.make_params(qv, kv, vv, o, lse, G, **kw)
    binding.s2attn_fwd_ex(p)
    p = binding.make_params(qv, kv, vv, o, lse, G, dout=dov, dq=dq, dk=dk, dv=dv, **kw)
    ws = torch.empty(binding.bwd_workspace_bytes_ex(p), dtype=torch.uint8, device="cuda")
    p = binding.make_params(qv, kv, vv, o, lse, G, dout=dov, dq=dq, dk=dk, dv=dv, workspace=ws, **kw)
    binding.s2attn_bwd_ex(p)
    torch.cuda.synchronize()
    return dict(o=to_np(o), lse=to_np(lse), dq=to_np(dq), dk=to_np(dk), dv=to_np(dv))
