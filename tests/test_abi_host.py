"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and the pure-host argument validator returns the
documented codes."""
import ctypes
import os
import re

import pytest

from paper_2309_12307_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "s2attn.h")).read()
    return sorted(set(re.findall(r"S2ATTN_API\s+[\w\s\*]+?\b(s2attn_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), n


def test_strerror_and_flops():
    assert binding.strerror(0) == "ok"
    for code in range(-13, 0):
        if code != -7:        # -7 is unused
            assert "error code" not in binding.strerror(code)
    assert "error code" in binding.strerror(-99)
    # C3 of the benchmark: 7.698 effective TFLOP forward+backward
    assert abs(binding.effective_flops(1, 32768, 32, 128, 8192, 2) / 1e12 - 7.698) < 1e-3
    assert binding.effective_flops(1, 32768, 32, 128, 8192, 0) * 3.5 == pytest.approx(
        binding.effective_flops(1, 32768, 32, 128, 8192, 2))


def params(**kw):
    d = dict(B=1, N=1024, H=4, Hkv=4, D=128, G=256, dtype=binding.BF16)
    d.update(kw)
    p = binding.S2AttnParams()
    fake = 0x10000
    for f in ("q", "k", "v", "o", "lse", "dout", "dq", "dk", "dv", "workspace"):
        setattr(p, f, kw.get(f, fake))
    p.workspace_bytes = kw.get("workspace_bytes", 1 << 40)
    for f in ("B", "N", "H", "Hkv", "D", "G", "dtype"):
        setattr(p, f, d[f])
    for f in ("q", "k", "v", "dq", "dk", "dv"):
        if f + "_strides" in kw:
            setattr(p, f + "_strides", (ctypes.c_longlong * 3)(*kw[f + "_strides"]))
    p.shift = kw.get("shift", -1)
    p.shift_rule = kw.get("shift_rule", 0)
    p.wrap_variant = kw.get("wrap_variant", 0)
    p.scale = 0.0
    p.heads_total = kw.get("heads_total", 0)
    p.head_offset = kw.get("head_offset", 0)
    p.bwd_algo = kw.get("bwd_algo", 0)
    return p


def ds_bytes(B, N, H, G, heads=None):
    """Bytes of stored dS for `heads` query heads (default all): 16 KB per (64 query x 128 key)
    tile at or below the diagonal, T (T + 1) of them per (head, group) with T = G / 128."""
    T = G // 128
    return B * (H if heads is None else heads) * (N // G) * T * (T + 1) * 16384


def test_validator_accepts_benchmark_shapes():
    from paper_2309_12307_amd.inputs import CONFIGS
    for c in CONFIGS.values():
        p = params(B=c.B, N=c.N, H=c.H, Hkv=c.Hkv, D=c.D, G=c.G,
                   dtype=binding.BF16 if c.dtype == "bf16" else binding.F32)
        assert binding.check_args(p, True) == 0, c.name


@pytest.mark.parametrize("kw,code", [
    (dict(q=0), -1),
    (dict(dv=0), -1),
    (dict(k=0x10008), -2),
    (dict(workspace=0x10010), -2),
    (dict(N=0), -3),
    (dict(N=1000), -4),                       # N % G != 0
    (dict(G=255, N=1020, dtype=1, D=64), -4),  # odd G
    (dict(shift=256), -4),
    (dict(H=3, Hkv=3), -5),
    (dict(H=4, Hkv=3), -5),
    (dict(D=96), -6),
    (dict(D=256), -6),
    (dict(workspace_bytes=16), -8),
    (dict(workspace=0), -8),
    (dict(dtype=5), -9),
    (dict(shift_rule=7), -9),
    (dict(wrap_variant=1), -9),
    (dict(B=40000), -12),
    (dict(q_strides=(1024 * 4 * 128 * 3, 3 * 4 * 128, 100)), -13),    # head stride not a multiple of 8
    (dict(k_strides=(1024 * 4 * 128, -512, 128)), -13),               # negative
    (dict(dv_strides=(1024 * 4 * 128, 512, 64)), -13),                # heads would overlap
    (dict(dq_strides=(1024 * 4 * 128, 256, 128)), -13),               # tokens would overlap the 4 heads of a token
    (dict(dk_strides=(1024 * 128, 128, 1024 * 128), B=2), -13),       # batches would overlap the heads
    (dict(k_strides=((1 << 26) * 1024, 1 << 26, 128)), -13),          # token stride beyond the kernels' 32-bit row offsets
])
def test_validator_codes(kw, code):
    assert binding.check_args(params(**kw), True) == code


@pytest.mark.parametrize("kw", [
    dict(G=64, N=1024),                 # group smaller than a tile
    dict(G=200, N=1000),                # partial last tile, shift 100 inside a tile
    dict(G=25000, N=100000),            # the paper's 100k-token setting (Section 4.2), G = N / 4
    dict(shift=2),
    dict(wrap_variant=2),               # aligned Variant 2
    dict(D=64),                           # head dimension 64 in bf16
    dict(G=200, N=1000, wrap_variant=2),  # Variant 2 with a partial last tile
    dict(shift=100, wrap_variant=2),      # Variant 2 split inside a tile
    dict(G=384, N=1536, wrap_variant=2),  # split at 192: a multiple of 64 but not of the 128-key tile
    dict(dq_strides=(4 * 1024 * 128, 128, 1024 * 128), dk_strides=(4 * 1024 * 128, 128, 1024 * 128),
         dv_strides=(4 * 1024 * 128, 128, 1024 * 128)),   # head-major (B, H, N, D) gradients: rows stay disjoint
])
def test_validator_accepts_unaligned_groups_in_bf16(kw):
    assert binding.check_args(params(**kw), True) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(H=3, Hkv=3, heads_total=12, head_offset=3), 0),     # an odd shard of a 12-head layer
    (dict(H=4, Hkv=2, heads_total=16, head_offset=6), 0),     # shard straddles the layer's middle
    (dict(H=4, Hkv=2, heads_total=16, head_offset=5), -5),    # offset splits a kv head's query heads
    (dict(H=4, Hkv=4, heads_total=15, head_offset=0), -5),    # the layer's head count must be even
    (dict(H=4, Hkv=4, heads_total=6, head_offset=4), -5),     # shard runs past the layer
    (dict(H=4, Hkv=4, heads_total=8, head_offset=-4), -5),
    (dict(H=4, Hkv=4, head_offset=4), -5),                    # offset without a layer size
])
def test_head_sharding_fields(kw, code):
    assert binding.check_args(params(**kw), True) == code


def test_workspace_size_follows_the_shard():
    # heads 6..9 of a 16-head layer with 2 query heads per kv head: local heads 2, 3 shift,
    # every kv head is wholly on one side -> no partial sums
    p = params(H=4, Hkv=2, heads_total=16, head_offset=6)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * 4 * 1024 * 4
    # heads 4..11 with 4 query heads per kv head: the layer's middle (head 8) is local head 4,
    # a kv-head boundary -> still none; with heads_total = 20 the middle is local head 6 -> mixed
    p = params(H=8, Hkv=2, heads_total=16, head_offset=4)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * 8 * 1024 * 4
    p = params(H=8, Hkv=2, heads_total=20, head_offset=4)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * 8 * 1024 * 4 + 4 * 1024 * 2 * 128 * 4
    # the stored-dS backward adds room for dS
    p = params(H=8, Hkv=2, heads_total=16, head_offset=4, bwd_algo=binding.BWD_STORED_DS)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * 8 * 1024 * 4 + ds_bytes(1, 1024, 8, 256)
    # whole layer: same as the plain query
    p = params()
    assert binding.bwd_workspace_bytes_ex(p) == binding.bwd_workspace_bytes(1, 1024, 4, 4, 128, 256)


def test_packed_qkv_strides_are_accepted():
    # the three slices of a packed (B, N, 3, H, D) tensor
    B, N, H, D = 1, 1024, 4, 128
    st = (N * 3 * H * D, 3 * H * D, D)
    p = params(q_strides=st, k_strides=st, v_strides=st, dq_strides=st, dk_strides=st, dv_strides=st)
    assert binding.check_args(p, True) == 0


def test_forward_check_ignores_backward_fields():
    p = params(dout=0, dq=0, dk=0, dv=0, workspace=0, workspace_bytes=0)
    assert binding.check_args(p, False) == 0
    assert binding.check_args(p, True) == -1


def test_workspace_size():
    rows = 2 * 32 * 32768 * 4      # delta and base-2 lse: 2 * B*H*N floats (each rounded to 256 bytes)
    assert binding.bwd_workspace_bytes(1, 32768, 32, 32, 128, 8192) == rows
    # MQA: one kv head serves shifted and unshifted heads -> fp32 partials too
    w = binding.bwd_workspace_bytes(1, 256, 4, 1, 64, 64, binding.F32)
    assert w == 2 * 4 * 256 * 4 + 4 * 256 * 64 * 4
    # stored-dS backward.  The 7B-shaped layer at N = 32768: dS of all 32 heads (8.7 GB, under the
    # 16 GiB the query asks for at most)
    st = binding.BWD_STORED_DS
    p = params(B=1, N=32768, H=32, Hkv=32, D=128, G=8192, bwd_algo=st)
    assert binding.bwd_workspace_bytes_ex(p) == rows + ds_bytes(1, 32768, 32, 8192)
    # GQA layer (17.4 GB of dS in all): 7 of the 8 kv heads at a time
    per_kv_head = ds_bytes(1, 32768, 64, 8192, heads=8)
    p = params(B=1, N=32768, H=64, Hkv=8, D=128, G=8192, bwd_algo=st)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * rows + 7 * per_kv_head and 2 ** 34 // per_kv_head == 7
    # 100k-token layer: 6 heads at a time
    p = params(B=1, N=102400, H=32, Hkv=32, D=128, G=25600, bwd_algo=st)
    assert binding.bwd_workspace_bytes_ex(p) == 2 * 32 * 102400 * 4 + 6 * ds_bytes(1, 102400, 32, 25600, heads=1)


@pytest.mark.parametrize("kw,code", [
    (dict(bwd_algo=2), 0),
    (dict(bwd_algo=3), -9),
    (dict(bwd_algo=2, G=200, N=1000), -15),                    # unaligned group
    (dict(bwd_algo=2, shift=32), -15),
    (dict(bwd_algo=2, H=2, Hkv=1), -15),                       # the kv head serves both head classes
    (dict(bwd_algo=2, dtype=1, D=64), -15),
    (dict(bwd_algo=2, D=64), -15),                             # bf16 with head dimension 64
    (dict(bwd_algo=2, G=384, N=1536, wrap_variant=2), -15),    # Variant 2 split at 192
    (dict(bwd_algo=2, wrap_variant=2), 0),
    (dict(bwd_algo=2, workspace_bytes=2 * 4 * 1024 * 4), -8),  # row terms only: no room for one kv head's dS
    (dict(bwd_algo=0, workspace_bytes=2 * 4 * 1024 * 4), 0),   # the default needs the row terms only
])
def test_backward_algorithm_field(kw, code):
    assert binding.check_args(params(**kw), True) == code


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()


def test_static_scratch_backward_refuses_large_problems_on_the_host():
    """s2attn_bwd_ex_static checks the size before it looks at any pointer or at the GPU."""
    p = params(B=1, N=131072, H=32, Hkv=32, D=128, G=8192)     # 4 Mi rows: 32 MiB of row terms
    assert binding.lib().s2attn_bwd_ex_static(ctypes.byref(p), None) == -14
    assert "static" in binding.strerror(-14)
    p = params(B=1, N=16384, H=4, Hkv=1, D=128, G=1024)        # MQA: 32 MiB of partial sums
    assert binding.lib().s2attn_bwd_ex_static(ctypes.byref(p), None) == -14
