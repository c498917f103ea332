"""bf16 mode: HIP path vs the CPU oracle (which reads the same bf16-rounded inputs
up-cast to fp32 and is not rounded at the end).

Tolerance on o, dq, dk, dv, per element: |err| <= 2e-2 + half-ulp_bf16(ref).  The stated
bound is max-abs 2e-2; the second term is what storing the exact result as bf16 costs by
itself (0.0078 for 2 <= |ref| < 4, 0.031 for 8 <= |ref| < 16; such values occur in dk, dv at
the first keys of a group, where P is close to 1 for many queries, and under GQA where
several heads' gradients are summed).  The bound carries no allowance for the number of
heads or terms summed.  o and dq never leave the binades where the plain 2e-2 holds and
are also held to it.  lse is an fp32 output: <= 2e-3."""
import numpy as np
import pytest

from oracle import s2attn_oracle as orc
from paper_2309_12307_amd import inputs

pytestmark = pytest.mark.gpu


def compare(out, ref):
    from gpu_util import TOL_BF16, TOL_LSE, check_bf16_tensor
    o, lse, dq, dk, dv = ref
    e_lse = np.abs(out["lse"] - lse).max()
    assert np.isfinite(e_lse) and e_lse <= TOL_LSE, ("lse", e_lse)
    errs = {name: check_bf16_tensor(name, out[name], r)[0]
            for name, r in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv))}
    assert errs["o"] <= TOL_BF16 and errs["dq"] <= TOL_BF16, errs
    return errs


# (B, N, H, Hkv, D, G)
SHAPES = [
    (1, 512, 2, 2, 128, 128),      # one query tile per group
    (2, 1024, 4, 4, 128, 256),     # two tiles per group, batch 2
    (1, 1536, 4, 2, 128, 384),     # three 128-row tiles, GQA
    (1, 2048, 8, 2, 128, 1024),    # 4 query heads per kv head
    (1, 768, 2, 1, 128, 256),      # MQA: the kv head serves both classes
    (1, 1536, 6, 3, 128, 512),     # odd Hkv: middle kv head is mixed
    (1, 640, 2, 2, 128, 640),      # one group, 5 tiles
    (1, 1024, 8, 1, 128, 512),     # MQA, four query heads per class walked tile by tile
]


@pytest.mark.parametrize("shape", SHAPES)
def test_shapes(shape):
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=sum(shape), dtype="bf16")
    out = run_hip(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


# The two ways the backward gets dS into its dQ kernel (stored by the dK/dV kernel, or
# recomputed) on tile-aligned shapes; everything else in this file runs the default, which
# recomputes.
ALIGNED_SHAPES = [
    (1, 512, 2, 2, 128, 128),      # one key tile per group: only diagonal tiles
    (2, 1024, 4, 4, 128, 256),     # batch 2
    (1, 2048, 8, 2, 128, 1024),    # 4 query heads per kv head
    (1, 1536, 4, 2, 128, 384),     # three key tiles
    (1, 640, 2, 2, 128, 640),      # one group, five key tiles
]


@pytest.mark.parametrize("shape", ALIGNED_SHAPES)
@pytest.mark.parametrize("algo", ["recompute", "stored"])
def test_backward_algorithms(shape, algo):
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=sum(shape), dtype="bf16")
    out = run_hip(inp, G, "bf16", bwd_algo=binding.BWD_RECOMPUTE if algo == "recompute" else binding.BWD_STORED_DS)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


@pytest.mark.parametrize("heads_at_a_time", [1, 3])
def test_stored_ds_backward_in_several_passes(heads_at_a_time):
    """A workspace with room for the dS of only some kv heads: the backward runs the kv heads
    in passes over the same dS area."""
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 1024, 8, 4, 128, 256
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=77, dtype="bf16")
    size = lambda rows, wanted: rows + (wanted - rows) // Hkv * heads_at_a_time + 100
    out = run_hip(inp, G, "bf16", ws_bytes=size, bwd_algo=binding.BWD_STORED_DS)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


def test_stored_ds_backward_with_variant2_and_custom_shift():
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 1536, 4, 2, 128, 512
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=78, dtype="bf16")
    for kw, okw in ((dict(wrap_variant=binding.WRAP_SPLIT), dict(variant2=True)),
                    (dict(wrap_variant=binding.WRAP_SPLIT, shift=128), dict(variant2=True, shift=128)),
                    (dict(shift=192, shift_rule=binding.SHIFT_ALL), dict(shift=192, shift_heads="all"))):
        out = run_hip(inp, G, "bf16", bwd_algo=binding.BWD_STORED_DS, **kw)
        ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, **okw)
        compare(out, ref)


# Head dimension 64 (runs on the kernels built for partial tiles, with the upper half of the
# 128-element tile rows read as zeros).
D64_SHAPES = [
    (1, 512, 2, 2, 64, 128),       # aligned group
    (2, 1024, 4, 4, 64, 256),      # batch 2
    (1, 2048, 8, 2, 64, 1024),     # GQA, 4 query heads per kv head
    (1, 768, 2, 1, 64, 256),       # MQA: the kv head serves both classes (fp32 partial sums)
    (1, 1536, 6, 3, 64, 512),      # odd Hkv
    (1, 1000, 4, 2, 64, 500),      # partial tiles
    (1, 390, 2, 2, 64, 130),
    (1, 24, 2, 1, 64, 6),
]


@pytest.mark.parametrize("shape", D64_SHAPES)
def test_head_dimension_64(shape):
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=64 + sum(shape), dtype="bf16")
    out = run_hip(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


def test_head_dimension_64_options():
    """Variant 2, a custom shift with the all-heads rule, packed views and the static-scratch
    backward at D = 64."""
    from gpu_util import run_hip, run_hip_packed
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 1536, 4, 2, 64, 384
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=640, dtype="bf16")
    out = run_hip(inp, G, "bf16", wrap_variant=binding.WRAP_SPLIT)
    compare(out, orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, variant2=True))
    out = run_hip(inp, G, "bf16", shift=100, shift_rule=binding.SHIFT_ALL)
    compare(out, orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, shift=100, shift_heads="all"))
    out = run_hip_packed(inp, G, "bf16")
    compare(out, orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G))


def test_full_causal_attention_mode():
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D = 1, 1024, 2, 2, 128
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=177, dtype="bf16")
    out = run_hip(inp, N, "bf16", shift_rule=binding.SHIFT_NONE)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], N, shift_heads="none")
    compare(out, ref)


@pytest.mark.parametrize("rule,name", [(1, "none"), (2, "all")])
def test_shift_rules(rule, name):
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = 1, 1024, 4, 2, 128, 256
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=178 + rule, dtype="bf16")
    out = run_hip(inp, G, "bf16", shift_rule=rule)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, shift_heads=name)
    compare(out, ref)


def test_custom_shift_and_scale():
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = 1, 1536, 4, 4, 128, 512
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=180, dtype="bf16")
    out = run_hip(inp, G, "bf16", shift=128, scale=0.05)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, shift=128, scale=0.05)
    compare(out, ref)


@pytest.mark.parametrize("shape", [(1, 1024, 4, 4, 128, 256), (1, 1536, 4, 2, 128, 512), (1, 768, 2, 1, 128, 256)])
def test_variant2_split_wrap_group(shape):
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=181, dtype="bf16")
    out = run_hip(inp, G, "bf16", wrap_variant=binding.WRAP_SPLIT)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, variant2=True)
    compare(out, ref)


# Variant 2 where the split G - shift is not a multiple of the 128-key tile of the dK/dV
# kernels (64 mod 128, or inside a 64-row run), with partial last tiles, GQA and MQA.
@pytest.mark.parametrize("shape,shift", [
    ((1, 1536, 4, 4, 128, 384), None),     # split at 192
    ((1, 1024, 4, 2, 128, 256), 64),       # split at 192
    ((1, 1024, 4, 2, 128, 256), 192),      # split at 64
    ((1, 2048, 4, 4, 128, 512), 64),       # split at 448: the first block spans 3.5 key tiles
    ((1, 1000, 4, 2, 128, 500), None),     # partial tiles, split at 250
    ((1, 1024, 2, 2, 128, 256), 100),      # split at 156, wrap point inside a tile
    ((1, 400, 2, 1, 128, 200), 3),         # MQA; second block of 3 rows
    ((1, 390, 2, 2, 128, 130), 129),       # first block of one row
    ((2, 1280, 4, 4, 128, 640), None),     # five tiles, split at 320; batch 2
])
def test_variant2_split_not_on_a_tile_boundary(shape, shift):
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=182 + sum(shape), dtype="bf16")
    kw = {} if shift is None else dict(shift=shift)
    out = run_hip(inp, G, "bf16", wrap_variant=binding.WRAP_SPLIT, **kw)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, variant2=True, shift=shift)
    compare(out, ref)


def test_variant2_split_inside_a_workgroup_of_the_eight_wave_forward():
    """G = 2304 = 9 x 256 runs the eight-wave forward kernel (256 query rows per workgroup);
    the default shift 1152 puts the Variant 2 split in the middle of a workgroup's rows."""
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 4608, 4, 2, 128, 2304
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=184, dtype="bf16")
    out = run_hip(inp, G, "bf16", wrap_variant=binding.WRAP_SPLIT)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, variant2=True, dtype=np.float32)
    compare(out, ref)
    out = run_hip(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, dtype=np.float32)
    compare(out, ref)


def test_variant2_with_all_heads_shifted_and_head_shards():
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    B, N, H, Hkv, D, G = 1, 1152, 4, 2, 128, 384
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=183, dtype="bf16")
    out = run_hip(inp, G, "bf16", wrap_variant=binding.WRAP_SPLIT, shift_rule=binding.SHIFT_ALL)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, variant2=True, shift_heads="all")
    compare(out, ref)


@pytest.mark.parametrize("shape", [(2, 1024, 4, 4, 128, 256), (1, 1536, 8, 2, 128, 512), (1, 768, 2, 1, 128, 256),
                                   (1, 640, 2, 2, 128, 640)])
def test_packed_qkv_views(shape):
    """q, k, v (and dq, dk, dv) as strided views of one packed projection tensor."""
    from gpu_util import run_hip_packed
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=190 + sum(shape), dtype="bf16")
    out = run_hip_packed(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


# Group sizes and shifts that are not multiples of the kernels' tile sizes (128 rows,
# 64-token runs): partial last tiles and a wrap point inside a tile.
RAGGED_SHAPES = [
    (1, 400, 2, 2, 128, 200),      # two tiles per group, the second partial; shift 100
    (1, 192, 2, 1, 128, 64),       # group smaller than a tile, MQA (both classes share the kv head)
    (2, 780, 4, 4, 128, 390),      # batch 2, four tiles with a 6-row tail
    (1, 1000, 4, 2, 128, 500),     # GQA
    (1, 1000, 2, 2, 128, 1000),    # one group; last wave of the last tile is all padding
    (1, 1290, 6, 3, 128, 258),     # two-row tail; odd Hkv: middle kv head is mixed
    (1, 10000, 2, 2, 128, 2500),   # N = 100000, G = 25000 (Section 4.2) scaled down by 10
    (1, 4, 2, 2, 128, 2),          # smallest group: two tokens, shift 1
    (1, 24, 2, 1, 128, 6),
    (1, 130, 2, 2, 128, 130),      # one group whose second tile holds two rows
    (1, 600, 8, 2, 128, 300),      # four query heads per kv head, three tiles, the last partial
]


@pytest.mark.parametrize("shape", RAGGED_SHAPES)
def test_unaligned_group_sizes(shape):
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = shape
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=300 + sum(shape), dtype="bf16")
    out = run_hip(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, dtype=np.float32)
    compare(out, ref)


@pytest.mark.parametrize("G,shift", [(256, 2), (256, 100), (512, 447), (200, 1), (200, 199)])
def test_unaligned_shift(G, shift):
    from gpu_util import run_hip
    B, N, H, Hkv, D = 1, 4 * G, 4, 2, 128
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=320 + G + shift, dtype="bf16")
    out = run_hip(inp, G, "bf16", shift=shift)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, shift=shift)
    compare(out, ref)


@pytest.mark.parametrize("rule,name", [(1, "none"), (2, "all")])
def test_unaligned_group_shift_rules(rule, name):
    from gpu_util import run_hip
    B, N, H, Hkv, D, G = 1, 900, 4, 2, 128, 300
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=330 + rule, dtype="bf16")
    out = run_hip(inp, G, "bf16", shift_rule=rule)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G, shift_heads=name)
    compare(out, ref)


def test_unaligned_group_packed_qkv_views():
    from gpu_util import run_hip_packed
    B, N, H, Hkv, D, G = 1, 1000, 4, 2, 128, 500
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=340, dtype="bf16")
    out = run_hip_packed(inp, G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    compare(out, ref)


@pytest.mark.parametrize("layer,shards", [
    ((1, 1024, 8, 4, 128, 256), [(0, 4), (4, 8), (2, 6)]),
    ((1, 768, 12, 3, 128, 256), [(4, 8)]),          # the layer's middle splits the shard's kv head
    ((1, 1000, 8, 8, 128, 500), [(3, 8)]),          # unaligned group, odd shard
])
def test_head_shards_reproduce_the_layer(layer, shards):
    from gpu_util import run_hip_head_shard
    B, N, H, Hkv, D, G = layer
    r = H // Hkv
    inp = inputs.make_inputs(B, N, H, Hkv, D, seed=500 + sum(layer), dtype="bf16")
    o, lse, dq, dk, dv = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], G)
    for h0, h1 in shards:
        out = run_hip_head_shard(inp, G, "bf16", h0, h1)
        compare(out, (o[:, :, h0:h1], lse[:, h0:h1], dq[:, :, h0:h1], dk[:, :, h0 // r:h1 // r],
                      dv[:, :, h0 // r:h1 // r]))


def test_outputs_are_deterministic():
    from gpu_util import run_hip
    inp = inputs.make_inputs(1, 1024, 4, 2, 128, seed=5, dtype="bf16")
    a = run_hip(inp, 256, "bf16")
    b = run_hip(inp, 256, "bf16")
    for name in a:
        assert np.array_equal(a[name], b[name]), name


def test_config_c2_full_tensors():
    """Llama2-7B-shaped layer, N = 8192, G = 2048: every element against the oracle."""
    from gpu_util import run_hip
    cfg = inputs.CONFIGS["C2"]
    inp = inputs.make_config_inputs(cfg)
    out = run_hip(inp, cfg.G, "bf16")
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], cfg.G, dtype=np.float32)
    errs = compare(out, ref)
    print("C2 max-abs errors", errs)


def test_config_c2_full_tensors_stored_ds_backward():
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    cfg = inputs.CONFIGS["C2"]
    inp = inputs.make_config_inputs(cfg)
    out = run_hip(inp, cfg.G, "bf16", bwd_algo=binding.BWD_STORED_DS)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], cfg.G, dtype=np.float32)
    errs = compare(out, ref)
    print("C2 (stored-dS backward) max-abs errors", errs)


def test_config_c2_variant2_full_tensors():
    """Same layer with the wrap-around group split (Appendix B.3 Variant 2), on the aligned
    kernels (split at 1024)."""
    from gpu_util import run_hip
    from paper_2309_12307_amd import binding
    cfg = inputs.CONFIGS["C2"]
    inp = inputs.make_config_inputs(cfg)
    out = run_hip(inp, cfg.G, "bf16", wrap_variant=binding.WRAP_SPLIT)
    ref = orc.s2attn_fwd_bwd(inp["q"], inp["k"], inp["v"], inp["do"], cfg.G, variant2=True, dtype=np.float32)
    compare(out, ref)
