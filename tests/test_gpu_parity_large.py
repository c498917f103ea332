"""bf16 benchmark configurations at full size, in the launch configuration bench.py
times.  The oracle cannot do the whole tensors in reasonable time, so parity is checked
on whole (kv head, group) slices that the oracle computes one by one -- an unshifted
group, a shifted group, the wrap-around group of a shifted head and, under GQA, all
query heads of the sampled kv heads -- plus properties that hold at any size."""
import numpy as np
import pytest

from oracle import s2attn_oracle as orc
from paper_2309_12307_amd import inputs

pytestmark = pytest.mark.gpu
TOL, RTOL, TOL_LSE = 2e-2, 5e-3, 2e-3


def check(name, got, ref, heads_summed=1):
    """|err| <= max(2e-2 * sqrt(r), 5e-3 * |ref|): dk and dv add the gradients of the r
    query heads of a kv head, each carrying the bf16 rounding of its own P / dS operands,
    so their absolute error budget grows like sqrt(r); r = 1 for o, dq and plain MHA."""
    err = np.abs(got.astype(np.float64) - ref)
    tol = np.maximum(TOL * np.sqrt(heads_summed), RTOL * np.abs(ref))
    assert np.all(np.isfinite(got)), name
    if (err > tol).any():
        idx = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{name}: worst at {idx}: got {got[idx]}, ref {ref[idx]}, err {err[idx]}")
    return float(err.max())


def run_and_check(cfg_name, slices, cfg=None):
    from gpu_util import run_hip
    cfg = cfg or inputs.CONFIGS[cfg_name]
    inp = inputs.make_config_inputs(cfg)
    out = run_hip(inp, cfg.G, "bf16")
    N, G, H, Hkv = cfg.N, cfg.G, cfg.H, cfg.Hkv
    r = H // Hkv
    # properties at full size: everything finite; the first row of every group sees only
    # itself, so O equals V there exactly (bf16 values pass through unrounded)
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.isfinite(out[name]).all(), name
    for h in (0, H // 2 - 1, H // 2, H - 1):
        s = G // 2 if h >= H // 2 else 0
        first = (np.arange(N // G) * G + s) % N
        assert np.array_equal(out["o"][0, first, h], inp["v"][0, first, h // r]), h
    worst = {}
    for (c, g) in slices:
        ref = orc.s2attn_group_slice(inp["q"], inp["k"], inp["v"], inp["do"], G, 0, c, g, dtype=np.float32)
        tok, heads = ref["tokens"], ref["heads"]
        e = {
            "o": check("o", out["o"][0][np.ix_(tok, heads)], ref["o"]),
            "dq": check("dq", out["dq"][0][np.ix_(tok, heads)], ref["dq"]),
            "dk": check("dk", out["dk"][0, tok, c], ref["dk"], r),
            "dv": check("dv", out["dv"][0, tok, c], ref["dv"], r),
        }
        e_lse = float(np.abs(out["lse"][0][np.ix_(heads, tok)] - ref["lse"]).max())
        assert e_lse <= TOL_LSE, e_lse
        assert e["o"] <= TOL and e["dq"] <= TOL, e
        for k_, v_ in e.items():
            worst[k_] = max(worst.get(k_, 0.0), v_)
        print(f"{cfg_name} kv head {c} group {g}: max-abs {e} lse {e_lse:.2e}", flush=True)
    print(f"{cfg_name} worst max-abs over sampled slices: {worst}", flush=True)


def test_config_c3_sampled_slices():
    # Llama2-7B-shaped, N = 32768, G = 8192: first/last group of an unshifted head, first
    # group and wrap-around group of a shifted head
    run_and_check("C3", [(0, 0), (15, 3), (16, 0), (31, 3)])


def test_config_c4_gqa_sampled_slices():
    # Llama2-70B-shaped GQA, 8 query heads per kv head: an unshifted and a shifted kv head
    run_and_check("C4", [(0, 1), (7, 3)])


def test_config_c5_100k_sampled_slices():
    # N = 102400, G = 25600: one unshifted group and the wrap-around group
    run_and_check("C5", [(3, 1), (31, 3)])


def test_100k_tokens_unaligned_group():
    # the paper's longest 7B context (Section 4.2) at its exact length: N = 100000 with
    # G = N / 4 = 25000 and shift 12500, neither a multiple of the kernels' tile sizes;
    # 4 heads keep the run short.  A first group, and the wrap-around group of a shifted head.
    cfg = inputs.S2Config("N100000", 6, "bf16", 1, 100000, 4, 4, 128, 25000)
    run_and_check("N100000", [(1, 0), (3, 3)], cfg)
