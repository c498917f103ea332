"""Pins of the CPU oracle against facts fixed by the paper and by mathematics,
none of which come from the oracle itself or from the HIP path."""
import os

import numpy as np
import pytest
import torch

from oracle import s2attn_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


def rand_problem(B, N, H, Hkv, D, seed=0):
    r = np.random.default_rng(seed)
    return (r.standard_normal((B, N, H, D)), r.standard_normal((B, N, Hkv, D)),
            r.standard_normal((B, N, Hkv, D)), r.standard_normal((B, N, H, D)))


def textbook_causal(q, k, v, scale):
    """Full causal attention for one head through a library routine (torch SDPA, fp64)."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x))[None, None] for x in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0, 0].numpy()


# ---------------------------------------------------------------- index map
def read_kv(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [int(x) for x in vals]
    return out


def test_index_map_matches_paper_worked_example():
    g = read_kv(os.path.join(GOLD, "index_example.txt"))
    N, G = g["N"][0], g["G"][0]
    s = orc.head_shift(1, 2, G)                     # a head of the second half
    assert s == g["shift"][0]
    assert orc.head_shift(0, 2, G) == 0
    # pattern 1 (unshifted head), first group, 1-based
    t = orc.group_tokens(0, 0, N, G) + 1
    assert [t[0], t[-1]] == g["pattern1_group1"] and np.all(np.diff(t) == 1)
    # pattern 2 (shifted head), first group
    t = orc.group_tokens(0, s, N, G) + 1
    assert [t[0], t[-1]] == g["pattern2_group1"] and np.all(np.diff(t) == 1)
    # wrap group: last 1024 tokens followed by the first 1024
    t = orc.group_tokens(N // G - 1, s, N, G) + 1
    a, b, c, d = g["pattern2_wrap_group"]
    assert t[0] == a and t[G // 2 - 1] == b and t[G // 2] == c and t[-1] == d
    assert np.all(np.diff(t[:G // 2]) == 1) and np.all(np.diff(t[G // 2:]) == 1)


def test_second_half_of_heads_shifts():
    H, G = 8, 64
    assert [orc.head_shift(h, H, G) for h in range(H)] == [0, 0, 0, 0, 32, 32, 32, 32]


def test_roll_round_trip_and_index_inverse():
    N, s = 96, 16
    x = rng.standard_normal((N, 3))
    assert np.array_equal(np.roll(np.roll(x, -s, 0), s, 0), x)
    p = np.arange(N)
    assert np.array_equal(orc.token_to_rolled(orc.rolled_to_token(p, s, N), s, N), p)
    assert np.array_equal(np.roll(x, -s, 0), x[orc.rolled_to_token(p, s, N)])


# ---------------------------------------------------------------- FLOP table
def test_flop_counter_reproduces_paper_table():
    for line in open(os.path.join(GOLD, "flops_table.txt")):
        if line.startswith("#"):
            continue
        n, full, s2 = line.split()
        n = int(n)
        assert round(orc.attn_flops_paper(n, n, 4096, 32) / 1e12, 1) == float(full)
        assert round(orc.attn_flops_paper(n, n // 4, 4096, 32) / 1e12, 1) == float(s2)


def test_causal_flop_counter_counts_pairs():
    B, N, H, D, G = 2, 24, 4, 8, 6
    pairs = sum(1 for b in range(B) for h in range(H) for g in range(N // G)
                for i in range(G) for j in range(i + 1))
    assert orc.attn_flops_causal(B, N, H, D, G, backward=False) == 4 * D * pairs
    assert orc.attn_flops_causal(B, N, H, D, G) == 14 * D * pairs
    c3 = orc.attn_flops_causal(1, 32768, 32, 128, 8192)
    assert abs(c3 / 1e12 - 7.698) < 1e-3


# ---------------------------------------------------------------- forward pins
def test_full_group_no_shift_is_textbook_causal_attention():
    B, N, H, Hkv, D = 1, 40, 2, 2, 8
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 1)
    o, lse = orc.s2attn_fwd(q, k, v, G=N, shift=0)
    for h in range(H):
        ref = textbook_causal(q[0, :, h], k[0, :, h], v[0, :, h], 1 / np.sqrt(D))
        assert np.abs(o[0, :, h] - ref).max() < 1e-12
    # lse against a direct logsumexp of the masked scores
    S = (q[0, :, 0] @ k[0, :, 0].T) / np.sqrt(D)
    S[np.triu_indices(N, 1)] = -np.inf
    ref = torch.logsumexp(torch.from_numpy(S), dim=1).numpy()
    assert np.abs(lse[0, 0] - ref).max() < 1e-12


def test_unshifted_heads_are_block_diagonal_causal_attention():
    B, N, H, Hkv, D, G = 2, 48, 4, 4, 8, 12
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 2)
    o, _ = orc.s2attn_fwd(q, k, v, G)
    for b in range(B):
        for h in range(H // 2):
            for g in range(N // G):
                sl = slice(g * G, (g + 1) * G)
                ref = textbook_causal(q[b, sl, h], k[b, sl, h], v[b, sl, h], 1 / np.sqrt(D))
                assert np.abs(o[b, sl, h] - ref).max() < 1e-12


def test_shifted_heads_are_textbook_attention_on_paper_token_ranges():
    """Shifted head: group g is tokens [g*G+G/2, (g+1)*G+G/2) and the last group is
    the last G/2 tokens followed by the first G/2 (Section 3.2 example)."""
    B, N, H, Hkv, D, G = 1, 48, 2, 2, 8, 12
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 3)
    o, _ = orc.s2attn_fwd(q, k, v, G)
    h = 1
    for g in range(N // G):
        tok = (np.arange(G) + g * G + G // 2) % N     # typed from the paper's example, not from the oracle
        ref = textbook_causal(q[0, tok, h], k[0, tok, h], v[0, tok, h], 1 / np.sqrt(D))
        assert np.abs(o[0, tok, h] - ref).max() < 1e-12


def test_roll_free_mask_formulation_agrees():
    for (B, N, H, Hkv, D, G) in [(2, 32, 4, 4, 4, 8), (1, 24, 4, 2, 6, 12), (1, 16, 2, 1, 4, 4)]:
        q, k, v, _ = rand_problem(B, N, H, Hkv, D, 4)
        o1, l1 = orc.s2attn_fwd(q, k, v, G)
        o2, l2 = orc.s2attn_fwd_masked(q, k, v, G)
        assert np.abs(o1 - o2).max() < 1e-12 and np.abs(l1 - l2).max() < 1e-12


@pytest.mark.parametrize("shift", [3, 1, 7])
def test_roll_free_mask_formulation_agrees_at_a_custom_shift(shift):
    B, N, H, Hkv, D, G = 1, 32, 4, 2, 4, 8
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 41)
    for heads in ("second_half", "all"):
        o1, l1 = orc.s2attn_fwd(q, k, v, G, shift=shift, shift_heads=heads)
        o2, l2 = orc.s2attn_fwd_masked(q, k, v, G, shift=shift, shift_heads=heads)
        assert np.abs(o1 - o2).max() < 1e-12 and np.abs(l1 - l2).max() < 1e-12


def test_custom_shift_and_all_heads_rule_are_textbook_attention_on_their_token_ranges():
    """Shift s on every head: group g is tokens [g*G + s, (g+1)*G + s) mod N, each a plain
    causal attention (token ranges written out here, not taken from the oracle)."""
    B, N, H, Hkv, D, G, s = 1, 40, 2, 2, 8, 10, 3
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 42)
    o, _ = orc.s2attn_fwd(q, k, v, G, shift=s, shift_heads="all")
    for h in range(H):
        for g in range(N // G):
            tok = (np.arange(G) + g * G + s) % N
            ref = textbook_causal(q[0, tok, h], k[0, tok, h], v[0, tok, h], 1 / np.sqrt(D))
            assert np.abs(o[0, tok, h] - ref).max() < 1e-12


def test_shift_direction_variant1_gives_the_same_result():
    """Appendix B.3 Variant 1 rolls the shifted heads by +G/2 going in and -G/2 coming out
    (the opposite direction).  The groups are the same token sets in the same order, only
    numbered differently, so outputs and gradients equal the default method's."""
    B, N, H, Hkv, D, G = 2, 32, 4, 2, 4, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 43)
    ref = orc.s2attn_fwd_bwd(q, k, v, do, G)
    # the oracle rolls by -shift in and +shift out: shift = -G/2 is Variant 1
    var1 = orc.s2attn_fwd_bwd(q, k, v, do, G, shift=-(G // 2))
    for a, b in zip(ref, var1):
        assert np.abs(a - b).max() < 1e-13
    # written out with numpy alone for one shifted head: roll by +G/2, plain block-diagonal
    # causal attention, roll back by -G/2
    h = H - 1
    qr, kr, vr = (np.roll(x[0, :, hh], G // 2, axis=0) for x, hh in ((q, h), (k, h // 2), (v, h // 2)))
    out = np.empty_like(qr)
    for g in range(N // G):
        sl = slice(g * G, (g + 1) * G)
        out[sl] = textbook_causal(qr[sl], kr[sl], vr[sl], 1 / np.sqrt(D))
    assert np.abs(np.roll(out, -(G // 2), axis=0) - ref[0][0, :, h]).max() < 1e-12


def test_closed_forms():
    B, N, H, Hkv, D, G = 1, 32, 4, 4, 4, 8
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 5)
    # Q = 0: uniform attention over the visible prefix -> running mean of V, lse = ln(i+1)
    o, lse = orc.s2attn_fwd(np.zeros_like(q), k, v, G)
    for h in range(H):
        s = G // 2 if h >= H // 2 else 0
        for g in range(N // G):
            tok = (np.arange(G) + g * G + s) % N
            ref = np.cumsum(v[0, tok, h], axis=0) / np.arange(1, G + 1)[:, None]
            assert np.abs(o[0, tok, h] - ref).max() < 1e-12
            assert np.abs(lse[0, h, tok] - np.log(np.arange(1, G + 1))).max() < 1e-12
    # constant V rows -> O equals that row everywhere
    vc = np.broadcast_to(np.array([1.0, -2.0, 3.0, 0.5]), v.shape)
    o, _ = orc.s2attn_fwd(q, k, vc, G)
    assert np.abs(o - vc).max() < 1e-12
    # first row of each group sees only itself: O = V there, lse = its own score
    o, lse = orc.s2attn_fwd(q, k, v, G)
    for h in range(H):
        s = G // 2 if h >= H // 2 else 0
        first = (np.arange(N // G) * G + s) % N
        assert np.abs(o[0, first, h] - v[0, first, h]).max() < 1e-12
        own = (q[0, first, h] * k[0, first, h]).sum(-1) / np.sqrt(D)
        assert np.abs(lse[0, h, first] - own).max() < 1e-12
    # softmax shift invariance: adding one vector to every K row changes nothing in O
    o2, _ = orc.s2attn_fwd(q, k + rng.standard_normal(D), v, G)
    # (each query's scores all move by q.c, a per-row constant)
    assert np.abs(o - o2).max() < 1e-10


def test_rows_of_P_sum_to_one_and_are_causal():
    G, D = 10, 4
    q, k, v = (rng.standard_normal((G, D)) for _ in range(3))
    P, o, lse = orc.dense_group_attention(q, k, v, 0.5)
    assert np.abs(P.sum(1) - 1).max() < 1e-14
    assert np.all(P[np.triu_indices(G, 1)] == 0)
    assert np.all(P[np.tril_indices(G)] > 0)


def test_locality_of_a_perturbation():
    """Changing k,v at one token moves O only at tokens of the same (head-dependent)
    group with an equal or later in-group index; includes the wrap-around group."""
    B, N, H, Hkv, D, G = 1, 32, 4, 4, 4, 8
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 6)
    o0, _ = orc.s2attn_fwd(q, k, v, G)
    for t in (1, 5, 30):          # token 1 sits in the wrap group of shifted heads
        k2, v2 = k.copy(), v.copy()
        k2[0, t] += 1.0
        v2[0, t] -= 1.0
        o1, _ = orc.s2attn_fwd(q, k2, v2, G)
        changed = np.abs(o1 - o0).max(axis=-1)[0] > 1e-13      # (N, H)
        for h in range(H):
            s = G // 2 if h >= H // 2 else 0
            p_t = (t - s) % N
            expect = np.zeros(N, bool)
            for tt in range(N):
                p = (tt - s) % N
                expect[tt] = (p // G == p_t // G) and (p % G >= p_t % G)
            assert np.array_equal(changed[:, h], expect), (t, h)
    # in particular the wrap leak of the default method: token 1 (first half) influences
    # nobody in [N-G/2, N) but is influenced by them
    k2 = k.copy(); k2[0, N - 1] += 1.0
    o1, _ = orc.s2attn_fwd(q, k2, v, G)
    assert np.abs(o1[0, 1, H - 1] - o0[0, 1, H - 1]).max() > 1e-6


def test_variant2_splits_the_wrap_group():
    B, N, H, Hkv, D, G = 1, 32, 2, 2, 4, 8
    q, k, v, _ = rand_problem(B, N, H, Hkv, D, 8)
    o, _, _, _, _ = orc.s2attn_fwd_bwd(q, k, v, None, G, variant2=True)
    o_def, _ = orc.s2attn_fwd(q, k, v, G)
    h = 1
    tail = np.arange(N - G // 2, N)
    head = np.arange(0, G // 2)
    for tok in (tail, head):
        ref = textbook_causal(q[0, tok, h], k[0, tok, h], v[0, tok, h], 1 / np.sqrt(D))
        assert np.abs(o[0, tok, h] - ref).max() < 1e-12
    rest = np.arange(G // 2, N - G // 2)
    assert np.array_equal(o[0, rest], o_def[0, rest])
    assert np.array_equal(o[0, :, 0], o_def[0, :, 0])


# ---------------------------------------------------------------- backward pins
def finite_difference_check(q, k, v, do, G, **kw):
    """Central differences of L = sum(o * do) in every element of q, k, v against the
    oracle's softmax-Jacobian gradients, for the oracle options in kw."""
    _, _, dq, dk, dv = orc.s2attn_fwd_bwd(q, k, v, do, G, **kw)

    def loss(q_, k_, v_):
        o, _ = orc.s2attn_fwd(q_, k_, v_, G, **kw)
        return float((o * do).sum())

    eps = 1e-5
    for x, gx, name in ((q, dq, "q"), (k, dk, "k"), (v, dv, "v")):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = loss(q, k, v)
            x[idx] = old - eps
            lm = loss(q, k, v)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        err = np.abs(num - gx).max() / max(1.0, np.abs(num).max())
        assert err < 1e-6, (name, kw, err)


@pytest.mark.parametrize("Hkv", [4, 2, 1])
def test_gradients_match_central_finite_differences(Hkv):
    B, N, H, D, G = 2, 16, 4, 4, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 10 + Hkv)
    finite_difference_check(q, k, v, do, G)


@pytest.mark.parametrize("kw", [
    dict(variant2=True),                          # Appendix B.3 Variant 2: the wrap group split in two
    dict(shift=3),                                # a shift other than G/2
    dict(shift=3, variant2=True),                 # ... with the split at G - shift = 5
    dict(shift_heads="all"),                      # every head shifted (Section 4.3 ablation)
    dict(shift_heads="none"),
])
def test_gradients_of_the_oracle_options_match_finite_differences(kw):
    B, N, H, Hkv, D, G = 1, 16, 4, 2, 4, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 40)
    finite_difference_check(q, k, v, do, G, **kw)


def test_gradients_match_autograd_through_library_attention():
    """G = N without shift: gradients equal autograd through torch's causal SDPA."""
    B, N, H, Hkv, D = 1, 24, 2, 2, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 20)
    _, _, dq, dk, dv = orc.s2attn_fwd_bwd(q, k, v, do, G=N, shift=0)
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3).clone().requires_grad_(True) for x in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    (o * torch.from_numpy(do).permute(0, 2, 1, 3)).sum().backward()
    for mine, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.abs(mine - ref.permute(0, 2, 1, 3).numpy()).max() < 1e-12


def test_gqa_gradients_equal_expanded_problem_summed():
    B, N, H, Hkv, D, G = 1, 16, 4, 2, 4, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 21)
    r = H // Hkv
    _, _, dq, dk, dv = orc.s2attn_fwd_bwd(q, k, v, do, G)
    ke, ve = np.repeat(k, r, axis=2), np.repeat(v, r, axis=2)
    oe, _, dqe, dke, dve = orc.s2attn_fwd_bwd(q, ke, ve, do, G)
    assert np.abs(dq - dqe).max() < 1e-13
    assert np.abs(dk - dke.reshape(B, N, Hkv, r, D).sum(3)).max() < 1e-13
    assert np.abs(dv - dve.reshape(B, N, Hkv, r, D).sum(3)).max() < 1e-13


def test_softmax_jacobian_identities():
    G, D = 9, 5
    q, k, v, do = (rng.standard_normal((G, D)) for _ in range(4))
    P, o, _ = orc.dense_group_attention(q, k, v, 0.3)
    dP = do @ v.T
    delta = (P * dP).sum(1)
    assert np.abs(delta - (do * o).sum(1)).max() < 1e-13        # delta_i = dO_i . O_i
    dS = P * (dP - delta[:, None])
    assert np.abs(dS.sum(1)).max() < 1e-13                      # rows of dS sum to zero
    assert np.all(dS[np.triu_indices(G, 1)] == 0)


def test_group_slice_agrees_with_full_tensor_run():
    B, N, H, Hkv, D, G = 1, 32, 8, 2, 4, 8
    q, k, v, do = rand_problem(B, N, H, Hkv, D, 22)
    o, lse, dq, dk, dv = orc.s2attn_fwd_bwd(q, k, v, do, G)
    for c in range(Hkv):
        for g in (0, N // G - 1):
            sl = orc.s2attn_group_slice(q, k, v, do, G, 0, c, g)
            tok, heads = sl["tokens"], sl["heads"]
            assert np.abs(o[0][np.ix_(tok, heads)] - sl["o"]).max() < 1e-13
            assert np.abs(dq[0][np.ix_(tok, heads)] - sl["dq"]).max() < 1e-13
            assert np.abs(lse[0][np.ix_(heads, tok)] - sl["lse"]).max() < 1e-13
            assert np.abs(dk[0, tok, c] - sl["dk"]).max() < 1e-13
            assert np.abs(dv[0, tok, c] - sl["dv"]).max() < 1e-13


def test_fp32_and_fp64_oracle_agree_on_a_long_group():
    G, D = 2048, 64
    r = np.random.default_rng(30)
    q, k, v, do = (r.standard_normal((1, G, 2, D)).astype(np.float32) for _ in range(4))
    a = orc.s2attn_fwd_bwd(q, k, v, do, G, shift=0, dtype=np.float32)
    b = orc.s2attn_fwd_bwd(q, k, v, do, G, shift=0, dtype=np.float64)
    for x, y in zip(a, b):
        assert np.abs(x - y).max() < 1e-4


def test_fp32_and_fp64_oracle_agree_at_the_benchmark_group_size():
    """One (kv head, group) slice at G = 8192, D = 128 (the size the GPU parity tests sample at
    the benchmark configurations, where the oracle runs in fp32): fp32 and fp64 runs of the same
    code agree to 1e-5, so the fp32 oracle's own rounding is far below the bf16 tolerance."""
    G, D = 8192, 128
    r = np.random.default_rng(31)
    q, k, v, do = (r.standard_normal((1, G, 2, D)).astype(np.float32) for _ in range(4))
    a = orc.s2attn_group_slice(q, k, v, do, G, 0, 0, 0, shift=0, dtype=np.float32)
    b = orc.s2attn_group_slice(q, k, v, do, G, 0, 0, 0, shift=0, dtype=np.float64)
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.abs(a[name] - b[name]).max() < 1e-5, name


def test_fp32_oracle_against_fp64_definition_at_the_100k_group_size():
    """G = 25600, D = 128 (the group size of the 100k-token configuration, where the GPU
    parity tests use the fp32 oracle): the fp32 run of one group against fp64 arithmetic
    written out here block by block from Equation 1 and the softmax Jacobian -- all of lse,
    o and dq on a row block in the middle and one at the end, dk and dv on the last keys
    (whose gradients need only the last rows) and on the first keys (all rows)."""
    G, D, scale = 25600, 128, 1 / np.sqrt(128)
    r = np.random.default_rng(32)
    q, k, v, do = (r.standard_normal((G, D)).astype(np.float32) for _ in range(4))
    P, o, lse = orc.dense_group_attention(q, k, v, np.float32(scale))
    dq, dk, dv = orc.dense_group_attention_grad(P, q, k, v, do, np.float32(scale))
    assert o.dtype == np.float32 and dq.dtype == np.float32
    del P
    q64, k64, v64, do64 = (x.astype(np.float64) for x in (q, k, v, do))

    def rows_fp64(i0, i1):
        S = scale * (q64[i0:i1] @ k64.T)
        S[np.arange(i0, i1)[:, None] < np.arange(G)[None, :]] = -np.inf
        m = S.max(1, keepdims=True)
        l = np.exp(S - m).sum(1, keepdims=True)
        Pb = np.exp(S - m) / l
        ob = Pb @ v64
        dP = do64[i0:i1] @ v64.T
        dS = Pb * (dP - (Pb * dP).sum(1, keepdims=True))
        return Pb, dS, ob, (m + np.log(l))[:, 0], scale * (dS @ k64)

    kb_first, kb_last = slice(0, 32), slice(G - 32, G)
    dk_first = np.zeros((32, D)); dv_first = np.zeros((32, D))
    step = 1600
    for i0 in range(0, G, step):
        Pb, dS, ob, lb, dqb = rows_fp64(i0, i0 + step)
        assert np.abs(lse[i0:i0 + step] - lb).max() < 2e-5
        if i0 in (12800, G - step):
            assert np.abs(o[i0:i0 + step] - ob).max() < 2e-5
            assert np.abs(dq[i0:i0 + step] - dqb).max() < 2e-5
        dv_first += Pb[:, kb_first].T @ do64[i0:i0 + step]
        dk_first += scale * (dS[:, kb_first].T @ q64[i0:i0 + step])
        if i0 == G - step:
            assert np.abs(dv[kb_last] - Pb[:, kb_last].T @ do64[i0:i0 + step]).max() < 2e-5
            assert np.abs(dk[kb_last] - scale * (dS[:, kb_last].T @ q64[i0:i0 + step])).max() < 2e-5
    assert np.abs(dv[kb_first] - dv_first).max() < 5e-5
    assert np.abs(dk[kb_first] - dk_first).max() < 5e-5
