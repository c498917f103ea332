"""Plain CPU oracle for shifted sparse attention (S2-Attn), forward and backward.

TEST INFRASTRUCTURE ONLY: a slow, obviously-correct numpy implementation used to
check the HIP kernels.  It shares no code with them and is never imported by the
product path.

What it computes (LongLoRA, arXiv 2309.12307):
  * Section 3.2 / Algorithm 1: the head axis is cut into two contiguous halves;
    the second half is rolled by -G/2 along the token axis; the token axis is
    folded into N/G groups of G tokens that become batch entries; a standard
    self-attention runs on every group; the second half of the output is rolled
    back by +G/2.
  * Equation 1 with the conventions a "standard self-attention function" of a
    decoder has: scores scaled by 1/sqrt(D) and a causal mask, both taken in the
    rolled, in-group index (key j is visible to query i iff j <= i).
  * The wrap-around group of the shifted heads (last G/2 tokens followed by the
    first G/2 tokens, Section 3.2 worked example) is kept as one causal group,
    as in the paper's default method; `variant2=True` gives Appendix B.3's
    Variant 2 instead, where the two halves of that group are separate groups.
  * The paper has no backward text; gradients are those of the forward map,
    written out with the softmax Jacobian:
        dV = P^T dO,  dP = dO V^T,
        dS_ik = P_ik (dP_ik - sum_j P_ij dP_ij),
        dQ = scale dS K,  dK = scale dS^T Q.
  * Grouped-query attention (Hkv < H; the paper fine-tunes Llama2-70B, Section
    4.1, but never discusses it): query head h reads kv head h // (H/Hkv); the
    shift is a property of the query head; dK, dV sum over the query heads that
    share a kv head.

Pins (tests/test_oracle_*.py): the paper's worked index example, the FLOP table
of the efficiency analysis, central finite differences, textbook/library full
causal attention for G=N without shift, block-diagonal attention for unshifted
heads, closed forms (Q=0, constant V, first row of a group), locality of
perturbations, and an independent N x N-mask formulation without any roll.
At the large benchmark shapes the values are not pinned separately: the same
code that passed the small pins is trusted there ("parity unpinned" beyond the
fp32-vs-fp64 self-agreement check).

Layouts: q, o, dO, dq are (B, N, H, D); k, v, dk, dv are (B, N, Hkv, D);
lse is (B, H, N), natural log of the sum of exp of scaled masked scores,
indexed by ORIGINAL token position.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "head_shift", "rolled_to_token", "token_to_rolled", "group_tokens",
    "dense_group_attention", "dense_group_attention_grad",
    "s2attn_fwd", "s2attn_fwd_bwd", "s2attn_fwd_masked",
    "s2attn_group_slice", "attn_flops_paper", "attn_flops_causal",
]


# --------------------------------------------------------------------------
# Index map (Algorithm 1, "Key line 1"/"Key line 2"; Section 3.2 worked example)
# --------------------------------------------------------------------------
def head_shift(h: int, H: int, G: int, shift: int | None = None,
               shift_heads: str = "second_half") -> int:
    """Shift s_h of query head h.  Default: G/2 for the second contiguous half
    of the heads (chunk(2, head_axis)[1]) and 0 for the first half."""
    s = G // 2 if shift is None else shift
    if shift_heads == "second_half":
        return s if h >= H // 2 else 0
    if shift_heads == "none":
        return 0
    if shift_heads == "all":
        return s
    raise ValueError(shift_heads)


def rolled_to_token(p, s: int, N: int):
    """roll(x, -s)[p] = x[(p + s) mod N]: rolled position p holds token (p+s) mod N."""
    return (np.asarray(p) + s) % N


def token_to_rolled(t, s: int, N: int):
    return (np.asarray(t) - s) % N


def group_tokens(g: int, s: int, N: int, G: int) -> np.ndarray:
    """Original token indices of group g (in in-group order) for a head with shift s."""
    return rolled_to_token(np.arange(g * G, (g + 1) * G), s, N)


# --------------------------------------------------------------------------
# One group: dense causal softmax attention and its gradient (Equation 1)
# --------------------------------------------------------------------------
def dense_group_attention(q, k, v, scale, split: int | None = None):
    """q, k, v: (G, D) rows in in-group order.  Returns P (G,G), o (G,D), lse (G,).

    split: if given, rows/cols [0,split) and [split,G) form two independent
    causal blocks (Variant 2 of Appendix B.3 for the wrap-around group)."""
    G = q.shape[0]
    S = scale * (q @ k.T)
    i = np.arange(G)[:, None]
    j = np.arange(G)[None, :]
    visible = j <= i
    if split is not None:
        visible &= (i < split) == (j < split)
    S = np.where(visible, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    P = E / l
    o = P @ v
    lse = m[:, 0] + np.log(l[:, 0])
    return P, o, lse


def dense_group_attention_grad(P, q, k, v, do, scale):
    """Gradients of sum(o * do) for one group, from the softmax Jacobian."""
    dv = P.T @ do
    dP = do @ v.T
    delta = (P * dP).sum(axis=1, keepdims=True)
    dS = P * (dP - delta)
    dq = scale * (dS @ k)
    dk = scale * (dS.T @ q)
    return dq, dk, dv


# --------------------------------------------------------------------------
# Whole op, following Algorithm 1 step by step (roll materialised)
# --------------------------------------------------------------------------
def _check(q, k, v, G):
    B, N, H, D = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, N, Hkv, D) or v.shape != k.shape:
        raise ValueError("k/v shape")
    if N % G or G % 2 or H % 2 or H % Hkv:
        raise ValueError("need N % G == 0, G even, H even, H % Hkv == 0")
    return B, N, H, Hkv, D


def s2attn_fwd_bwd(q, k, v, do, G, scale=None, shift=None,
                   shift_heads="second_half", variant2=False, dtype=np.float64):
    """Forward and (if do is not None) backward of S2-Attn.

    Returns (o, lse, dq, dk, dv); the gradients are None when do is None."""
    B, N, H, Hkv, D = _check(q, k, v, G)
    r = H // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    q = np.asarray(q, dtype=dtype)
    k = np.asarray(k, dtype=dtype)
    v = np.asarray(v, dtype=dtype)
    o = np.empty((B, N, H, D), dtype=dtype)
    lse = np.empty((B, H, N), dtype=dtype)
    bwd = do is not None
    if bwd:
        do = np.asarray(do, dtype=dtype)
        dq = np.empty((B, N, H, D), dtype=dtype)
        dk = np.zeros((B, N, Hkv, D), dtype=dtype)
        dv = np.zeros((B, N, Hkv, D), dtype=dtype)
    for b in range(B):
        for h in range(H):
            c = h // r                                   # GQA: kv head of query head h
            s = head_shift(h, H, G, shift, shift_heads)
            # Key line 1: roll by -s on the token axis, then fold into groups
            qr = np.roll(q[b, :, h, :], -s, axis=0).reshape(N // G, G, D)
            kr = np.roll(k[b, :, c, :], -s, axis=0).reshape(N // G, G, D)
            vr = np.roll(v[b, :, c, :], -s, axis=0).reshape(N // G, G, D)
            orl = np.empty((N // G, G, D), dtype=dtype)
            lser = np.empty((N // G, G), dtype=dtype)
            if bwd:
                dor = np.roll(do[b, :, h, :], -s, axis=0).reshape(N // G, G, D)
                dqr = np.empty_like(qr)
                dkr = np.empty_like(kr)
                dvr = np.empty_like(vr)
            for g in range(N // G):
                split = None
                if variant2 and 0 < s < G and g == N // G - 1:
                    split = G - s        # in-group rows [0,G-s) are tokens [N-G+s,N); the rest are tokens [0,s)
                P, orl[g], lser[g] = dense_group_attention(qr[g], kr[g], vr[g], scale, split)
                if bwd:
                    dqr[g], dkr[g], dvr[g] = dense_group_attention_grad(
                        P, qr[g], kr[g], vr[g], dor[g], scale)
            # Key line 2: roll back by +s
            o[b, :, h, :] = np.roll(orl.reshape(N, D), s, axis=0)
            lse[b, h, :] = np.roll(lser.reshape(N), s, axis=0)
            if bwd:
                dq[b, :, h, :] = np.roll(dqr.reshape(N, D), s, axis=0)
                dk[b, :, c, :] += np.roll(dkr.reshape(N, D), s, axis=0)   # GQA reduce
                dv[b, :, c, :] += np.roll(dvr.reshape(N, D), s, axis=0)
    if bwd:
        return o, lse, dq, dk, dv
    return o, lse, None, None, None


def s2attn_fwd(q, k, v, G, **kw):
    o, lse, _, _, _ = s2attn_fwd_bwd(q, k, v, None, G, **kw)
    return o, lse


# --------------------------------------------------------------------------
# Independent formulation: N x N mask in ORIGINAL token coordinates, no roll
# --------------------------------------------------------------------------
def s2attn_fwd_masked(q, k, v, G, scale=None, shift=None, shift_heads="second_half",
                      dtype=np.float64):
    """Same op written without any roll: for head h with shift s, token t sits at
    rolled position p(t) = (t - s) mod N, in group p // G at in-group index p % G;
    query t sees key t' iff both are in the same group and index(t') <= index(t)."""
    B, N, H, Hkv, D = _check(q, k, v, G)
    r = H // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    q = np.asarray(q, dtype=dtype); k = np.asarray(k, dtype=dtype); v = np.asarray(v, dtype=dtype)
    o = np.empty((B, N, H, D), dtype=dtype)
    lse = np.empty((B, H, N), dtype=dtype)
    t = np.arange(N)
    for b in range(B):
        for h in range(H):
            s = head_shift(h, H, G, shift, shift_heads)
            p = (t - s) % N
            grp, idx = p // G, p % G
            M = (grp[:, None] == grp[None, :]) & (idx[None, :] <= idx[:, None])
            S = scale * (q[b, :, h, :] @ k[b, :, h // r, :].T)
            S = np.where(M, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            l = E.sum(axis=1, keepdims=True)
            o[b, :, h, :] = (E / l) @ v[b, :, h // r, :]
            lse[b, h, :] = m[:, 0] + np.log(l[:, 0])
    return o, lse


# --------------------------------------------------------------------------
# One (batch, kv head, group) slice of a big problem, for sampled parity checks
# --------------------------------------------------------------------------
def s2attn_group_slice(q, k, v, do, G, b, c, g, scale=None, shift=None,
                       shift_heads="second_half", dtype=np.float64):
    """Outputs restricted to the tokens of group g for kv head c and all of its
    r = H/Hkv query heads, which must share one shift (true whenever Hkv is even
    under the default rule).  Returns dict with tokens (G,), heads (r,),
    o (G,r,D), lse (r,G), dq (G,r,D), dk (G,D), dv (G,D)."""
    B, N, H, Hkv, D = _check(q, k, v, G)
    r = H // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    heads = np.arange(c * r, (c + 1) * r)
    shifts = {head_shift(int(h), H, G, shift, shift_heads) for h in heads}
    if len(shifts) != 1:
        raise ValueError("query heads of this kv head do not share a shift")
    s = shifts.pop()
    tok = group_tokens(g, s, N, G)
    kg = np.asarray(k[b, tok, c, :], dtype=dtype)
    vg = np.asarray(v[b, tok, c, :], dtype=dtype)
    out = dict(tokens=tok, heads=heads,
               o=np.empty((G, r, D), dtype), lse=np.empty((r, G), dtype),
               dq=np.empty((G, r, D), dtype),
               dk=np.zeros((G, D), dtype), dv=np.zeros((G, D), dtype))
    for n, h in enumerate(heads):
        qg = np.asarray(q[b, tok, h, :], dtype=dtype)
        P, out["o"][:, n], out["lse"][n] = dense_group_attention(qg, kg, vg, scale)
        if do is not None:
            dog = np.asarray(do[b, tok, h, :], dtype=dtype)
            dqg, dkg, dvg = dense_group_attention_grad(P, qg, kg, vg, dog, scale)
            out["dq"][:, n] = dqg
            out["dk"] += dkg
            out["dv"] += dvg
    return out


# --------------------------------------------------------------------------
# FLOP counters
# --------------------------------------------------------------------------
def attn_flops_paper(N, G, d_model, n_layers):
    """Convention of the efficiency-analysis FLOP table: two N x G x d_model
    matmuls per layer at 2 FLOPs per multiply-add, forward only, no causal
    discount.  G = N gives the full-attention row."""
    return 4 * N * G * d_model * n_layers


def attn_flops_causal(B, N, H, D, G, backward=True):
    """Effective FLOPs of one S2-Attn layer counting only in-group causal pairs:
    B*H*N*(G+1)/2 (query, key) pairs; 2 matmuls forward (4D per pair) and
    5 backward (10D per pair)."""
    pairs = B * H * N * (G + 1) // 2
    fwd = 4 * D * pairs
    return fwd + (10 * D * pairs if backward else 0)
