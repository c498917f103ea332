"""Where the bf16 kernels round, written out in numpy (CPU, small shapes only).

This is not the oracle and takes no part in it.  The oracle is the exact arithmetic of LongLoRA
Section 3.2 / Algorithm 1; this model is the same arithmetic in fp64 with the three roundings
that a bf16 attention backward of the flash-attention kind makes by construction:
  1. P and dS = P * (dP - delta) are rounded to bf16 before they enter the second matrix product
     (dV = P^T dO, dQ = scale dS K, dK = scale dS^T Q);
  2. delta_i = sum_d dO_id O_id is formed from the output O as it was stored, i.e. rounded to bf16
     (the exact value is sum_j P_ij dP_ij);
  3. the results are rounded to bf16 when stored.
The GPU tests use it for one thing: an element that misses the stated bound against the oracle
has to be explained by these roundings, i.e. agree with this model.  (2) is what puts the worst
errors at the first keys of every causal run: there P is concentrated on a few keys, |O| is of
the size of a single V row, and the error of delta enters dS without averaging."""
import numpy as np


def to_bf16(x):
    """Round to nearest-even bf16, returned as float64."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).astype(np.float64)


def bf16_backward_model(q, k, v, do, G, shift=None, shift_heads="second_half", variant2=False, rounded=True):
    """q, do: (B, N, H, D); k, v: (B, N, Hkv, D), values already representable in bf16.
    Returns dq, dk, dv in fp64 with roundings 1 and 2 applied (not 3); rounded=False applies
    none, which must reproduce the oracle."""
    rnd = to_bf16 if rounded else (lambda x: x)
    q, k, v, do = (np.asarray(x, dtype=np.float64) for x in (q, k, v, do))
    B, N, H, D = q.shape
    Hkv = k.shape[2]
    r = H // Hkv
    scale = 1.0 / np.sqrt(D)
    s_arg = G // 2 if shift is None else shift
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    causal = np.tril(np.ones((G, G), dtype=bool))
    for b in range(B):
        for h in range(H):
            c = h // r
            s = {"second_half": s_arg if h >= H // 2 else 0, "none": 0, "all": s_arg}[shift_heads]
            fold = lambda x: np.roll(x, -s, axis=0).reshape(N // G, G, D)
            Q, K, V, DO = fold(q[b, :, h]), fold(k[b, :, c]), fold(v[b, :, c]), fold(do[b, :, h])
            for g in range(N // G):
                mask = causal
                if variant2 and s > 0 and g == N // G - 1:      # Appendix B.3 Variant 2
                    mask = causal.copy()
                    mask[G - s:, :G - s] = False
                S = np.where(mask, scale * Q[g] @ K[g].T, -np.inf)
                P = np.exp(S - S.max(axis=1, keepdims=True))
                P /= P.sum(axis=1, keepdims=True)
                delta = (DO[g] * rnd(P @ V[g])).sum(axis=1, keepdims=True)          # rounding 2
                dS = rnd(P * (DO[g] @ V[g].T - delta))                              # rounding 1
                rows = (np.arange(g * G, (g + 1) * G) + s) % N
                dq[b, rows, h] += scale * dS @ K[g]
                dk[b, rows, c] += scale * dS.T @ Q[g]
                dv[b, rows, c] += rnd(P).T @ DO[g]                                  # rounding 1
    return dq, dk, dv
