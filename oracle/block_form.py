"""Algorithm 1 and Algorithm 2 of the paper, taken step by step in fp64 numpy.

TEST INFRASTRUCTURE ONLY.  One head at a time: Q, K, V, dO are [n, d], lambda a
scalar, B a block size dividing n.  Notation follows the paper: M is the B x B
decay mask, Lambda = diag(lambda^1 .. lambda^B) (the definition given in both
algorithm boxes; the shifted diag(1 .. lambda^(B-1)) printed once in Sec. 3.2.1 is
not used), and lambda^B Lambda^-1 = diag(lambda^(B-1) .. 1) is written out
explicitly so no inverse is ever formed.  In Algorithm 2's second loop the block
gradients dK_i, dV_i use the tiles of block i together with the dKV accumulated
from the blocks after i, and only then dKV is updated with block i.
"""
import numpy as np


def _mask(lam, B):
    i = np.arange(B)[:, None]
    j = np.arange(B)[None, :]
    e = (i - j).astype(np.float64)
    return np.where(i >= j, np.power(float(lam), np.maximum(e, 0.0)), 0.0)


def alg1_forward(Q, K, V, lam, B, return_states=False):
    """Algorithm 1.  Returns O [n, d] (and the list KV_0 .. KV_T when asked)."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    n, d = Q.shape
    assert n % B == 0
    T = n // B
    M = _mask(lam, B)
    r = np.arange(1, B + 1, dtype=np.float64)
    Lam = np.power(float(lam), r)            # diagonal of Lambda
    LamB_inv = np.power(float(lam), B - r)   # diagonal of lambda^B Lambda^-1
    KV = np.zeros((d, d))
    states = [KV.copy()]
    O = np.empty_like(Q)
    for i in range(T):
        sl = slice(i * B, (i + 1) * B)
        Qi, Ki, Vi = Q[sl], K[sl], V[sl]
        O_intra = ((Qi @ Ki.T) * M) @ Vi
        O_inter = (Lam[:, None] * Qi) @ KV
        KV = float(lam) ** B * KV + (LamB_inv[:, None] * Ki).T @ Vi
        O[sl] = O_intra + O_inter
        states.append(KV.copy())
    return (O, states) if return_states else O


def alg2_backward(Q, K, V, dO, lam, B):
    """Algorithm 2.  Returns dQ, dK, dV, each [n, d]."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    n, d = Q.shape
    assert n % B == 0
    T = n // B
    M = _mask(lam, B)
    r = np.arange(1, B + 1, dtype=np.float64)
    Lam = np.power(float(lam), r)
    LamB_inv = np.power(float(lam), B - r)
    lamB = float(lam) ** B
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    KV = np.zeros((d, d))
    for i in range(T):
        sl = slice(i * B, (i + 1) * B)
        Ki, Vi, dOi = K[sl], V[sl], dO[sl]
        dQ_intra = ((dOi @ Vi.T) * M) @ Ki
        dQ_inter = (Lam[:, None] * dOi) @ KV.T
        KV = lamB * KV + (LamB_inv[:, None] * Ki).T @ Vi
        dQ[sl] = dQ_intra + dQ_inter
    dKV = np.zeros((d, d))
    for i in range(T - 1, -1, -1):
        sl = slice(i * B, (i + 1) * B)
        Qi, Ki, Vi, dOi = Q[sl], K[sl], V[sl], dO[sl]
        dK_intra = ((dOi @ Vi.T) * M).T @ Qi
        dK_inter = (LamB_inv[:, None] * Vi) @ dKV.T
        dV_intra = ((Qi @ Ki.T) * M).T @ dOi
        dV_inter = (LamB_inv[:, None] * Ki) @ dKV
        dKV = lamB * dKV + (Lam[:, None] * Qi).T @ dOi
        dK[sl] = dK_intra + dK_inter
        dV[sl] = dV_intra + dV_inter
    return dQ, dK, dV
