"""The block decomposition of Sec. 3.2.1 / 3.2.2, checked from the definitions in fp64 numpy.

TEST INFRASTRUCTURE ONLY.  One head at a time: Q, K, V, dO are [n, d], lambda a scalar, B a block size that
divides n; positions are numbered 1 .. n and block t (1 .. T) holds positions (t-1) B + 1 .. t B.

Nothing here runs a loop over blocks with a running state.  The two families of states are written down from
their definitions for ALL block boundaries at once,

    KV_t  = sum_{s <= t B} lambda^(t B - s) k_s^T v_s          (Sec. 3.2.1, definition of KV_t),      t = 0 .. T
    dKV_t = sum_{s >  t B} lambda^(s - t B) q_s^T do_s          (Sec. 3.2.2, the reverse sum),         t = 0 .. T

and every block's output is then formed independently of the others as intra-block part (the masked B x B
product inside the block) plus inter-block part (the block's rows, each carrying the decay from the block
boundary to its own position, times the state at that boundary).  That the states also obey the one-step
updates that Algorithms 1 and 2 carry from block to block is a separate statement, returned as residuals by
state_update_residuals().  Row r (1 .. B) of a block is lambda^r away from the block's lower boundary and
lambda^(B - r) away from its upper one: the first is the diagonal the algorithm boxes call Lambda, the second
what they write as lambda^B Lambda^-1 (no inverse is formed here).
"""
import numpy as np


def _boundary_weights(lam, n, B, after):
    """W[t, s-1]: weight of position s in the state at block boundary t (t = 0 .. n/B).
    after = False: positions s <= t B, lambda^(t B - s); after = True: positions s > t B, lambda^(s - t B)."""
    s = np.arange(1, n + 1, dtype=np.float64)[None, :]
    edge = (np.arange(n // B + 1, dtype=np.float64) * B)[:, None]
    dist = (s - edge) if after else (edge - s)
    inside = (s > edge) if after else (s <= edge)
    return np.where(inside, np.power(float(lam), np.where(inside, dist, 0.0)), 0.0)


def _blocks(X, B):
    n, d = X.shape
    return X.reshape(n // B, B, d)


def _decay_mask(lam, B):
    """[r, c] -> lambda^(r - c) for r >= c, else 0 (the mask M of both algorithm boxes)."""
    r = np.arange(B)[:, None]
    c = np.arange(B)[None, :]
    return np.where(r >= c, np.power(float(lam), np.where(r >= c, r - c, 0).astype(np.float64)), 0.0)


def block_forward(Q, K, V, lam, B):
    """O [n, d] from the block decomposition, and KV_0 .. KV_T [T + 1, d, d] from their definition."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    n, d = Q.shape
    assert n % B == 0
    KV = np.einsum("ts,si,sj->tij", _boundary_weights(lam, n, B, after=False), K, V)
    Qb, Kb, Vb = _blocks(Q, B), _blocks(K, B), _blocks(V, B)
    to_lower = np.power(float(lam), np.arange(1, B + 1, dtype=np.float64))     # lambda^r
    scores = np.einsum("trk,tck->trc", Qb, Kb) * _decay_mask(lam, B)[None]
    intra = np.einsum("trc,tcj->trj", scores, Vb)
    inter = np.einsum("tri,tij->trj", Qb * to_lower[None, :, None], KV[:-1])    # block t starts from KV_{t-1}
    return (intra + inter).reshape(n, d), KV


def block_backward(Q, K, V, dO, lam, B):
    """dQ, dK, dV [n, d] from the block decomposition, and dKV_0 .. dKV_T [T + 1, d, d] from their definition."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    n, d = Q.shape
    assert n % B == 0
    KV = np.einsum("ts,si,sj->tij", _boundary_weights(lam, n, B, after=False), K, V)
    dKV = np.einsum("ts,si,sj->tij", _boundary_weights(lam, n, B, after=True), Q, dO)
    Qb, Kb, Vb, Gb = _blocks(Q, B), _blocks(K, B), _blocks(V, B), _blocks(dO, B)
    r = np.arange(1, B + 1, dtype=np.float64)
    to_lower, to_upper = np.power(float(lam), r), np.power(float(lam), B - r)
    M = _decay_mask(lam, B)[None]
    qk = np.einsum("trk,tck->trc", Qb, Kb) * M       # [(Q K^T) * M] per block
    gv = np.einsum("trk,tck->trc", Gb, Vb) * M       # [(dO V^T) * M] per block
    dQ = np.einsum("trc,tcj->trj", gv, Kb) + np.einsum("trj,tij->tri", Gb * to_lower[None, :, None], KV[:-1])
    dK = np.einsum("trc,trj->tcj", gv, Qb) + np.einsum("trj,tij->tri", Vb * to_upper[None, :, None], dKV[1:])
    dV = np.einsum("trc,trj->tcj", qk, Gb) + np.einsum("tri,tij->trj", Kb * to_upper[None, :, None], dKV[1:])
    return dQ.reshape(n, d), dK.reshape(n, d), dV.reshape(n, d), dKV


def state_update_residuals(Q, K, V, dO, lam, B):
    """Largest absolute violation of the two one-step state updates by the states as defined:
        KV_t      = lambda^B KV_{t-1} + (rows of K_t weighted lambda^(B - r))^T V_t         (Algorithm 1)
        dKV_{t-1} = lambda^B dKV_t    + (rows of Q_t weighted lambda^r)^T dO_t              (Algorithm 2)
    Both are exact identities of the sums, so the residuals are round-off."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    _, KV = block_forward(Q, K, V, lam, B)
    _, _, _, dKV = block_backward(Q, K, V, dO, lam, B)
    r = np.arange(1, B + 1, dtype=np.float64)
    to_lower, to_upper = np.power(float(lam), r), np.power(float(lam), B - r)
    lamB = float(lam) ** B
    fwd = KV[1:] - (lamB * KV[:-1] + np.einsum("tri,trj->tij", _blocks(K, B) * to_upper[None, :, None], _blocks(V, B)))
    rev = dKV[:-1] - (lamB * dKV[1:] + np.einsum("tri,trj->tij", _blocks(Q, B) * to_lower[None, :, None], _blocks(dO, B)))
    return float(np.max(np.abs(fwd))) if fwd.size else 0.0, float(np.max(np.abs(rev))) if rev.size else 0.0
