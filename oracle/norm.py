"""fp64 oracle of the normalised operator O = Norm(Q (K^T V)) with the decay and causal mask
(Sec. 2.1 eq. (2) with the recurrence of Sec. 3.2.1 inside the Norm).  TEST INFRASTRUCTURE ONLY.

The paper names Norm without defining it and leaves it out of its derivations (Sec. 3.2.1).  Reading
taken here: root-mean-square normalisation of every output row over the head's feature dimension,
without a learnable gain:

    u_t = sum_{s<=t} lambda^(t-s) (q_t . k_s) v_s            (the un-normalised output row)
    r_t = 1 / sqrt( mean_j u_{t,j}^2 + eps )
    o_t = r_t u_t

Backward: with g_t the gradient of the loss with respect to o_t, the gradient with respect to u_t is

    dU_t = r_t ( g_t - o_t * mean_j(g_{t,j} o_{t,j}) )

(differentiate r_t: d r_t / d u_{t,j} = - r_t^3 u_{t,j} / d; exact for any eps >= 0), and dQ, dK, dV
are the un-normalised operator's gradients for dU.  Everything is plain numpy on top of the direct
O(n^2) forms of the C oracle.
"""
import numpy as np

from . import ref


def fwd_norm(q, k, v, lam, eps):
    """Returns (o, rstd): o [batch, heads, n, d] normalised rows, rstd [batch, heads, n] = r_t."""
    u = ref.fwd_direct(q, k, v, lam)
    rstd = 1.0 / np.sqrt(np.mean(u * u, axis=-1) + eps)
    return u * rstd[..., None], rstd


def fwd_norm_state(q, k, v, lam, eps, kv_init=None):
    """One segment of a longer sequence (recurrence of Sec. 3.2.1 started from kv_init): returns (o, rstd,
    kv_final).  The state carries the un-normalised recurrence; only the output rows are normalised."""
    u, kv_final = ref.fwd_recurrent(q, k, v, lam, kv_init=kv_init, return_state=True)
    rstd = 1.0 / np.sqrt(np.mean(u * u, axis=-1) + eps)
    return u * rstd[..., None], rstd, kv_final


def bwd_norm_state(q, k, v, d_o, lam, eps, kv_init=None, d_kv_final=None):
    """Gradients (dq, dk, dv, d_kv_init) of sum(d_o * o) + sum(d_kv_final * kv_final) for fwd_norm_state."""
    o, rstd, _ = fwd_norm_state(q, k, v, lam, eps, kv_init)
    du = norm_backward_rows(o, rstd, d_o)
    return ref.bwd_recurrent_state(q, k, v, du, lam, kv_init=kv_init, d_kv_final=d_kv_final)


def norm_backward_rows(o, rstd, g):
    """dU from the normalised output o, r_t and the incoming gradient g (all per row)."""
    o = np.asarray(o, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    c = np.mean(g * o, axis=-1, keepdims=True)
    return np.asarray(rstd, dtype=np.float64)[..., None] * (g - o * c)


def bwd_norm(q, k, v, d_o, lam, eps):
    """Returns (dq, dk, dv) of sum(d_o * fwd_norm(q, k, v)[0])."""
    o, rstd = fwd_norm(q, k, v, lam, eps)
    du = norm_backward_rows(o, rstd, d_o)
    return ref.bwd_direct(q, k, v, du, lam)


def fwd_norm_packed(q, k, v, lam, cu_seqlens, eps):
    """The normalised operator over PACKED sequences: q, k, v are [total_positions, heads, d]; sequence b is the rows
    cu_seqlens[b] .. cu_seqlens[b + 1] - 1 and a chain of its own.  Returns (o [total, heads, d], rstd [heads, total]);
    rows outside every sequence are zero."""
    q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
    total, heads, _ = q.shape
    o = np.zeros_like(q)
    rstd = np.zeros((heads, total))
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if hi > lo:
            seq = [np.ascontiguousarray(x[lo:hi].transpose(1, 0, 2))[None] for x in (q, k, v)]   # [1, heads, n, d]
            ob, rb = fwd_norm(seq[0], seq[1], seq[2], lam, eps)
            o[lo:hi] = ob[0].transpose(1, 0, 2)
            rstd[:, lo:hi] = rb[0]
    return o, rstd


def bwd_norm_packed(q, k, v, d_o, lam, cu_seqlens, eps):
    """(dq, dk, dv), each [total_positions, heads, d], of sum(d_o * fwd_norm_packed(...)[0]); zero outside the sequences."""
    q, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, k, v, d_o))
    grads = [np.zeros_like(q) for _ in range(3)]
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if hi > lo:
            seq = [np.ascontiguousarray(x[lo:hi].transpose(1, 0, 2))[None] for x in (q, k, v, d_o)]
            for dst, gb in zip(grads, bwd_norm(seq[0], seq[1], seq[2], seq[3], lam, eps)):
                dst[lo:hi] = gb[0].transpose(1, 0, 2)
    return tuple(grads)
