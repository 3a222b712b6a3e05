"""Pins for the fp64 CPU oracle: closed forms, textbook special cases, brute force,
finite differences and invariants.  None of these re-type the oracle's own loops."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _attention_matrix(q, k, lam):
    """A[t, s] = lam^(t-s) (q_t . k_s) for s <= t else 0, built with numpy (one head)."""
    n = q.shape[0]
    t = np.arange(n)[:, None]
    s = np.arange(n)[None, :]
    decay = np.where(t >= s, np.power(lam, np.maximum(t - s, 0)), 0.0)
    return (q @ k.T) * decay


FWD_FORMS = {
    "direct": lambda q, k, v, lam: oracle.fwd_direct(q, k, v, lam),
    "recurrent": lambda q, k, v, lam: oracle.fwd_recurrent(q, k, v, lam),
}
BWD_FORMS = {
    "direct": oracle.bwd_direct,
    "recurrent": oracle.bwd_recurrent,
}


# ---- P1: closed form (geometric series), Sec. 3.2.1 first equation with q = k = v = 1 ----------
@pytest.mark.parametrize("form", list(FWD_FORMS))
@pytest.mark.parametrize("d", [1, 3])
def test_closed_form_all_ones(form, d):
    n = 40
    lam = np.array([0.5, 0.9, 0.99])
    one = np.ones((2, 3, n, d))
    o = FWD_FORMS[form](one, one, one, lam)
    t = np.arange(1, n + 1)
    for h in range(3):
        expect = d * (1 - lam[h] ** t) / (1 - lam[h])
        assert np.allclose(o[:, h], expect[None, :, None], rtol=1e-13, atol=0)


def test_golden_geometric_series_lambda_half():
    """Stored dyadic values of sum_{m<t} (1/2)^m; exact in binary floating point."""
    vals = np.loadtxt(os.path.join(GOLDEN, "geometric_series_lambda_0p5.txt"), comments="#")
    n = vals.shape[0]
    one = np.ones((1, 1, n, 1))
    for form in FWD_FORMS.values():
        o = form(one, one, one, 0.5)[0, 0, :, 0]
        assert np.array_equal(o, vals[:, 1])
    rows = np.arange(n)
    assert np.array_equal(oracle.fwd_rows(one[0, 0], one[0, 0], one[0, 0], 0.5, rows)[:, 0], vals[:, 1])
    assert np.array_equal(oracle.block_forward(one[0, 0], one[0, 0], one[0, 0], 0.5, 4)[0][:, 0], vals[:, 1])


# ---- P2: lambda = 1 is the plain causal (lower-triangular) product / a prefix sum ----------------
@pytest.mark.parametrize("form", list(FWD_FORMS))
def test_lambda_one_is_tril_product(form):
    q, k, v = (_rand((1, 2, 33, 5), s) for s in (1, 2, 3))
    o = FWD_FORMS[form](q, k, v, 1.0)
    for h in range(2):
        expect = np.tril(q[0, h] @ k[0, h].T) @ v[0, h]
        assert np.allclose(o[0, h], expect, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("form", list(FWD_FORMS))
def test_lambda_one_scalar_is_cumsum(form):
    n = 100
    v = _rand((1, 1, n, 1), 4)
    one = np.ones_like(v)
    o = FWD_FORMS[form](one, one, v, 1.0)
    assert np.allclose(o[0, 0, :, 0], np.cumsum(v[0, 0, :, 0]), rtol=1e-12, atol=1e-12)


# ---- brute force with explicit Python loops on a tiny case ------------------------------------------
def test_python_triple_loop_tiny():
    n, d, lam = 6, 2, 0.7
    q, k, v, do = (_rand((1, 1, n, d), s) for s in (5, 6, 7, 8))
    o = np.zeros((n, d))
    dq, dk, dv = np.zeros((n, d)), np.zeros((n, d)), np.zeros((n, d))
    Q, K, V, DO = q[0, 0], k[0, 0], v[0, 0], do[0, 0]
    for t in range(n):
        for s in range(t + 1):
            w = lam ** (t - s)
            qk = sum(Q[t, i] * K[s, i] for i in range(d))
            dov = sum(DO[t, j] * V[s, j] for j in range(d))
            for j in range(d):
                o[t, j] += w * qk * V[s, j]
                dv[s, j] += w * qk * DO[t, j]
                dq[t, j] += w * dov * K[s, j]
                dk[s, j] += w * dov * Q[t, j]
    for f in FWD_FORMS.values():
        assert np.allclose(f(q, k, v, lam)[0, 0], o, rtol=1e-13, atol=1e-13)
    for f in BWD_FORMS.values():
        g = f(q, k, v, do, lam)
        for got, exp in zip(g, (dq, dk, dv)):
            assert np.allclose(got[0, 0], exp, rtol=1e-13, atol=1e-13)


# ---- matrix form with library matmuls: O = A V, dV = A^T dO, dA = (dO V^T) * decay -------------------
@pytest.mark.parametrize("lam", [0.3, 0.95, 1.0])
def test_matrix_form(lam):
    n, d = 48, 8
    q, k, v, do = (_rand((1, 1, n, d), s) for s in (9, 10, 11, 12))
    Q, K, V, DO = q[0, 0], k[0, 0], v[0, 0], do[0, 0]
    A = _attention_matrix(Q, K, lam)
    G = _attention_matrix(DO, V, lam)          # dL/d(QK^T) with the decay folded in
    for f in FWD_FORMS.values():
        assert np.allclose(f(q, k, v, lam)[0, 0], A @ V, rtol=1e-12, atol=1e-12)
    for f in BWD_FORMS.values():
        dq, dk, dv = f(q, k, v, do, lam)
        assert np.allclose(dq[0, 0], G @ K, rtol=1e-12, atol=1e-12)
        assert np.allclose(dk[0, 0], G.T @ Q, rtol=1e-12, atol=1e-12)
        assert np.allclose(dv[0, 0], A.T @ DO, rtol=1e-12, atol=1e-12)


# ---- P3: the two forms agree (multi batch / multi head / per-head lambda) -----------------------------
def test_direct_equals_recurrent():
    shape = (2, 3, 64, 8)
    q, k, v, do = (_rand(shape, s) for s in (13, 14, 15, 16))
    lam = np.array([0.43, 0.9, 0.9961])
    o1, o2 = oracle.fwd_direct(q, k, v, lam), oracle.fwd_recurrent(q, k, v, lam)
    assert np.max(np.abs(o1 - o2)) <= 1e-12 * np.max(np.abs(o1))
    for a, b in zip(oracle.bwd_direct(q, k, v, do, lam), oracle.bwd_recurrent(q, k, v, do, lam)):
        assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))


def test_head_and_batch_indexing():
    """Each (batch, head) slice must equal a one-head call with that head's lambda."""
    shape = (2, 3, 20, 4)
    q, k, v, do = (_rand(shape, s) for s in (17, 18, 19, 20))
    lam = np.array([0.5, 0.8, 0.99])
    o = oracle.fwd_direct(q, k, v, lam)
    g = oracle.bwd_direct(q, k, v, do, lam)
    for b, h in itertools.product(range(2), range(3)):
        A = _attention_matrix(q[b, h], k[b, h], lam[h])
        assert np.allclose(o[b, h], A @ v[b, h], rtol=1e-12, atol=1e-12)
        assert np.allclose(g[2][b, h], A.T @ do[b, h], rtol=1e-12, atol=1e-12)


# ---- P4: the block decomposition of Algorithms 1 and 2 equals the definition for every B | n --------------
@pytest.mark.parametrize("B", [1, 2, 4, 8, 16, 32])
def test_block_form_equals_direct(B):
    n, d, lam = 32, 4, 0.85
    q, k, v, do = (_rand((1, 1, n, d), s) for s in (21, 22, 23, 24))
    o = oracle.fwd_direct(q, k, v, lam)[0, 0]
    O, states = oracle.block_forward(q[0, 0], k[0, 0], v[0, 0], lam, B)
    assert np.allclose(O, o, rtol=1e-12, atol=1e-13)
    # the state at block boundary t is sum_{s <= tB} lam^(tB - s) k_s^T v_s (definition of KV_t), spelled out here
    # with plain loops
    for t, KV in enumerate(states):
        expect = np.zeros((d, d))
        for s in range(1, t * B + 1):
            expect += lam ** (t * B - s) * np.outer(k[0, 0, s - 1], v[0, 0, s - 1])
        assert np.allclose(KV, expect, rtol=1e-12, atol=1e-13)
    dq, dk, dv = oracle.bwd_direct(q, k, v, do, lam)
    bq, bk, bv, dstates = oracle.block_backward(q[0, 0], k[0, 0], v[0, 0], do[0, 0], lam, B)
    for a, b in ((bq, dq), (bk, dk), (bv, dv)):
        assert np.allclose(a, b[0, 0], rtol=1e-12, atol=1e-13)
    for t, dKV in enumerate(dstates):
        expect = np.zeros((d, d))
        for s in range(t * B + 1, n + 1):
            expect += lam ** (s - t * B) * np.outer(q[0, 0, s - 1], do[0, 0, s - 1])
        assert np.allclose(dKV, expect, rtol=1e-12, atol=1e-13)
    # ... and the states obey the one-step updates the two algorithms carry from block to block
    rf, rr = oracle.state_update_residuals(q[0, 0], k[0, 0], v[0, 0], do[0, 0], lam, B)
    assert rf <= 1e-13 and rr <= 1e-13


def test_recurrent_final_state_is_block_state():
    n, d, lam = 24, 3, 0.9
    q, k, v = (_rand((1, 1, n, d), s) for s in (25, 26, 27))
    _, kvf = oracle.fwd_recurrent(q, k, v, lam, return_state=True)
    _, states = oracle.block_forward(q[0, 0], k[0, 0], v[0, 0], lam, 8)
    assert np.allclose(kvf[0, 0], states[-1], rtol=1e-12, atol=1e-13)


def test_reverse_state_at_the_first_boundary_is_the_gradient_of_the_start_state():
    """dKV_0 of the block form is d_kv_init of the segment backward (Sec. 3.2.2's recursion carried one step past
    the first position)."""
    n, d, lam = 24, 3, 0.8
    q, k, v, do = (_rand((1, 1, n, d), s) for s in (35, 36, 37, 38))
    *_, g0 = oracle.bwd_recurrent_state(q, k, v, do, lam)
    *_, dstates = oracle.block_backward(q[0, 0], k[0, 0], v[0, 0], do[0, 0], lam, 6)
    assert np.allclose(g0[0, 0], dstates[0], rtol=1e-12, atol=1e-13)


# ---- P5: central finite differences of L = sum(O * dO) -------------------------------------------------
@pytest.mark.parametrize("form", list(BWD_FORMS))
def test_finite_differences(form):
    shape = (1, 2, 7, 3)
    q, k, v, do = (_rand(shape, s) for s in (28, 29, 30, 31))
    lam = np.array([0.6, 0.97])
    dq, dk, dv = BWD_FORMS[form](q, k, v, do, lam)

    def loss(q_, k_, v_):
        return float(np.sum(oracle.fwd_direct(q_, k_, v_, lam) * do))

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        fd = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": q, "k": k, "v": v}
            args_m = dict(args_p)
            args_p[name], args_m[name] = xp, xm
            fd[idx] = (loss(**{a + "_": args_p[a] for a in "qkv"}) - loss(**{a + "_": args_m[a] for a in "qkv"})) / (2 * eps)
        assert np.allclose(fd, g, rtol=1e-7, atol=1e-8), name


# ---- P6: Euler identity (L is linear in each of Q, K, V) -------------------------------------------------
def test_euler_identity():
    shape = (2, 2, 50, 6)
    q, k, v, do = (_rand(shape, s) for s in (32, 33, 34, 35))
    lam = np.array([0.7, 0.99])
    o = oracle.fwd_direct(q, k, v, lam)
    dq, dk, dv = oracle.bwd_direct(q, k, v, do, lam)
    L = np.sum(o * do)
    for g, x in ((dq, q), (dk, k), (dv, v)):
        assert abs(np.sum(g * x) - L) <= 1e-11 * abs(L) + 1e-11


# ---- P7: causality ------------------------------------------------------------------------------------------
def test_causality():
    shape = (1, 1, 30, 4)
    q, k, v, do = (_rand(shape, s) for s in (36, 37, 38, 39))
    lam, cut = 0.9, 17
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for x in (q2, k2, v2):
        x[..., cut:, :] += 1.0
    for f in FWD_FORMS.values():
        assert np.array_equal(f(q, k, v, lam)[..., :cut, :], f(q2, k2, v2, lam)[..., :cut, :])
    do2 = do.copy()
    do2[..., :cut, :] -= 2.0
    for f in BWD_FORMS.values():
        a, b = f(q, k, v, do, lam), f(q, k, v, do2, lam)
        assert np.array_equal(a[1][..., cut:, :], b[1][..., cut:, :])
        assert np.array_equal(a[2][..., cut:, :], b[2][..., cut:, :])


# ---- P8: lambda -> 0+ leaves only the diagonal term ------------------------------------------------------------
@pytest.mark.parametrize("form", list(FWD_FORMS))
def test_lambda_to_zero(form):
    shape = (1, 1, 12, 5)
    q, k, v = (_rand(shape, s) for s in (40, 41, 42))
    o = FWD_FORMS[form](q, k, v, 1e-200)
    expect = np.sum(q * k, axis=-1, keepdims=True) * v
    assert np.allclose(o, expect, rtol=1e-13, atol=1e-13)


# ---- P9: decode steps reproduce the forward, and the state's definition ---------------------------------------
def test_decode_equals_forward():
    b, H, n, d = 2, 2, 19, 4
    q, k, v = (_rand((b, H, n, d), s) for s in (43, 44, 45))
    lam = np.array([0.5, 0.95])
    o = oracle.fwd_direct(q, k, v, lam)
    kv = np.zeros((b, H, d, d))
    for t in range(n):
        ot = oracle.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], lam, kv)
        assert np.allclose(ot, o[:, :, t], rtol=1e-12, atol=1e-13)
    for bi, h in itertools.product(range(b), range(H)):
        expect = sum(lam[h] ** (n - 1 - s) * np.outer(k[bi, h, s], v[bi, h, s]) for s in range(n))
        assert np.allclose(kv[bi, h], expect, rtol=1e-12, atol=1e-13)


def test_decode_step_formula_and_order():
    b, H, d = 2, 3, 5
    q, k, v = (_rand((b, H, d), s) for s in (46, 47, 48))
    kv0 = _rand((b, H, d, d), 49)
    lam = np.array([0.4, 0.9, 1.0])
    kv = kv0.copy()
    o = oracle.decode_step(q, k, v, lam, kv)
    expect_kv = lam[None, :, None, None] * kv0 + np.einsum("bhi,bhj->bhij", k, v)
    assert np.allclose(kv, expect_kv, rtol=1e-14, atol=1e-14)
    assert np.allclose(o, np.einsum("bhi,bhij->bhj", q, expect_kv), rtol=1e-13, atol=1e-13)
    # the output reads the UPDATED state: from a zero state o = (q . k) v
    z = np.zeros((b, H, d, d))
    o0 = oracle.decode_step(q, k, v, lam, z)
    assert np.allclose(o0, np.sum(q * k, -1, keepdims=True) * v, rtol=1e-13, atol=1e-13)


def test_recurrent_initial_state():
    """Running on the second half from the first half's final state equals the full run."""
    b, H, n, d = 1, 2, 16, 3
    q, k, v = (_rand((b, H, n, d), s) for s in (50, 51, 52))
    lam = np.array([0.8, 0.99])
    full = oracle.fwd_direct(q, k, v, lam)
    _, st = oracle.fwd_recurrent(q[:, :, :8], k[:, :, :8], v[:, :, :8], lam, return_state=True)
    second = oracle.fwd_recurrent(q[:, :, 8:], k[:, :, 8:], v[:, :, 8:], lam, kv_init=st)
    assert np.allclose(second, full[:, :, 8:], rtol=1e-12, atol=1e-13)


# ---- P10: time-reversal duality of the backward ---------------------------------------------------------------
def test_time_reversal_duality():
    shape = (1, 2, 21, 4)
    q, k, v, do = (_rand(shape, s) for s in (53, 54, 55, 56))
    lam = np.array([0.6, 0.98])
    dq, dk, dv = oracle.bwd_direct(q, k, v, do, lam)
    rev = lambda x: x[:, :, ::-1, :].copy()
    # dV(s) = sum_{t>=s} lam^(t-s) (k_s . q_t) do_t : forward on the reversed sequence with q<-k, k<-q, v<-do
    assert np.allclose(rev(oracle.fwd_direct(rev(k), rev(q), rev(do), lam)), dv, rtol=1e-12, atol=1e-13)
    assert np.allclose(rev(oracle.fwd_direct(rev(v), rev(do), rev(q), lam)), dk, rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.fwd_direct(do, v, k, lam), dq, rtol=1e-12, atol=1e-13)


# ---- the sampled-row entry points equal the full tensors ---------------------------------------------------------
def test_rows_equal_full():
    n, d, lam = 70, 6, 0.93
    q, k, v, do = (_rand((1, 1, n, d), s) for s in (57, 58, 59, 60))
    rows = np.array([0, 1, 31, 32, 63, 64, 69])
    o = oracle.fwd_direct(q, k, v, lam)[0, 0]
    assert np.allclose(oracle.fwd_rows(q[0, 0], k[0, 0], v[0, 0], lam, rows), o[rows], rtol=1e-13, atol=1e-14)
    G = _attention_matrix(do[0, 0], v[0, 0], lam)
    A = _attention_matrix(q[0, 0], k[0, 0], lam)
    rq, rk, rv = oracle.bwd_rows(q[0, 0], k[0, 0], v[0, 0], do[0, 0], lam, rows)
    assert np.allclose(rq, (G @ k[0, 0])[rows], rtol=1e-12, atol=1e-13)
    assert np.allclose(rk, (G.T @ q[0, 0])[rows], rtol=1e-12, atol=1e-13)
    assert np.allclose(rv, (A.T @ do[0, 0])[rows], rtol=1e-12, atol=1e-13)


def test_empty_sequence():
    z = np.zeros((1, 1, 0, 4))
    assert oracle.fwd_direct(z, z, z, 0.9).shape == (1, 1, 0, 4)
    assert oracle.fwd_recurrent(z, z, z, 0.9).shape == (1, 1, 0, 4)
    assert all(g.shape == (1, 1, 0, 4) for g in oracle.bwd_direct(z, z, z, z, 0.9))


# ---- P11: segments with state hand-over (Sec. 3.2.1 recursion started from a non-zero state; the
# chain rule through it).  The reference is always the whole sequence in the DIRECT form, which knows
# nothing about states.
def _segments(n, cuts):
    edges = [0] + list(cuts) + [n]
    return [slice(a, b) for a, b in zip(edges[:-1], edges[1:])]


@pytest.mark.parametrize("cuts", [(8,), (1,), (15,), (5, 11), (3, 3, 9)])
def test_state_handover_forward_and_backward_equal_the_whole_sequence(cuts):
    b, H, n, d = 2, 2, 16, 3
    q, k, v, do = (_rand((b, H, n, d), s) for s in (70, 71, 72, 73))
    lam = np.array([0.7, 0.97])
    o_full = oracle.fwd_direct(q, k, v, lam)
    dq_full, dk_full, dv_full = oracle.bwd_direct(q, k, v, do, lam)
    segs = _segments(n, cuts)
    # forward, left to right
    state, starts, outs = None, [], []
    for s in segs:
        starts.append(state)
        o, state = oracle.fwd_recurrent(q[:, :, s], k[:, :, s], v[:, :, s], lam, kv_init=state, return_state=True)
        outs.append(o)
    assert np.allclose(np.concatenate(outs, axis=2), o_full, rtol=1e-12, atol=1e-13)
    # backward, right to left: the gradient of a segment's start state is the next-left segment's d_kv_final
    g, grads = None, []
    for s, st in zip(reversed(segs), reversed(starts)):
        dq, dk, dv, g = oracle.bwd_recurrent_state(q[:, :, s], k[:, :, s], v[:, :, s], do[:, :, s], lam,
                                                   kv_init=st, d_kv_final=g)
        grads.append((dq, dk, dv))
    grads.reverse()
    for i, ref in enumerate((dq_full, dk_full, dv_full)):
        assert np.allclose(np.concatenate([x[i] for x in grads], axis=2), ref, rtol=1e-12, atol=1e-13)


def test_state_closed_form_scalar():
    """d = 1, q = k = v = 1: kv_t = lam^t kv_0 + (1 - lam^t)/(1 - lam), o_t = kv_t."""
    n, lam, kv0 = 25, 0.9, 3.5
    one = np.ones((1, 1, n, 1))
    o, kvf = oracle.fwd_recurrent(one, one, one, lam, kv_init=np.full((1, 1, 1, 1), kv0), return_state=True)
    t = np.arange(1, n + 1)
    expect = lam ** t * kv0 + (1 - lam ** t) / (1 - lam)
    assert np.allclose(o[0, 0, :, 0], expect, rtol=1e-13, atol=0)
    assert np.isclose(kvf[0, 0, 0, 0], expect[-1], rtol=1e-13, atol=0)
    # gradients of L = sum_t w_t o_t + c kv_n with respect to kv_0: sum_t w_t lam^t + c lam^n
    w = _rand((1, 1, n, 1), 74)
    c = 1.7
    *_, g0 = oracle.bwd_recurrent_state(one, one, one, w, lam, kv_init=np.full((1, 1, 1, 1), kv0),
                                        d_kv_final=np.full((1, 1, 1, 1), c))
    assert np.isclose(g0[0, 0, 0, 0], np.sum(w[0, 0, :, 0] * lam ** t) + c * lam ** n, rtol=1e-12, atol=0)


def test_state_gradients_by_finite_differences():
    b, H, n, d = 1, 2, 7, 3
    q, k, v, do = (_rand((b, H, n, d), s) for s in (75, 76, 77, 78))
    kv0, wfin = _rand((b, H, d, d), 79), _rand((b, H, d, d), 80)
    lam = np.array([0.85, 0.6])

    def loss(q_, k_, v_, kv0_):
        o, kvf = oracle.fwd_recurrent(q_, k_, v_, lam, kv_init=kv0_, return_state=True)
        return np.sum(o * do) + np.sum(kvf * wfin)

    dq, dk, dv, dkv0 = oracle.bwd_recurrent_state(q, k, v, do, lam, kv_init=kv0, d_kv_final=wfin)
    eps = 1e-6
    args = [q, k, v, kv0]
    for ai, grad in enumerate((dq, dk, dv, dkv0)):
        rng = np.random.default_rng(81 + ai)
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in args[ai].shape)
            hi = [a.copy() for a in args]
            lo = [a.copy() for a in args]
            hi[ai][idx] += eps
            lo[ai][idx] -= eps
            fd = (loss(*hi) - loss(*lo)) / (2 * eps)
            assert np.isclose(grad[idx], fd, rtol=1e-6, atol=1e-8), (ai, idx, grad[idx], fd)


def test_state_edge_cases():
    b, H, d = 1, 2, 3
    lam = np.array([0.9, 0.5])
    z = np.zeros((b, H, 0, d))
    kv0, g = _rand((b, H, d, d), 90), _rand((b, H, d, d), 91)
    # empty segment: the state passes through unchanged in both directions
    _, kvf = oracle.fwd_recurrent(z, z, z, lam, kv_init=kv0, return_state=True)
    assert np.array_equal(kvf, kv0)
    *_, g0 = oracle.bwd_recurrent_state(z, z, z, z, lam, kv_init=kv0, d_kv_final=g)
    assert np.array_equal(g0, g)
    # without states the segment backward is the plain backward
    q, k, v, do = (_rand((b, H, 9, d), s) for s in (92, 93, 94, 95))
    got = oracle.bwd_recurrent_state(q, k, v, do, lam)
    for a, ref in zip(got[:3], oracle.bwd_direct(q, k, v, do, lam)):
        assert np.allclose(a, ref, rtol=1e-12, atol=1e-13)
    # prefill -> decode hand-over: the final state continues with single steps
    o_full = oracle.fwd_direct(*(np.concatenate([x, y], axis=2) for x, y in
                                 zip((q, k, v), (_rand((b, H, 1, d), s) for s in (96, 97, 98)))), lam)
    qn, kn, vn = (_rand((b, H, 1, d), s)[:, :, 0] for s in (96, 97, 98))
    _, kvf = oracle.fwd_recurrent(q, k, v, lam, return_state=True)
    assert np.allclose(oracle.decode_step(qn, kn, vn, lam, kvf), o_full[:, :, -1], rtol=1e-12, atol=1e-13)


# ---- P12: the normalised operator, Sec. 2.1 eq. (2) (Norm read as RMS normalisation of every output row) -----
def test_norm_single_position_by_hand():
    """n = 1: u = (q . k) v, so o = sign(q . k) v / rms(v) at eps = 0 (worked by hand for d = 2)."""
    q = np.array([[[[2.0, -1.0]]]])
    k = np.array([[[[0.5, 3.0]]]])          # q . k = -2
    v = np.array([[[[3.0, -4.0]]]])         # rms(v) = sqrt(12.5)
    o, rstd = oracle.fwd_norm(q, k, v, 0.9, 0.0)
    assert np.allclose(o[0, 0, 0], [-3.0 / np.sqrt(12.5), 4.0 / np.sqrt(12.5)], rtol=1e-15)
    assert np.allclose(rstd[0, 0, 0], 1.0 / (2.0 * np.sqrt(12.5)), rtol=1e-15)
    # with eps: mean(u^2) = 4 * 12.5 = 50
    o, rstd = oracle.fwd_norm(q, k, v, 0.9, 14.0)
    assert np.allclose(rstd[0, 0, 0], 1.0 / 8.0, rtol=1e-15)
    assert np.allclose(o[0, 0, 0], [-6.0 / 8.0, 8.0 / 8.0], rtol=1e-15)


def test_norm_rows_have_unit_rms_and_keep_direction():
    shape = (2, 3, 33, 8)
    q, k, v = (_rand(shape, s) for s in (90, 91, 92))
    lam = np.array([0.5, 0.9, 1.0])
    o, rstd = oracle.fwd_norm(q, k, v, lam, 0.0)
    assert np.allclose(np.mean(o * o, axis=-1), 1.0, rtol=1e-13)
    u = oracle.fwd_recurrent(q, k, v, lam)   # the other form of the un-normalised operator
    assert np.allclose(o, u * rstd[..., None], rtol=1e-11, atol=1e-13)
    assert np.all(rstd > 0)
    # positive eps shrinks every row: rms < 1, same direction
    o2, rstd2 = oracle.fwd_norm(q, k, v, lam, 0.3)
    assert np.all(np.mean(o2 * o2, axis=-1) < 1.0)
    assert np.allclose(o2 * rstd[..., None], o * rstd2[..., None], rtol=1e-12, atol=1e-15)
    assert np.allclose(1.0 / rstd2 ** 2 - 1.0 / rstd ** 2, 0.3, rtol=1e-10)


def test_norm_scale_invariance_and_large_eps_limit():
    shape = (1, 2, 20, 4)
    q, k, v = (_rand(shape, s) for s in (93, 94, 95))
    lam = np.array([0.8, 0.97])
    o, _ = oracle.fwd_norm(q, k, v, lam, 0.0)
    for a, b, c in ((3.0, 1.0, 1.0), (1.0, 0.25, 1.0), (1.0, 1.0, 7.0)):
        o2, _ = oracle.fwd_norm(a * q, b * k, c * v, lam, 0.0)
        assert np.allclose(o2, o, rtol=1e-12, atol=1e-14)
    o3, _ = oracle.fwd_norm(-q, k, v, lam, 0.0)
    assert np.allclose(o3, -o, rtol=1e-12, atol=1e-14)
    # eps far above mean(u^2): Norm tends to u / sqrt(eps), the un-normalised operator up to a constant
    big = 1e12
    o4, _ = oracle.fwd_norm(q, k, v, lam, big)
    assert np.allclose(o4 * np.sqrt(big), oracle.fwd_direct(q, k, v, lam), rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("eps", [0.0, 0.05])
def test_norm_gradients_by_finite_differences(eps):
    shape = (1, 2, 6, 3)
    q, k, v, do = (_rand(shape, s) for s in (96, 97, 98, 99))
    lam = np.array([0.6, 0.95])
    grads = dict(zip("qkv", oracle.bwd_norm(q, k, v, do, lam, eps)))

    def loss(**a):
        return float(np.sum(oracle.fwd_norm(a["q"], a["k"], a["v"], lam, eps)[0] * do))

    h = 1e-6
    base = {"q": q, "k": k, "v": v}
    for name in "qkv":
        fd = np.zeros(shape)
        for idx in np.ndindex(*shape):
            ap, am = dict(base), dict(base)
            ap[name], am[name] = base[name].copy(), base[name].copy()
            ap[name][idx] += h
            am[name][idx] -= h
            fd[idx] = (loss(**ap) - loss(**am)) / (2 * h)
        assert np.allclose(fd, grads[name], rtol=2e-6, atol=2e-8), name


def test_norm_with_state_by_finite_differences_and_composition():
    """The normalised operator on a segment with state hand-over: two segments compose to the whole sequence,
    and the gradients (also with respect to the start state, also of a loss on the final state) match central
    finite differences of the forward function."""
    shape = (1, 2, 7, 3)
    q, k, v, do = (_rand(shape, s) for s in (196, 197, 198, 199))
    kv0, dkvn = _rand((1, 2, 3, 3), 200), _rand((1, 2, 3, 3), 201)
    lam, eps = np.array([0.6, 0.95]), 0.05
    # composition: [0, 4) then [4, 7) from the first segment's state == the whole sequence, == fwd_norm from zero
    o, r, kvn = oracle.fwd_norm_state(q, k, v, lam, eps, kv0)
    o1, r1, s1 = oracle.fwd_norm_state(q[:, :, :4], k[:, :, :4], v[:, :, :4], lam, eps, kv0)
    o2, r2, s2 = oracle.fwd_norm_state(q[:, :, 4:], k[:, :, 4:], v[:, :, 4:], lam, eps, s1)
    assert np.allclose(np.concatenate([o1, o2], 2), o, rtol=1e-12, atol=1e-14)
    assert np.allclose(np.concatenate([r1, r2], 2), r, rtol=1e-12) and np.allclose(s2, kvn, rtol=1e-12, atol=1e-14)
    oz, rz, _ = oracle.fwd_norm_state(q, k, v, lam, eps, None)
    of, rf = oracle.fwd_norm(q, k, v, lam, eps)
    assert np.allclose(oz, of, rtol=1e-12, atol=1e-14) and np.allclose(rz, rf, rtol=1e-12)
    # gradients
    grads = dict(zip(("q", "k", "v", "kv0"), oracle.bwd_norm_state(q, k, v, do, lam, eps, kv0, dkvn)))

    def loss(**a):
        o_, _, kvn_ = oracle.fwd_norm_state(a["q"], a["k"], a["v"], lam, eps, a["kv0"])
        return float(np.sum(o_ * do) + np.sum(kvn_ * dkvn))

    h = 1e-6
    base = {"q": q, "k": k, "v": v, "kv0": kv0}
    for name in base:
        fd = np.zeros(base[name].shape)
        for idx in np.ndindex(*base[name].shape):
            ap, am = dict(base), dict(base)
            ap[name], am[name] = base[name].copy(), base[name].copy()
            ap[name][idx] += h
            am[name][idx] -= h
            fd[idx] = (loss(**ap) - loss(**am)) / (2 * h)
        assert np.allclose(fd, grads[name], rtol=2e-6, atol=2e-8), name


def test_norm_gradients_are_orthogonal_to_their_inputs_at_eps_zero():
    """At eps = 0 the loss is homogeneous of degree 0 in each of Q, K, V: <dX, X> = 0; with eps > 0 it is not."""
    shape = (2, 2, 40, 5)
    q, k, v, do = (_rand(shape, s) for s in (100, 101, 102, 103))
    lam = np.array([0.7, 0.99])
    dq, dk, dv = oracle.bwd_norm(q, k, v, do, lam, 0.0)
    scale = np.sum(np.abs(dq * q))
    for g, x in ((dq, q), (dk, k), (dv, v)):
        assert abs(np.sum(g * x)) <= 1e-11 * scale
    # per row: dU_t is orthogonal to o_t
    o, rstd = oracle.fwd_norm(q, k, v, lam, 0.0)
    du = oracle.norm_backward_rows(o, rstd, do)
    assert np.max(np.abs(np.sum(du * o, axis=-1))) <= 1e-12 * np.max(np.abs(du))
    dq2, _, _ = oracle.bwd_norm(q, k, v, do, lam, 0.5)
    assert abs(np.sum(dq2 * q)) > 1e-3 * np.sum(np.abs(dq2 * q))


def test_norm_packed_is_the_dense_operator_sequence_by_sequence():
    """Packed sequences are chains of their own: equal lengths reproduce the dense batch; a sequence's rows do not
    depend on its neighbours; finite differences of the packed loss agree with the packed gradients."""
    H, d, eps = 2, 3, 1e-3
    lam = np.array([0.7, 0.95])
    # equal lengths == dense batch
    b, n = 3, 5
    q, k, v, g = (_rand((b, H, n, d), s) for s in (90, 91, 92, 93))
    pack = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3).reshape(b * n, H, d))
    cu = np.arange(0, (b + 1) * n, n)
    o_p, r_p = oracle.fwd_norm_packed(pack(q), pack(k), pack(v), lam, cu, eps)
    o_d, r_d = oracle.fwd_norm(q, k, v, lam, eps)
    assert np.array_equal(o_p, pack(o_d))
    assert np.array_equal(r_p, r_d.transpose(1, 0, 2).reshape(H, b * n))
    for got, ref in zip(oracle.bwd_norm_packed(pack(q), pack(k), pack(v), pack(g), lam, cu, eps), oracle.bwd_norm(q, k, v, g, lam, eps)):
        assert np.array_equal(got, pack(ref))
    # unequal lengths with a gap in front: neighbours do not interact, rows outside stay zero
    cu = np.array([2, 6, 6, 13])
    total = 15
    q, k, v, g = (_rand((total, H, d), s) for s in (94, 95, 96, 97))
    o1, r1 = oracle.fwd_norm_packed(q, k, v, lam, cu, eps)
    k2 = k.copy()
    k2[6:13] += 1.0                      # the last sequence changes
    o2, _ = oracle.fwd_norm_packed(q, k2, v, lam, cu, eps)
    assert np.array_equal(o1[:6], o2[:6]) and not np.allclose(o1[6:13], o2[6:13])
    assert np.all(o1[:2] == 0) and np.all(o1[13:] == 0) and np.all(r1[:, :2] == 0)
    dq, dk, dv = oracle.bwd_norm_packed(q, k, v, g, lam, cu, eps)
    loss = lambda q_, k_, v_: float(np.sum(oracle.fwd_norm_packed(q_, k_, v_, lam, cu, eps)[0] * g))
    rng = np.random.default_rng(5)
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(6):
            idx = (int(rng.integers(0, total)), int(rng.integers(0, H)), int(rng.integers(0, d)))
            h = 1e-6
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name], args_m[name] = xp, xm
            fd = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])
