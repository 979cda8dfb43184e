"""Pins for the fp64 attention oracle: everything here is fixed by the paper's definition
(section 2.1), by closed forms, by invariants of softmax attention, or by a library routine
on tiny inputs -- never by the oracle's own output and never by the HIP path."""
import math

import numpy as np
import pytest
import scipy.special

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _library_attention(q, k, v, alpha, causal):
    """Textbook route on one head: scipy's softmax / logsumexp on the dense score matrix."""
    s = alpha * (q @ k.T)
    if causal:
        n = s.shape[0]
        s = np.where(np.tril(np.ones((n, n), bool)), s, -np.inf)
    return scipy.special.softmax(s, axis=1) @ v, scipy.special.logsumexp(s, axis=1)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(1, 1), (2, 3), (7, 4), (16, 8), (33, 5)])
def test_matches_library_softmax_on_tiny_inputs(N, d, causal):
    B, H = 2, 3
    q, k, v = (_rand(s, B, H, N, d) for s in (1, 2, 3))
    alpha = 0.37
    o, lse = oracle.attention_fwd(q, k, v, alpha, causal)
    for b in range(B):
        for h in range(H):
            o_ref, l_ref = _library_attention(q[b, h], k[b, h], v[b, h], alpha, causal)
            np.testing.assert_allclose(o[b, h], o_ref, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[b, h], l_ref, rtol=1e-12, atol=1e-13)


def test_hand_computed_two_keys():
    # N=2, d=1, alpha=0.5: q=[1,2], k=[1,-1], v=[3,5]; scores row0 = [.5,-.5], row1 = [1,-1]
    q = np.array([1.0, 2.0]).reshape(1, 1, 2, 1)
    k = np.array([1.0, -1.0]).reshape(1, 1, 2, 1)
    v = np.array([3.0, 5.0]).reshape(1, 1, 2, 1)
    o, lse = oracle.attention_fwd(q, k, v, 0.5, False)
    for i, s in enumerate([0.5, 1.0]):
        ea, eb = math.exp(s), math.exp(-s)
        assert o[0, 0, i, 0] == pytest.approx((3 * ea + 5 * eb) / (ea + eb), rel=1e-14)
        assert lse[0, 0, i] == pytest.approx(math.log(ea + eb), rel=1e-14)
    # causal: row 0 sees only key 0
    o, lse = oracle.attention_fwd(q, k, v, 0.5, True)
    assert o[0, 0, 0, 0] == 3.0 and lse[0, 0, 0] == pytest.approx(0.5)
    ea, eb = math.exp(1.0), math.exp(-1.0)
    assert o[0, 0, 1, 0] == pytest.approx((3 * ea + 5 * eb) / (ea + eb), rel=1e-14)


def test_single_key_returns_that_value_row():
    q, k, v = (_rand(s, 1, 2, 1, 8) for s in (4, 5, 6))
    o, lse = oracle.attention_fwd(q, k, v, 0.25, False)
    np.testing.assert_allclose(o, v, rtol=0, atol=0)
    np.testing.assert_allclose(lse[..., 0], 0.25 * np.sum(q * k, axis=-1)[..., 0], rtol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_softmax_rows_sum_to_one_and_mask_is_lower_triangular(causal):
    N, d = 40, 8
    q, k, v = (_rand(s, N, d) for s in (7, 8, 9))
    P = oracle.attention_probs(q, k, v, 0.3, causal)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert (P >= 0).all()
    if causal:
        assert np.all(np.triu(P, 1) == 0) and np.all(np.diag(P) > 0)
    # exp(s - L) reproduces P: ties L to the scores it claims to summarise
    _, lse = oracle.attention_fwd(q[None, None], k[None, None], v[None, None], 0.3, causal)
    s = 0.3 * q @ k.T
    P2 = np.exp(s - lse[0, 0][:, None])
    if causal:
        P2 = np.tril(P2)
    np.testing.assert_allclose(P, P2, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("causal", [False, True])
def test_constant_value_rows_give_that_row(causal):
    B, H, N, d = 1, 2, 50, 16
    q, k = _rand(10, B, H, N, d), _rand(11, B, H, N, d)
    row = _rand(12, d)
    v = np.broadcast_to(row, (B, H, N, d)).copy()
    o, _ = oracle.attention_fwd(q, k, v, 0.2, causal)
    np.testing.assert_allclose(o, v, rtol=1e-13, atol=1e-14)


def test_causal_row_zero_is_first_value_row():
    B, H, N, d = 2, 2, 19, 8
    q, k, v = (_rand(s, B, H, N, d) for s in (13, 14, 15))
    o, lse = oracle.attention_fwd(q, k, v, 0.5, True)
    np.testing.assert_array_equal(o[:, :, 0], v[:, :, 0])
    np.testing.assert_allclose(lse[:, :, 0], 0.5 * np.sum(q[:, :, 0] * k[:, :, 0], -1), rtol=1e-14)
    # last causal row equals the last non-causal row
    o_nc, lse_nc = oracle.attention_fwd(q, k, v, 0.5, False)
    np.testing.assert_allclose(o[:, :, -1], o_nc[:, :, -1], rtol=1e-14)
    np.testing.assert_allclose(lse[:, :, -1], lse_nc[:, :, -1], rtol=1e-14)


def test_zero_queries_give_means_and_log_counts():
    B, H, N, d = 1, 2, 37, 4
    k, v = _rand(16, B, H, N, d), _rand(17, B, H, N, d)
    q = np.zeros_like(k)
    o, lse = oracle.attention_fwd(q, k, v, 0.7, False)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(N), rtol=1e-14)
    o, lse = oracle.attention_fwd(q, k, v, 0.7, True)
    prefix = np.cumsum(v, axis=2) / np.arange(1, N + 1)[None, None, :, None]
    np.testing.assert_allclose(o, prefix, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, np.broadcast_to(np.log(np.arange(1, N + 1)), lse.shape), rtol=1e-14)


def test_key_shift_leaves_output_and_shifts_logsumexp():
    B, H, N, d = 1, 1, 23, 6
    q, k, v = (_rand(s, B, H, N, d) for s in (18, 19, 20))
    c = _rand(21, d)
    alpha = 0.41
    o0, l0 = oracle.attention_fwd(q, k, v, alpha, False)
    o1, l1 = oracle.attention_fwd(q, k + c, v, alpha, False)
    np.testing.assert_allclose(o1, o0, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, alpha * (q @ c), rtol=1e-11, atol=1e-12)


def test_joint_key_value_permutation_invariance():
    B, H, N, d = 1, 2, 29, 4
    q, k, v = (_rand(s, B, H, N, d) for s in (22, 23, 24))
    perm = np.random.default_rng(25).permutation(N)
    o0, l0 = oracle.attention_fwd(q, k, v, 0.3, False)
    o1, l1 = oracle.attention_fwd(q, k[:, :, perm], v[:, :, perm], 0.3, False)
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l1, l0, rtol=1e-13)


def test_large_scale_selects_argmax_key():
    B, H, N, d = 1, 1, 17, 5
    q, k, v = (_rand(s, B, H, N, d) for s in (26, 27, 28))
    o, _ = oracle.attention_fwd(q, k, v, 1e4, False)
    best = np.argmax(q[0, 0] @ k[0, 0].T, axis=1)
    np.testing.assert_allclose(o[0, 0], v[0, 0][best], rtol=1e-9, atol=1e-9)


def test_split_merge_identity_through_logsumexp():
    # attention over [K1; K2] is the exp(L)-weighted mean of attention over the halves
    B, H, N, d = 1, 2, 24, 8
    q, k, v = (_rand(s, B, H, N, d) for s in (29, 30, 31))
    a = 0.35
    o, l = oracle.attention_fwd(q, k, v, a, False)
    h = 10
    # the halves are not square problems, so they go through the library softmax
    for hh in range(H):
        s = a * q[0, hh] @ k[0, hh].T
        o1, l1 = scipy.special.softmax(s[:, :h], 1) @ v[0, hh, :h], scipy.special.logsumexp(s[:, :h], 1)
        o2, l2 = scipy.special.softmax(s[:, h:], 1) @ v[0, hh, h:], scipy.special.logsumexp(s[:, h:], 1)
        w1, w2 = np.exp(l1 - l[0, hh]), np.exp(l2 - l[0, hh])
        np.testing.assert_allclose(w1 + w2, 1.0, rtol=1e-12)
        np.testing.assert_allclose(w1[:, None] * o1 + w2[:, None] * o2, o[0, hh], rtol=1e-11, atol=1e-13)


def test_row_subset_equals_full():
    B, H, N, d = 2, 2, 31, 8
    q, k, v = (_rand(s, B, H, N, d) for s in (32, 33, 34))
    for causal in (False, True):
        o, l = oracle.attention_fwd(q, k, v, 0.3, causal)
        rows = np.array([0, 5, 30, 31, 77, B * H * N - 1])
        o_r, l_r = oracle.attention_fwd_rows(q, k, v, rows, 0.3, causal)
        np.testing.assert_array_equal(o_r, o.reshape(-1, d)[rows])
        np.testing.assert_array_equal(l_r, l.reshape(-1)[rows])


# ---------------------------------------------------------------- backward


def _phi(q, k, v, dout, alpha, causal):
    o, _ = oracle.attention_fwd(q, k, v, alpha, causal)
    return float(np.sum(o * dout))


@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_central_finite_differences(causal):
    B, H, N, d = 1, 2, 6, 4
    q, k, v, dout = (_rand(s, B, H, N, d) for s in (40, 41, 42, 43))
    alpha = 0.6
    g = oracle.attention_bwd(q, k, v, dout, alpha, causal)
    h = 1e-6
    for name, x, grad in (("dq", q, g["dq"]), ("dk", k, g["dk"]), ("dv", v, g["dv"])):
        fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + h
            fp = _phi(q, k, v, dout, alpha, causal)
            x[idx] = old - h
            fm = _phi(q, k, v, dout, alpha, causal)
            x[idx] = old
            fd[idx] = (fp - fm) / (2 * h)
        np.testing.assert_allclose(grad, fd, rtol=2e-6, atol=2e-8, err_msg=name)


@pytest.mark.parametrize("causal", [False, True])
def test_backward_identities(causal):
    B, H, N, d = 1, 2, 21, 8
    q, k, v, dout = (_rand(s, B, H, N, d) for s in (44, 45, 46, 47))
    alpha = 0.3
    g = oracle.attention_bwd(q, k, v, dout, alpha, causal)
    o, lse = oracle.attention_fwd(q, k, v, alpha, causal)
    np.testing.assert_array_equal(g["o"], o)
    np.testing.assert_array_equal(g["lse"], lse)
    # <Q,dQ> = <K,dK> (both are alpha * sum_ij dS_ij s_ij / alpha)
    assert np.sum(q * g["dq"]) == pytest.approx(np.sum(k * g["dk"]), rel=1e-10)
    for hh in range(H):
        P = oracle.attention_probs(q[0, hh], k[0, hh], v[0, hh], alpha, causal)
        dP = dout[0, hh] @ v[0, hh].T
        # D = rowsum(dO o O) equals rowsum(P o dP)  (Algorithm 3 writes D in R^d; it is one scalar per row)
        np.testing.assert_allclose(g["D"][0, hh], np.sum(P * dP, axis=1), rtol=1e-11, atol=1e-13)
        # dsoftmax in its Jacobian form (diag(p) - p p^T) dp, row by row
        dS = np.stack([(np.diag(P[i]) - np.outer(P[i], P[i])) @ dP[i] for i in range(N)])
        np.testing.assert_allclose(dS.sum(axis=1), 0.0, atol=1e-13)
        np.testing.assert_allclose(g["dq"][0, hh], alpha * dS @ k[0, hh], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(g["dk"][0, hh], alpha * dS.T @ q[0, hh], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(g["dv"][0, hh], P.T @ dout[0, hh], rtol=1e-10, atol=1e-13)


def test_backward_constant_values_have_zero_query_key_gradients():
    B, H, N, d = 1, 1, 12, 4
    q, k, dout = (_rand(s, B, H, N, d) for s in (48, 49, 50))
    v = np.broadcast_to(_rand(51, d), (B, H, N, d)).copy()
    g = oracle.attention_bwd(q, k, v, dout, 0.5, False)
    np.testing.assert_allclose(g["dq"], 0.0, atol=1e-13)
    np.testing.assert_allclose(g["dk"], 0.0, atol=1e-13)
    # dV columns sum to the column sums of dO (P is row-stochastic)
    np.testing.assert_allclose(g["dv"].sum(axis=2), dout.sum(axis=2), rtol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_backward_restricted_to_rows_and_key_ranges(causal):
    """The row-sampled dQ and the key-range dK/dV (used where the whole problem is too long to
    differentiate on the CPU) against matrix products written with numpy from P, and against the
    whole-tensor backward."""
    B, H, N, d = 2, 2, 23, 8
    q, k, v, dout = (_rand(s, B, H, N, d) for s in (52, 53, 54, 55))
    alpha = 0.4
    g = oracle.attention_bwd(q, k, v, dout, alpha, causal)
    rows = np.array([0, 5, N - 1, N, 2 * N + 7, B * H * N - 1], dtype=np.int64)
    dq_rows = oracle.attention_bwd_dq_rows(q, k, v, dout, rows, alpha, causal)
    np.testing.assert_allclose(dq_rows, g["dq"].reshape(-1, d)[rows], rtol=1e-12, atol=1e-14)
    for b, hh, j0, j1 in ((0, 0, 0, N), (1, 1, 17, N), (0, 1, 9, 14), (1, 0, N - 1, N), (1, 0, 4, 4)):
        dk, dv = oracle.attention_bwd_dkdv_keys(q[b, hh], k[b, hh], v[b, hh], dout[b, hh], j0, j1, alpha, causal)
        P = oracle.attention_probs(q[b, hh], k[b, hh], v[b, hh], alpha, causal)
        dP = dout[b, hh] @ v[b, hh].T
        dS = P * (dP - np.sum(P * dP, axis=1, keepdims=True))
        np.testing.assert_allclose(dk, (alpha * dS.T @ q[b, hh])[j0:j1], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(dv, (P.T @ dout[b, hh])[j0:j1], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(dk, g["dk"][b, hh, j0:j1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(dv, g["dv"][b, hh, j0:j1], rtol=1e-12, atol=1e-14)


# ---- multi-query / grouped-query attention (section 3.1, "Attention variants") -------------------------
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,H_kv", [(4, 4), (4, 2), (6, 2), (3, 1)])
def test_gqa_forward_matches_library_softmax_per_query_head(H, H_kv, causal):
    B, N, d = 2, 9, 4
    q = _rand(11, B, H, N, d)
    k, v = _rand(12, B, H_kv, N, d), _rand(13, B, H_kv, N, d)
    o, lse = oracle.attention_fwd_gqa(q, k, v, 0.41, causal)
    for b in range(B):
        for h in range(H):
            g = h // (H // H_kv)  # written out here independently of the oracle's helper
            o_ref, l_ref = _library_attention(q[b, h], k[b, g], v[b, g], 0.41, causal)
            np.testing.assert_allclose(o[b, h], o_ref, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[b, h], l_ref, rtol=1e-12, atol=1e-13)


def test_gqa_head_mapping_is_blocked_not_interleaved():
    # two key/value heads with constant, distinct value rows: query heads 0,1 must return the first, 2,3 the second
    B, H, H_kv, N, d = 1, 4, 2, 5, 3
    q, k = _rand(14, B, H, N, d), _rand(15, B, H_kv, N, d)
    v = np.empty((B, H_kv, N, d))
    v[:, 0], v[:, 1] = 1.0, -2.0
    o, _ = oracle.attention_fwd_gqa(q, k, v, 1.0, False)
    np.testing.assert_allclose(o[:, :2], 1.0, rtol=1e-14)
    np.testing.assert_allclose(o[:, 2:], -2.0, rtol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_gqa_backward_matches_finite_differences_of_the_forward(causal):
    B, H, H_kv, N, d = 1, 4, 2, 6, 3
    alpha = 0.6
    q, dout = _rand(16, B, H, N, d), _rand(19, B, H, N, d)
    k, v = _rand(17, B, H_kv, N, d), _rand(18, B, H_kv, N, d)
    r = oracle.attention_bwd_gqa(q, k, v, dout, alpha, causal)
    assert r["dk"].shape == k.shape and r["dv"].shape == v.shape and r["dq"].shape == q.shape

    def loss(q_, k_, v_):
        o, _ = oracle.attention_fwd_gqa(q_, k_, v_, alpha, causal)
        return float((o * dout).sum())

    eps = 1e-6
    for name, x, g in (("dq", q, r["dq"]), ("dk", k, r["dk"]), ("dv", v, r["dv"])):
        rng = np.random.default_rng(20)
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"dq": (xp, k, v), "dk": (q, xp, v), "dv": (q, k, xp)}[name]
            args_m = {"dq": (xm, k, v), "dk": (q, xm, v), "dv": (q, k, xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert g[idx] == pytest.approx(fd, rel=2e-6, abs=2e-8), (name, idx)


def test_gqa_with_one_group_per_head_is_ordinary_attention():
    q, k, v, dout = (_rand(s, 2, 3, 7, 4) for s in (21, 22, 23, 24))
    o1, l1 = oracle.attention_fwd(q, k, v, 0.5, True)
    o2, l2 = oracle.attention_fwd_gqa(q, k, v, 0.5, True)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    r1, r2 = oracle.attention_bwd(q, k, v, dout, 0.5, True), oracle.attention_bwd_gqa(q, k, v, dout, 0.5, True)
    for key in ("dq", "dk", "dv"):
        assert np.array_equal(r1[key], r2[key])
