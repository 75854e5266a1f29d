"""Pins for the fp64 CPU oracle (no GPU).

Each check ties the oracle to something other than itself: closed forms, invariants of
softmax attention, finite differences, a hand-derived rational example and an independent
numpy/scipy evaluation of the same definitions (paper Eq. 1, Sec. 3.2.1 Eq. 2-3, Sec. 3.3
Eq. 4).  Every check takes the oracle as an argument, so that the last test can run the same
checks against deliberately broken copies of the oracle and show that each planted mistake is
caught.
"""
import math
import os
import re

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def rng():
    return np.random.default_rng(20250212)


def numpy_attention(Q, K, V, dO, scale, causal, keep=None, keep_scale=1.0):
    """Independent evaluation with library matmul / softmax / logsumexp.  With a keep mask,
    the dropped and rescaled probabilities Pd = keep_scale * keep * P replace P in O = Pd V,
    and the chain rule through Pd gives dP = keep_scale * keep * (dO V^T)."""
    S = scale * Q @ np.swapaxes(K, -1, -2)
    if causal:
        S = np.where(np.tril(np.ones(S.shape[-2:], dtype=bool)), S, -np.inf)
    P = softmax(S, axis=-1)
    LSE = logsumexp(S, axis=-1)
    G = np.ones_like(P) if keep is None else keep_scale * keep.astype(np.float64)
    O = (G * P) @ V
    dV = np.swapaxes(G * P, -1, -2) @ dO
    dP = G * (dO @ np.swapaxes(V, -1, -2))
    dS = P * (dP - (P * dP).sum(-1, keepdims=True))
    dQ = scale * dS @ K
    dK = scale * np.swapaxes(dS, -1, -2) @ Q
    return dict(P=P, LSE=LSE, O=O, dQ=dQ, dK=dK, dV=dV)


# ----------------------------------------------------------------------------------------
# checks (orc = an oracle.OracleLib or the oracle module itself)
# ----------------------------------------------------------------------------------------
def check_rows_of_P_sum_to_one(orc):
    r = rng()
    for causal in (False, True):
        Q, K, V = r.standard_normal((2, 3, 37, 8)) * 2, r.standard_normal((2, 3, 37, 8)) * 2, r.standard_normal((2, 3, 37, 8))
        O, LSE, P = orc.mha_fwd(Q, K, V, 0.3, causal, return_P=True)
        assert np.abs(P.sum(-1) - 1).max() <= 1e-12
        assert (P >= 0).all()
        if causal:
            assert np.all(np.triu(P, 1) == 0)


def check_zero_Q_gives_uniform_attention(orc):
    r = rng()
    N, d = 29, 5
    K, V = r.standard_normal((1, 2, N, d)), r.standard_normal((1, 2, N, d))
    Q = np.zeros_like(K)
    O, LSE = orc.mha_fwd(Q, K, V, 0.7, False)
    np.testing.assert_allclose(O, np.broadcast_to(V.mean(2, keepdims=True), V.shape), atol=1e-13)
    np.testing.assert_allclose(LSE, math.log(N), atol=1e-13)
    O, LSE = orc.mha_fwd(Q, K, V, 0.7, True)
    prefix_mean = np.cumsum(V, axis=2) / np.arange(1, N + 1)[None, None, :, None]
    np.testing.assert_allclose(O, prefix_mean, atol=1e-13)
    np.testing.assert_allclose(LSE, np.broadcast_to(np.log(np.arange(1, N + 1)), LSE.shape), atol=1e-13)


def check_causal_row0_sees_only_key0(orc):
    r = rng()
    Q, K, V = (r.standard_normal((2, 2, 16, 4)) for _ in range(3))
    scale = 0.5
    O, LSE = orc.mha_fwd(Q, K, V, scale, True)
    np.testing.assert_allclose(O[:, :, 0], V[:, :, 0], atol=1e-14)
    np.testing.assert_allclose(LSE[:, :, 0], scale * (Q[:, :, 0] * K[:, :, 0]).sum(-1), atol=1e-13)


def check_constant_V_rows(orc):
    r = rng()
    N, d = 21, 6
    for causal in (False, True):
        Q, K, dO = (r.standard_normal((1, 2, N, d)) for _ in range(3))
        V = np.broadcast_to(r.standard_normal(d), (1, 2, N, d)).copy()
        g = orc.mha_bwd(Q, K, V, dO, 0.4, causal)
        np.testing.assert_allclose(g["O"], V, atol=1e-13)
        assert np.abs(g["dQ"]).max() <= 1e-12
        assert np.abs(g["dK"]).max() <= 1e-12


def check_backward_sum_invariants(orc):
    r = rng()
    for causal in (False, True):
        Q, K, V, dO = (r.standard_normal((2, 2, 33, 8)) for _ in range(4))
        g = orc.mha_bwd(Q, K, V, dO, 0.35, causal)
        # rows of dS sum to zero => columns of dK sum to zero over keys
        assert np.abs(g["dK"].sum(2)).max() <= 1e-11
        # rows of P sum to one => sum_j dV_j = sum_i dO_i
        np.testing.assert_allclose(g["dV"].sum(2), dO.sum(2), atol=1e-11)
        # D = rowsum(dO * O)
        np.testing.assert_allclose(g["D"], (dO * g["O"]).sum(-1), atol=1e-13)


def check_key_shift_invariance(orc):
    r = rng()
    N, d, scale = 24, 8, 0.3
    for causal in (False, True):
        Q, K, V, dO = (r.standard_normal((1, 3, N, d)) for _ in range(4))
        c = r.standard_normal(d) * 3
        g0 = orc.mha_bwd(Q, K, V, dO, scale, causal)
        g1 = orc.mha_bwd(Q, K + c, V, dO, scale, causal)
        for name in ("O", "dQ", "dK", "dV"):
            np.testing.assert_allclose(g1[name], g0[name], atol=1e-10, err_msg=name)
        np.testing.assert_allclose(g1["LSE"] - g0["LSE"], scale * Q @ c, atol=1e-11)


def check_key_permutation_noncausal(orc):
    r = rng()
    N, d = 19, 4
    Q, K, V, dO = (r.standard_normal((1, 2, N, d)) for _ in range(4))
    perm = r.permutation(N)
    g0 = orc.mha_bwd(Q, K, V, dO, 0.5, False)
    g1 = orc.mha_bwd(Q, K[:, :, perm], V[:, :, perm], dO, 0.5, False)
    np.testing.assert_allclose(g1["O"], g0["O"], atol=1e-12)
    np.testing.assert_allclose(g1["dQ"], g0["dQ"], atol=1e-12)
    np.testing.assert_allclose(g1["dK"], g0["dK"][:, :, perm], atol=1e-12)
    np.testing.assert_allclose(g1["dV"], g0["dV"][:, :, perm], atol=1e-12)


def check_finite_difference_gradients(orc):
    """dQ, dK, dV are the gradient of L = sum(O * dO) (central differences)."""
    r = rng()
    N, d, scale, h = 7, 3, 0.6, 1e-5
    for causal in (False, True):
        Q, K, V, dO = (r.standard_normal((1, 2, N, d)) for _ in range(4))
        g = orc.mha_bwd(Q, K, V, dO, scale, causal)

        def loss(q, k, v):
            return float((orc.mha_fwd(q, k, v, scale, causal)[0] * dO).sum())

        for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
            num = np.zeros_like(Q)
            base = [Q, K, V]
            it = np.nditer(base[idx], flags=["multi_index"])
            for _ in it:
                mi = it.multi_index
                args_p = [a.copy() for a in base]
                args_m = [a.copy() for a in base]
                args_p[idx][mi] += h
                args_m[idx][mi] -= h
                num[mi] = (loss(*args_p) - loss(*args_m)) / (2 * h)
            err = np.abs(num - g[name]).max() / max(np.abs(g[name]).max(), 1e-30)
            assert err <= 1e-6, (name, err)


def check_against_numpy_scipy(orc):
    r = rng()
    for shape in ((1, 1, 1, 1), (2, 3, 50, 16), (1, 2, 130, 64)):
        for causal in (False, True):
            Q, K, V, dO = (r.standard_normal(shape) for _ in range(4))
            Q *= 1.7
            scale = 1.0 / math.sqrt(shape[-1])
            ref = numpy_attention(Q, K, V, dO, scale, causal)
            O, LSE, P = orc.mha_fwd(Q, K, V, scale, causal, return_P=True)
            g = orc.mha_bwd(Q, K, V, dO, scale, causal)
            np.testing.assert_allclose(P, ref["P"], rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(O, ref["O"], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(LSE, ref["LSE"], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(g["O"], O, rtol=0, atol=0)
            np.testing.assert_allclose(g["LSE"], LSE, rtol=0, atol=0)
            for name in ("dQ", "dK", "dV"):
                denom = np.linalg.norm(ref[name])
                assert np.linalg.norm(g[name] - ref[name]) <= 1e-12 * max(denom, 1e-30), name


def _parse_golden(path):
    ln3, ln4 = math.log(3.0), math.log(4.0)
    vals = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *toks = line.split()
            out = []
            for t in toks:
                t = t.replace("ln3", repr(ln3)).replace("ln4", repr(ln4))
                prod = 1.0
                for fct in t.split("*"):
                    prod *= float(fct)
                out.append(prod)
            vals[name] = np.array(out)
    return vals


def check_hand_derived_rational_example(orc):
    g = _parse_golden(os.path.join(HERE, "golden", "two_key_rational.txt"))
    scale = float(g["scale"][0])
    sh = (1, 1, 2, 1)
    Q, K, V, dO = (g[n].reshape(sh) for n in ("Q", "K", "V", "dO"))
    O, LSE, P = orc.mha_fwd(Q, K, V, scale, False, return_P=True)
    b = orc.mha_bwd(Q, K, V, dO, scale, False)
    np.testing.assert_allclose(P.ravel(), g["P"], atol=1e-15)
    np.testing.assert_allclose(O.ravel(), g["O"], atol=1e-14)
    np.testing.assert_allclose(LSE.ravel(), g["LSE"], atol=1e-14)
    for n in ("dQ", "dK", "dV"):
        np.testing.assert_allclose(b[n].ravel(), g[n], atol=1e-14, err_msg=n)


def check_blockwise_merge_rule_equals_direct_softmax(orc):
    """Eq. 3's merge of two blocks (with l = sum of f) reproduces the oracle's O, LSE."""
    r = rng()
    N, d, scale = 48, 8, 0.5
    Q, K, V = r.standard_normal((1, 1, N, d)) * 2, r.standard_normal((1, 1, N, d)) * 2, r.standard_normal((1, 1, N, d))
    O, LSE = orc.mha_fwd(Q, K, V, scale, False)
    S = scale * Q[0, 0] @ K[0, 0].T
    m = np.full(N, -np.inf)
    l = np.zeros(N)
    acc = np.zeros((N, d))
    for j0 in range(0, N, 16):
        Sb = S[:, j0:j0 + 16]
        m_new = np.maximum(m, Sb.max(1))
        f = np.exp(Sb - m_new[:, None])
        alpha = np.exp(m - m_new)
        l = alpha * l + f.sum(1)
        acc = alpha[:, None] * acc + f @ V[0, 0, j0:j0 + 16]
        m = m_new
    np.testing.assert_allclose(acc / l[:, None], O[0, 0], atol=1e-13)
    np.testing.assert_allclose(m + np.log(l), LSE[0, 0], atol=1e-13)


def check_large_logits_do_not_overflow(orc):
    """Logits of magnitude ~1e3: exp(S) overflows fp64 unless the row max is subtracted."""
    r = rng()
    N, d = 16, 4
    Q, K, V = r.standard_normal((1, 1, N, d)) * 30, r.standard_normal((1, 1, N, d)) * 30, r.standard_normal((1, 1, N, d))
    O, LSE, P = orc.mha_fwd(Q, K, V, 1.0, False, return_P=True)
    assert np.isfinite(O).all() and np.isfinite(LSE).all()
    assert np.abs(P.sum(-1) - 1).max() <= 1e-12
    S = Q[0, 0] @ K[0, 0].T
    np.testing.assert_allclose(LSE[0, 0], logsumexp(S, axis=-1), rtol=1e-13)


RECT_SHAPES = ((5, 9), (9, 5), (1, 7), (7, 1), (40, 13))  # (Nq, Nk), non-causal only


def check_rect_against_numpy_scipy(orc):
    """Nq != Nk (cross-attention, Sec. 2.1): the same library evaluation, several heads."""
    r = rng()
    for Nq, Nk in RECT_SHAPES:
        B, H, d, scale = 2, 3, 6, 0.45
        Q, dO = r.standard_normal((B, H, Nq, d)) * 1.5, r.standard_normal((B, H, Nq, d))
        K, V = r.standard_normal((B, H, Nk, d)) * 1.5, r.standard_normal((B, H, Nk, d))
        ref = numpy_attention(Q, K, V, dO, scale, False)
        O, LSE, P = orc.mha_fwd(Q, K, V, scale, False, return_P=True)
        g = orc.mha_bwd(Q, K, V, dO, scale, False)
        assert P.shape == (B, H, Nq, Nk) and g["dK"].shape == K.shape and g["dQ"].shape == Q.shape
        np.testing.assert_allclose(P, ref["P"], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(O, ref["O"], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(LSE, ref["LSE"], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(g["O"], O, rtol=0, atol=0)
        np.testing.assert_allclose(g["D"], (dO * O).sum(-1), atol=1e-13)
        for name in ("dQ", "dK", "dV"):
            np.testing.assert_allclose(g[name], ref[name], rtol=1e-11, atol=1e-13, err_msg=name)


def check_rect_single_key_closed_form(orc):
    """Nk = 1: P = 1, so O_i = V_0, LSE_i = scale q_i.k_0, dV_0 = sum_i dO_i, dQ = dK = 0."""
    r = rng()
    Nq, d, scale = 11, 4, 0.8
    Q, dO = r.standard_normal((1, 2, Nq, d)), r.standard_normal((1, 2, Nq, d))
    K, V = r.standard_normal((1, 2, 1, d)), r.standard_normal((1, 2, 1, d))
    g = orc.mha_bwd(Q, K, V, dO, scale, False)
    np.testing.assert_allclose(g["O"], np.broadcast_to(V, Q.shape), atol=1e-14)
    np.testing.assert_allclose(g["LSE"], scale * (Q * K).sum(-1), atol=1e-13)
    np.testing.assert_allclose(g["dV"], dO.sum(2, keepdims=True), atol=1e-13)
    assert np.abs(g["dQ"]).max() <= 1e-13 and np.abs(g["dK"]).max() <= 1e-13


def check_rect_duplicated_keys(orc):
    """Every key/value listed twice: O and dQ unchanged, LSE grows by ln 2, each copy gets
    half of dK and dV.  Relates Nk keys to 2 Nk keys, so a wrong stride or bound shows."""
    r = rng()
    Nq, Nk, d, scale = 10, 5, 4, 0.6
    Q, dO = r.standard_normal((1, 2, Nq, d)), r.standard_normal((1, 2, Nq, d))
    K, V = r.standard_normal((1, 2, Nk, d)), r.standard_normal((1, 2, Nk, d))
    g1 = orc.mha_bwd(Q, K, V, dO, scale, False)
    g2 = orc.mha_bwd(Q, np.concatenate([K, K], 2), np.concatenate([V, V], 2), dO, scale, False)
    np.testing.assert_allclose(g2["O"], g1["O"], atol=1e-13)
    np.testing.assert_allclose(g2["LSE"], g1["LSE"] + math.log(2.0), atol=1e-13)
    np.testing.assert_allclose(g2["dQ"], g1["dQ"], atol=1e-13)
    for n in ("dK", "dV"):
        np.testing.assert_allclose(g2[n][:, :, :Nk], 0.5 * g1[n], atol=1e-13, err_msg=n)
        np.testing.assert_allclose(g2[n][:, :, Nk:], 0.5 * g1[n], atol=1e-13, err_msg=n)


def check_rect_queries_are_independent(orc):
    """Each query row is its own softmax: O, LSE, dQ of a subset of the queries equal the
    rows of the full problem, and dK, dV add over a partition of the queries."""
    r = rng()
    Nq, Nk, d, scale = 12, 7, 5, 0.5
    Q, dO = r.standard_normal((1, 2, Nq, d)), r.standard_normal((1, 2, Nq, d))
    K, V = r.standard_normal((1, 2, Nk, d)), r.standard_normal((1, 2, Nk, d))
    full = orc.mha_bwd(Q, K, V, dO, scale, False)
    a = orc.mha_bwd(Q[:, :, :4], K, V, dO[:, :, :4], scale, False)
    b = orc.mha_bwd(Q[:, :, 4:], K, V, dO[:, :, 4:], scale, False)
    for n in ("O", "LSE", "dQ"):
        np.testing.assert_allclose(np.concatenate([a[n], b[n]], 2), full[n], atol=1e-13, err_msg=n)
    for n in ("dK", "dV"):
        np.testing.assert_allclose(a[n] + b[n], full[n], atol=1e-13, err_msg=n)


def check_rect_causal_is_rejected(orc):
    Q, K = np.zeros((1, 1, 3, 2)), np.zeros((1, 1, 4, 2))
    with pytest.raises(RuntimeError):
        orc.mha_fwd(Q, K, K, 1.0, True)
    with pytest.raises(RuntimeError):
        orc.mha_bwd(Q, K, K, Q, 1.0, True)


def check_rect_finite_difference_gradients(orc):
    """dQ, dK, dV of the Nq != Nk case are the gradient of L = sum(O * dO)."""
    r = rng()
    scale, h = 0.6, 1e-5
    for Nq, Nk in ((3, 6), (6, 3)):
        Q, dO = r.standard_normal((1, 1, Nq, 3)), r.standard_normal((1, 1, Nq, 3))
        K, V = r.standard_normal((1, 1, Nk, 3)), r.standard_normal((1, 1, Nk, 3))
        g = orc.mha_bwd(Q, K, V, dO, scale, False)
        base = [Q, K, V]
        for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
            num = np.zeros_like(base[idx])
            for mi in np.ndindex(base[idx].shape):
                ap, am = [a.copy() for a in base], [a.copy() for a in base]
                ap[idx][mi] += h
                am[idx][mi] -= h
                lp = float((orc.mha_fwd(*ap, scale, False)[0] * dO).sum())
                lm = float((orc.mha_fwd(*am, scale, False)[0] * dO).sum())
                num[mi] = (lp - lm) / (2 * h)
            err = np.abs(num - g[name]).max() / max(np.abs(g[name]).max(), 1e-30)
            assert err <= 1e-6, (name, err)


def check_philox_known_answers(orc):
    """The generator behind the dropout mask reproduces its published known-answer vectors."""
    n = 0
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            assert orc.philox4x32_10(w[0:4], w[4:6]) == w[6:10], line
            n += 1
    assert n == 3


def check_dropout_mask_properties(orc):
    """Drop rate threshold/256, dependence on seed/offset/head, independence of the problem
    size (an entry's decision depends on its position only), and the stated byte layout."""
    B, H, Nq, Nk = 2, 3, 70, 90
    seed, offset = 0x123456789ABCDEF, 7
    assert orc.dropout_mask(B, H, Nq, Nk, seed, offset, 0).all()            # threshold 0 keeps all
    for thr in (26, 128, 230):
        M = orc.dropout_mask(B, H, Nq, Nk, seed, offset, thr)
        assert set(np.unique(M)) <= {0, 1}
        n, p = M.size, thr / 256.0
        assert abs((M == 0).mean() - p) <= 5 * math.sqrt(p * (1 - p) / n), thr
        # rows and columns carry the same rate (no stuck byte lane)
        for ax in (2, 3):
            for r in range(4):
                sl = M[:, :, r::4] if ax == 2 else M[:, :, :, r::4]
                assert abs((sl == 0).mean() - p) <= 6 * math.sqrt(p * (1 - p) / sl.size), (thr, ax, r)
    M = orc.dropout_mask(B, H, Nq, Nk, seed, offset, 128)
    assert (M[0, 0] != M[0, 1]).mean() > 0.4 and (M[0, 0] != M[1, 0]).mean() > 0.4   # heads differ
    assert (orc.dropout_mask(B, H, Nq, Nk, seed + 1, offset, 128) != M).mean() > 0.4
    assert (orc.dropout_mask(B, H, Nq, Nk, seed + (1 << 32), offset, 128) != M).mean() > 0.4
    assert (orc.dropout_mask(B, H, Nq, Nk, seed, offset + 1, 128) != M).mean() > 0.4
    # monotone in the threshold: whatever is kept at a high drop rate is kept at a lower one
    assert (orc.dropout_mask(B, H, Nq, Nk, seed, offset, 26) >= M).all()
    # position only: a smaller problem sees the top-left corner of the larger one's mask,
    # and heads are numbered b*H + h
    small = orc.dropout_mask(1, 2, 33, 41, seed, offset, 128)
    np.testing.assert_array_equal(small, M[:1, :2, :33, :41])
    # the stated layout, evaluated entry by entry from the generator's words
    for (h, i, j) in ((0, 0, 0), (0, 1, 2), (1, 5, 6), (4, 69, 89), (5, 34, 3), (3, 7, 88)):
        x = orc.philox4x32_10([j // 4, i // 4, h, offset], [seed & 0xFFFFFFFF, seed >> 32])
        u = (x[i % 4] >> (8 * (j % 4))) & 0xFF
        assert M.reshape(B * H, Nq, Nk)[h, i, j] == (1 if u >= 128 else 0), (h, i, j)


def check_dropout_against_numpy_scipy(orc):
    r = rng()
    for (Nq, Nk, causal) in ((33, 33, False), (33, 33, True), (20, 45, False)):
        B, H, d, scale, thr = 1, 3, 8, 0.4, 77
        keep = orc.dropout_mask(B, H, Nq, Nk, 99, 3, thr)
        ks = 256.0 / (256 - thr)
        Q, dO = r.standard_normal((B, H, Nq, d)) * 1.5, r.standard_normal((B, H, Nq, d))
        K, V = r.standard_normal((B, H, Nk, d)) * 1.5, r.standard_normal((B, H, Nk, d))
        ref = numpy_attention(Q, K, V, dO, scale, causal, keep, ks)
        O, LSE, P = orc.mha_fwd(Q, K, V, scale, causal, return_P=True, keep=keep, keep_scale=ks)
        g = orc.mha_bwd(Q, K, V, dO, scale, causal, keep=keep, keep_scale=ks)
        np.testing.assert_allclose(P, ref["P"], rtol=1e-12, atol=1e-15)      # P itself: before dropout
        np.testing.assert_allclose(LSE, ref["LSE"], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(O, ref["O"], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(g["O"], O, rtol=0, atol=0)
        for name in ("dQ", "dK", "dV"):
            np.testing.assert_allclose(g[name], ref[name], rtol=1e-11, atol=1e-13, err_msg=name)


def check_dropout_degenerate_masks(orc):
    """Keep everything with scale 1: no dropout.  Drop everything: O = 0 and all gradients 0."""
    r = rng()
    Q, K, V, dO = (r.standard_normal((1, 2, 17, 4)) for _ in range(4))
    ones, zeros = np.ones((1, 2, 17, 17), np.uint8), np.zeros((1, 2, 17, 17), np.uint8)
    for causal in (False, True):
        a = orc.mha_bwd(Q, K, V, dO, 0.5, causal)
        b = orc.mha_bwd(Q, K, V, dO, 0.5, causal, keep=ones, keep_scale=1.0)
        for n in ("O", "LSE", "dQ", "dK", "dV"):
            np.testing.assert_array_equal(a[n], b[n])
        z = orc.mha_bwd(Q, K, V, dO, 0.5, causal, keep=zeros, keep_scale=2.0)
        np.testing.assert_array_equal(z["LSE"], a["LSE"])
        for n in ("O", "dQ", "dK", "dV"):
            assert np.abs(z[n]).max() == 0.0, n


def check_dropout_finite_difference_gradients(orc):
    """With the mask held fixed, dQ, dK, dV are the gradient of L = sum(O * dO)."""
    r = rng()
    N, d, scale, h, thr = 6, 3, 0.6, 1e-5, 100
    ks = 256.0 / (256 - thr)
    for causal in (False, True):
        keep = orc.dropout_mask(1, 1, N, N, 5, 0, thr)
        assert 0 < keep.sum() < keep.size
        Q, K, V, dO = (r.standard_normal((1, 1, N, d)) for _ in range(4))
        g = orc.mha_bwd(Q, K, V, dO, scale, causal, keep=keep, keep_scale=ks)
        base = [Q, K, V]
        for name, idx in (("dQ", 0), ("dK", 1), ("dV", 2)):
            num = np.zeros_like(Q)
            for mi in np.ndindex(Q.shape):
                ap, am = [a.copy() for a in base], [a.copy() for a in base]
                ap[idx][mi] += h
                am[idx][mi] -= h
                lp = float((orc.mha_fwd(*ap, scale, causal, keep=keep, keep_scale=ks)[0] * dO).sum())
                lm = float((orc.mha_fwd(*am, scale, causal, keep=keep, keep_scale=ks)[0] * dO).sum())
                num[mi] = (lp - lm) / (2 * h)
            err = np.abs(num - g[name]).max() / max(np.abs(g[name]).max(), 1e-30)
            assert err <= 1e-6, (name, err)


def check_dropout_is_unbiased(orc):
    """Averaged over many masks, the dropped and rescaled O tends to the O without dropout
    (survivors scaled by 256 / (256 - threshold))."""
    r = rng()
    N, d, thr, reps = 24, 4, 64, 600
    Q, K, V = (r.standard_normal((1, 1, N, d)) for _ in range(3))
    O0 = orc.mha_fwd(Q, K, V, 0.5, False)[0]
    keep = orc.dropout_mask(1, reps, N, N, 2024, 0, thr)             # one mask per "head"
    Qr, Kr, Vr = (np.broadcast_to(a, (1, reps, N, d)).copy() for a in (Q, K, V))
    O = orc.mha_fwd(Qr, Kr, Vr, 0.5, False, keep=keep, keep_scale=256.0 / (256 - thr))[0]
    # per-entry std of the estimate is at most sqrt(p/(1-p)) * max|V| * sqrt(sum P^2) / sqrt(reps)
    tol = 5 * math.sqrt((thr / 256) / (1 - thr / 256)) * np.abs(V).max() / math.sqrt(reps)
    assert np.abs(O.mean(1) - O0[:, 0]).max() <= tol
    assert np.abs(O.mean(1) - O0[:, 0]).mean() <= 0.05 * np.abs(O0).mean() + 0.02


CHECKS = [
    check_rows_of_P_sum_to_one,
    check_zero_Q_gives_uniform_attention,
    check_causal_row0_sees_only_key0,
    check_constant_V_rows,
    check_backward_sum_invariants,
    check_key_shift_invariance,
    check_key_permutation_noncausal,
    check_finite_difference_gradients,
    check_against_numpy_scipy,
    check_hand_derived_rational_example,
    check_blockwise_merge_rule_equals_direct_softmax,
    check_large_logits_do_not_overflow,
    check_rect_single_key_closed_form,
    check_rect_duplicated_keys,
    check_rect_queries_are_independent,
    check_rect_finite_difference_gradients,
    check_rect_against_numpy_scipy,
    check_rect_causal_is_rejected,
    check_philox_known_answers,
    check_dropout_degenerate_masks,
    check_dropout_finite_difference_gradients,
    check_dropout_against_numpy_scipy,
    check_dropout_is_unbiased,
    check_dropout_mask_properties,
]


@pytest.mark.parametrize("check", CHECKS, ids=lambda c: c.__name__)
def test_pin(check):
    check(oracle.default())


# ----------------------------------------------------------------------------------------
# Planted mistakes: each edit of the C source is one plausible bug (a dropped term, a wrong
# sign or index, a swapped operand).  The broken oracle is built on the CPU and at least one
# pin must reject it; the pins that need no library routine are listed first on purpose.
# ----------------------------------------------------------------------------------------
MISTAKES = {
    "scale dropped from the logits": ("      s *= scale;\n", ""),
    "causal mask excludes the diagonal": ("const int jend = causal ? i + 1 : Nk;\n    double m = -INFINITY;",
                                          "const int jend = causal ? (i > 0 ? i : 1) : Nk;\n    double m = -INFINITY;"),
    "row max not subtracted": ("Pi[j] = exp(Pi[j] - m);", "Pi[j] = exp(Pi[j]);"),
    "P not normalised": ("for (int j = 0; j < jend; ++j) Pi[j] /= l;", ""),
    "LSE is the row max": ("LSE[i] = m + log(l);", "LSE[i] = m;"),
    "O uses K instead of V": ("Oi[k] += p * V[(size_t)j * d + k];", "Oi[k] += p * V[(size_t)i * d + k];"),
    "D from dO*dO": ("Di += dOh[(size_t)i * d + k] * O[(size_t)i * d + k];", "Di += dOh[(size_t)i * d + k] * dOh[(size_t)i * d + k];"),
    "dS sign": ("P[(size_t)i * Nk + j] * (dp - Di);", "P[(size_t)i * Nk + j] * (dp + Di);"),
    "dS without P": ("dS[(size_t)i * Nk + j] = P[(size_t)i * Nk + j] * (dp - Di);", "dS[(size_t)i * Nk + j] = (dp - Di);"),
    "dP uses K instead of V": ("dp += dOh[(size_t)i * d + k] * Vh[(size_t)j * d + k];", "dp += dOh[(size_t)i * d + k] * Kh[(size_t)j * d + k];"),
    "dQ without scale": ("for (int k = 0; k < d; ++k) dQi[k] *= scale;", ""),
    "dQ contracts with Q": ("dQi[k] += ds * Kh[(size_t)j * d + k];", "dQi[k] += ds * Qh[(size_t)j * d + k];"),
    "dK without scale": ("for (int k = 0; k < d; ++k) dKj[k] *= scale;", ""),
    "dK from P instead of dS": ("dKj[k] += ds * Qh[(size_t)i * d + k];", "dKj[k] += p * Qh[(size_t)i * d + k];"),
    "dK with the wrong Q row": ("dKj[k] += ds * Qh[(size_t)i * d + k];", "dKj[k] += ds * Qh[(size_t)j * d + k];"),
    "dV from dS instead of P": ("dVj[k] += pm * dOh[(size_t)i * d + k];", "dVj[k] += ds * dOh[(size_t)i * d + k];"),
    "dV transposed P": ("const double p = P[(size_t)i * Nk + j];\n        const double pm", "const double p = P[(size_t)j * Nk + i];\n        const double pm"),
    "causal backward starts one row late": ("const int ibeg = causal ? j : 0;", "const int ibeg = causal ? j + 1 : 0;"),
    # mistakes that only a problem with Nq != Nk can show
    "dK/dV sum over Nk queries": ("for (int i = ibeg; i < Nq; ++i) {", "for (int i = ibeg; i < (Nq < Nk ? Nq : Nk); ++i) {"),
    "softmax over the first Nq keys": ("const int jend = causal ? i + 1 : Nk;\n    double m = -INFINITY;",
                                       "const int jend = causal ? i + 1 : (Nq < Nk ? Nq : Nk);\n    double m = -INFINITY;"),
    "dQ sums over the first Nq keys": ("const int jend = causal ? i + 1 : Nk;\n      for (int j = 0; j < jend; ++j) {\n        double dp",
                                       "const int jend = causal ? i + 1 : (Nq < Nk ? Nq : Nk);\n      for (int j = 0; j < jend; ++j) {\n        double dp"),
    "K and V of head h taken at the Q offset": ("*Kh = K + offk, *Vh = V + offk,", "*Kh = K + (Nq < Nk ? offq : offk), *Vh = V + (Nq < Nk ? offq : offk),"),
    # mistakes in the dropout path and in the generator that draws the mask
    "dropout: survivors not rescaled in O": ("p = keep[(size_t)i * Nk + j] ? r * p : 0.0;", "p = keep[(size_t)i * Nk + j] ? p : 0.0;"),
    "dropout: dP not masked": ("        if (keeph) dp = keeph[(size_t)i * Nk + j] ? keep_scale * dp : 0.0;\n", ""),
    "dropout: dP masked but not rescaled": ("dp = keeph[(size_t)i * Nk + j] ? keep_scale * dp : 0.0;", "dp = keeph[(size_t)i * Nk + j] ? dp : 0.0;"),
    "dropout: dV from the undropped P": ("dVj[k] += pm * dOh[(size_t)i * d + k];", "dVj[k] += p * dOh[(size_t)i * d + k];"),
    "dropout: dS from the dropped P": ("dS[(size_t)i * Nk + j] = P[(size_t)i * Nk + j] * (dp - Di);",
                                       "dS[(size_t)i * Nk + j] = (keeph && !keeph[(size_t)i * Nk + j] ? 0.0 : P[(size_t)i * Nk + j]) * (dp - Di);"),
    "philox: key not advanced": ("    k0 += 0x9E3779B9u;\n", ""),
    "philox: multipliers swapped": ("const uint64_t p0 = (uint64_t)0xD2511F53u * c0;\n    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;",
                                    "const uint64_t p0 = (uint64_t)0xCD9E8D57u * c0;\n    const uint64_t p1 = (uint64_t)0xD2511F53u * c2;"),
    "philox: nine rounds": ("round < 10;", "round < 9;"),
    "philox: output words in the wrong order": ("const uint32_t n1 = (uint32_t)p1;\n    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;\n    const uint32_t n3 = (uint32_t)p0;",
                                                "const uint32_t n3 = (uint32_t)p1;\n    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;\n    const uint32_t n1 = (uint32_t)p0;"),
    "mask: keep below the threshold": ("u >= (unsigned)threshold ? 1 : 0;", "u < (unsigned)threshold ? 1 : 0;"),
    "mask: word and byte index exchanged": ("(x[i % 4] >> (8 * (j % 4)))", "(x[j % 4] >> (8 * (i % 4)))"),
    "mask: head not in the counter": ("(uint32_t)(i / 4), (uint32_t)h, offset}", "(uint32_t)(i / 4), 0u, offset}"),
    "LSE_out rows strided by Nk": ("LSE_out[(size_t)h * Nq + i] = LSE[i];", "LSE_out[(size_t)h * (Nq < Nk ? Nq : Nk) + i] = LSE[i];"),
}


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MISTAKES[name]
    src = open(os.path.join(os.path.dirname(HERE), "oracle", "mha_oracle.c")).read()
    assert src.count(old) == 1, "the edit must apply exactly once: " + name
    broken_c = tmp_path / "broken.c"
    broken_c.write_text(src.replace(old, new))
    lib = oracle.compile_source(str(broken_c), str(tmp_path / "libbroken.so"))
    broken = oracle.OracleLib(lib)
    caught = []
    for check in CHECKS:
        try:
            with np.errstate(all="ignore"):
                check(broken)
        except Exception:  # noqa: BLE001 - any failure of a pin counts
            caught.append(check.__name__)
            break
    assert caught, "no pin noticed the planted mistake: " + name
