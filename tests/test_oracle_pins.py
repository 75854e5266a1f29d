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


def numpy_attention(Q, K, V, dO, scale, causal):
    """Independent evaluation with library matmul / softmax / logsumexp."""
    S = scale * Q @ np.swapaxes(K, -1, -2)
    if causal:
        S = np.where(np.tril(np.ones(S.shape[-2:], dtype=bool)), S, -np.inf)
    P = softmax(S, axis=-1)
    LSE = logsumexp(S, axis=-1)
    O = P @ V
    dV = np.swapaxes(P, -1, -2) @ dO
    dP = dO @ np.swapaxes(V, -1, -2)
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
    "dV from dS instead of P": ("dVj[k] += p * dOh[(size_t)i * d + k];", "dVj[k] += ds * dOh[(size_t)i * d + k];"),
    "dV transposed P": ("const double p = P[(size_t)i * Nk + j];\n        const double ds", "const double p = P[(size_t)j * Nk + i];\n        const double ds"),
    "causal backward starts one row late": ("const int ibeg = causal ? j : 0;", "const int ibeg = causal ? j + 1 : 0;"),
    # mistakes that only a problem with Nq != Nk can show
    "dK/dV sum over Nk queries": ("for (int i = ibeg; i < Nq; ++i) {", "for (int i = ibeg; i < (Nq < Nk ? Nq : Nk); ++i) {"),
    "softmax over the first Nq keys": ("const int jend = causal ? i + 1 : Nk;\n    double m = -INFINITY;",
                                       "const int jend = causal ? i + 1 : (Nq < Nk ? Nq : Nk);\n    double m = -INFINITY;"),
    "dQ sums over the first Nq keys": ("const int jend = causal ? i + 1 : Nk;\n      for (int j = 0; j < jend; ++j) {\n        double dp",
                                       "const int jend = causal ? i + 1 : (Nq < Nk ? Nq : Nk);\n      for (int j = 0; j < jend; ++j) {\n        double dp"),
    "K and V of head h taken at the Q offset": ("*Kh = K + offk, *Vh = V + offk,", "*Kh = K + (Nq < Nk ? offq : offk), *Vh = V + (Nq < Nk ? offq : offk),"),
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
