"""Pins for oracle/mdbf_quantizer.py: closed forms and invariants the paper and linear algebra fix.  CPU only."""
import numpy as np
import pytest

from oracle import mdbf_oracle as orc
from oracle import mdbf_quantizer as qz


def _mat(seed, rows, cols, decay=0.7):
    rng = np.random.default_rng(seed)
    r = min(rows, cols)
    return rng.standard_normal((rows, r)) @ np.diag(1.0 / np.arange(1, r + 1) ** decay) @ rng.standard_normal((r, cols))


def _what(L):
    return orc.dense_reconstruct(L["SA"], L["SB"], L["A"], L["Q"], L["G"], L["B"])


# ---- Theorem 1 (Eq. "rankl-error"): the error of the fixed-mask optimum is the tail of the envelope's spectrum
@pytest.mark.parametrize("rows,cols,l", [(30, 20, 1), (30, 20, 3), (17, 40, 5), (12, 12, 12)])
def test_fixed_mask_error_is_the_spectral_tail(rows, cols, l):
    rng = np.random.default_rng(rows + cols + l)
    U = rng.standard_normal((rows, cols))
    S = np.where(rng.random((rows, cols)) < 0.5, -1, 1)          # an arbitrary mask, not sign(U)
    sig = np.linalg.svd(S * U, compute_uv=False)
    err = np.linalg.norm(U - qz.fixed_mask_optimum(U, S, l))
    assert err == pytest.approx(np.sqrt((sig[l:] ** 2).sum()), rel=1e-10, abs=1e-10)
    # and no member of F_l(S) built from another rank-l envelope does better
    E = rng.standard_normal((rows, l)) @ rng.standard_normal((l, cols))
    assert np.linalg.norm(U - S * E) >= err - 1e-12


@pytest.mark.parametrize("l", [1, 2, 4, 9])
def test_msvid_error_and_mask(l):
    Z = _mat(5, 33, 21)
    S, A, Q = qz.msvid(Z, l)
    np.testing.assert_array_equal(S, np.where(Z < 0, -1, 1))
    assert A.shape == (33, l) and Q.shape == (21, l)
    sig = np.linalg.svd(np.abs(Z), compute_uv=False)
    assert np.linalg.norm(Z - qz.msvid_value(Z, l)) == pytest.approx(np.sqrt((sig[l:] ** 2).sum()), rel=1e-10)


def test_msvid_error_falls_with_l_and_vanishes_at_full_rank():
    Z = _mat(6, 25, 18)
    errs = [np.linalg.norm(Z - qz.msvid_value(Z, l)) for l in range(1, 19)]
    assert all(a >= b - 1e-12 for a, b in zip(errs, errs[1:]))
    assert errs[-1] < 1e-10


def test_msvid_l1_is_the_rank_one_envelope():
    # l = 1: sign(Z) o (sigma_1 u_1 v_1^T) of |Z|, u_1 and v_1 entrywise positive (Perron)
    Z = _mat(7, 14, 9)
    S, A, Q = qz.msvid(Z, 1)
    Uf, s, Vt = np.linalg.svd(np.abs(Z))
    np.testing.assert_allclose(A @ Q.T, s[0] * np.outer(Uf[:, 0], Vt[0]), rtol=1e-10, atol=1e-12)
    assert np.all(A @ Q.T > 0)


def test_msvid_fixes_members_of_the_format():
    # Z = S o (A Q^T) with positive A, Q has |Z| of rank l: MSVID_l returns it unchanged
    rng = np.random.default_rng(8)
    A = np.abs(rng.standard_normal((20, 3))) + 0.1
    Q = np.abs(rng.standard_normal((15, 3))) + 0.1
    S = np.where(rng.random((20, 15)) < 0.5, -1, 1)
    Z = S * (A @ Q.T)
    np.testing.assert_allclose(qz.msvid_value(Z, 3), Z, rtol=1e-10, atol=1e-12)
    # l = 1 output is a fixed point for any input (its envelope is positive)
    Y = qz.msvid_value(_mat(9, 16, 11), 1)
    np.testing.assert_allclose(qz.msvid_value(Y, 1), Y, rtol=1e-10, atol=1e-12)


# ---- initialisation (Eq. "mesvid-balanced"): U_0 V_0^T is the rank-R truncation, the factors are balanced
def test_balanced_factors():
    W = _mat(10, 28, 19)
    sig = np.linalg.svd(W, compute_uv=False)
    for R in (1, 5, 19):
        U0, V0 = qz.balanced_factors(W, R)
        assert U0.shape == (28, R) and V0.shape == (19, R)
        assert np.linalg.norm(W - U0 @ V0.T) == pytest.approx(np.sqrt((sig[R:] ** 2).sum()), rel=1e-9, abs=1e-10)
        np.testing.assert_allclose(U0.T @ U0, np.diag(sig[:R]), atol=1e-10)
        np.testing.assert_allclose(V0.T @ V0, np.diag(sig[:R]), atol=1e-10)


# ---- least-squares step (Eq. "admm-U-tilde"): stationarity of ||W - X V^T||^2 + rho ||X - (U - Lam)||^2
def test_least_squares_step_is_the_minimiser():
    rng = np.random.default_rng(11)
    W, V = rng.standard_normal((13, 17)), rng.standard_normal((17, 6))
    U, Lam = rng.standard_normal((13, 6)), rng.standard_normal((13, 6))
    rho = 0.37
    X = qz.least_squares_step(W, V, U, Lam, rho)
    grad = (X @ V.T - W) @ V + rho * (X - (U - Lam))
    assert np.abs(grad).max() < 1e-10
    obj = lambda Y: np.linalg.norm(W - Y @ V.T) ** 2 + rho * np.linalg.norm(Y - (U - Lam)) ** 2
    for _ in range(5):
        assert obj(X + 1e-3 * rng.standard_normal(X.shape)) > obj(X)
    # limits: rho -> infinity pins X to U - Lam; rho -> 0 gives the plain least-squares solution
    np.testing.assert_allclose(qz.least_squares_step(W, V, U, Lam, 1e12), U - Lam, atol=1e-8)
    np.testing.assert_allclose(qz.least_squares_step(W, V, U, Lam, 1e-12),
                               np.linalg.lstsq(V, W.T, rcond=None)[0].T, atol=1e-7)


def test_refinement_bookkeeping():
    # one inner iteration by hand: prox of (U~ + 0), dual = U~ - U
    W = _mat(12, 20, 16)
    U0, V0 = qz.balanced_factors(W, 8)
    fU = qz.msvid(U0, 2)
    V = qz.msvid_value(V0, 2)
    Ut = qz.least_squares_step(W, V, qz.msvid_value(U0, 2), np.zeros((20, 8)), 2.0)
    S, A, Q = qz.refine_factor(W, fU, V, 2, 2.0, 1)
    np.testing.assert_allclose(S * (A @ Q.T), qz.msvid_value(Ut, 2), rtol=1e-12, atol=1e-12)


# ---- the whole pipeline returns a layer of the forward oracle's format
@pytest.mark.parametrize("outer", [0, 2])
def test_quantize_returns_a_consistent_layer(outer):
    W = _mat(13, 40, 28)
    L = qz.quantize(W, R=12, l=3, outer=outer)
    assert L["SA"].shape == (40, 12) and L["SB"].shape == (12, 28)
    assert L["A"].shape == (40, 3) and L["Q"].shape == (12, 3) and L["G"].shape == (12, 3) and L["B"].shape == (28, 3)
    assert set(np.unique(L["SA"])) <= {-1, 1} and set(np.unique(L["SB"])) <= {-1, 1}
    # demodulated envelopes have rank <= l (Definition of F_l(S))
    U = orc.factor_U(L["SA"], L["A"], L["Q"])
    assert np.linalg.matrix_rank(L["SA"] * U, tol=1e-9) <= 3
    x = np.random.default_rng(1).standard_normal((2, 28))
    np.testing.assert_allclose(orc.forward_factored(L["SA"], L["SB"], L["A"], L["Q"], L["G"], L["B"], x),
                               x @ _what(L).T, rtol=1e-10, atol=1e-10)


def test_initialisation_is_msvid_of_the_balanced_factors():
    W = _mat(14, 24, 30)
    L = qz.quantize(W, R=10, l=2, outer=0)
    U0, V0 = qz.balanced_factors(W, 10)
    np.testing.assert_allclose(orc.factor_U(L["SA"], L["A"], L["Q"]), qz.msvid_value(U0, 2), atol=1e-12)
    np.testing.assert_allclose(orc.factor_V(L["SB"], L["G"], L["B"]), qz.msvid_value(V0, 2).T, atol=1e-12)


def test_more_envelope_modes_fit_better_and_refinement_helps():
    # the behaviour the paper reports (error falls with l; refinement improves the initialisation);
    # an observation on seeded matrices, not a theorem
    W = _mat(0, 96, 80)
    e = {l: qz.relative_error(W, _what(qz.quantize(W, R=40, l=l, outer=0))) for l in (1, 2, 4, 8)}
    assert e[1] > e[2] > e[4] > e[8]
    e0 = qz.relative_error(W, _what(qz.quantize(W, R=40, l=4, outer=0)))
    e3 = qz.relative_error(W, _what(qz.quantize(W, R=40, l=4, outer=3)))
    assert e3 < e0


# ---- the refinement loop beyond its first iteration, and the U / V alternation, retyped with bare numpy
def _bare_msvid(Z, l):
    """sign(Z) o TSVD_l(|Z|) (Eq. "msvid-def") with numpy calls only; sign(0) = +1."""
    Uf, s, Vt = np.linalg.svd(np.abs(Z), full_matrices=False)
    return np.where(Z < 0, -1.0, 1.0) * ((Uf[:, :l] * s[:l]) @ Vt[:l, :])


def _bare_refine(W, U, V, l, rho, inner, dual_sign=+1.0, lam_in_prox=True):
    """Eqs. "admm-U-tilde", "admm-U-prox", "admm-U-dual" written out, dual variable starting at zero.
    dual_sign / lam_in_prox plant the two mistakes the pin must catch."""
    R = V.shape[1]
    Lam = np.zeros_like(U)
    for _ in range(inner):
        Ut = (W @ V + rho * (U - Lam)) @ np.linalg.inv(V.T @ V + rho * np.eye(R))
        U = _bare_msvid(Ut + (Lam if lam_in_prox else 0.0), l)
        Lam = Lam + dual_sign * (Ut - U)
    return U


@pytest.mark.parametrize("l,inner", [(1, 2), (2, 2), (2, 3)])
def test_refine_factor_by_hand_beyond_the_first_iteration(l, inner):
    rng = np.random.default_rng(40 + l + inner)
    W = _mat(41, 6, 5)
    R, rho = 3, 0.8
    U_start = _bare_msvid(rng.standard_normal((6, R)), l)      # a member of the format: the loop's own input form
    V = rng.standard_normal((5, R))
    # the oracle takes the factor as (S, A, Q): hand it the same matrix through its own parametrisation
    S0 = np.where(U_start < 0, -1, 1).astype(np.int8)
    Uf, s, Vt = np.linalg.svd(np.abs(U_start), full_matrices=False)
    fU = (S0, Uf[:, :l] * np.sqrt(s[:l]), Vt[:l, :].T * np.sqrt(s[:l]))
    np.testing.assert_allclose(S0 * (fU[1] @ fU[2].T), U_start, atol=1e-12)
    S, A, Q = qz.refine_factor(W, fU, V, l, rho, inner)
    want = _bare_refine(W, U_start, V, l, rho, inner)
    np.testing.assert_allclose(S * (A @ Q.T), want, rtol=1e-9, atol=1e-10)
    # the pin has teeth: a flipped dual update, or a prox without the dual variable, gives another matrix
    for kw in (dict(dual_sign=-1.0), dict(lam_in_prox=False)):
        wrong = _bare_refine(W, U_start, V, l, rho, inner, **kw)
        assert np.abs(wrong - want).max() > 1e-4 * np.abs(want).max(), kw


def test_quantize_one_outer_sweep_by_hand():
    """Initialisation, then U refined against the initial V, then V refined against the new U on the
    transposed problem (Sec. 4.3.2), rho = rho_rel * trace(V^T V) / R of the fixed factor."""
    W = _mat(43, 6, 5)
    R, l, inner, rho_rel = 3, 2, 2, 1.5
    Uf, s, Vt = np.linalg.svd(W, full_matrices=False)
    U = _bare_msvid(Uf[:, :R] * np.sqrt(s[:R]), l)
    V = _bare_msvid(Vt[:R, :].T * np.sqrt(s[:R]), l)
    U = _bare_refine(W, U, V, l, rho_rel * np.trace(V.T @ V) / R, inner)
    V_new = _bare_refine(W.T, V, U, l, rho_rel * np.trace(U.T @ U) / R, inner)
    L = qz.quantize(W, R, l, rho_rel=rho_rel, outer=1, inner=inner)
    np.testing.assert_allclose(orc.factor_U(L["SA"], L["A"], L["Q"]), U, rtol=1e-9, atol=1e-10)
    np.testing.assert_allclose(orc.factor_V(L["SB"], L["G"], L["B"]), V_new.T, rtol=1e-9, atol=1e-10)
    np.testing.assert_allclose(_what(L), U @ V_new.T, rtol=1e-9, atol=1e-10)
    # planted mistake: V refined against the OLD U (no alternation) is a different layer
    U_old = _bare_msvid(Uf[:, :R] * np.sqrt(s[:R]), l)
    V_stale = _bare_refine(W.T, V, U_old, l, rho_rel * np.trace(U_old.T @ U_old) / R, inner)
    assert np.abs(V_stale - V_new).max() > 1e-4 * np.abs(V_new).max()
