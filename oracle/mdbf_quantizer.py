"""CPU oracle for the MDBF layer-wise quantizer: MSVID_l, the balanced-SVD initialisation and the
ADMM-style refinement (paper Sec. 4.2 "Multi-Envelope Structure" and Sec. 4.3 "Layer-Wise Optimization").

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite may import it.  It shares no code
with the HIP library and never calls it.  Plain numpy in float64; `numpy.linalg.svd` and
`numpy.linalg.solve` serve as steps where the paper names a truncated SVD or an inverse.

What it is for: the forward kernels are checked on factors with the structure a real quantisation run
produces (mixed-sign envelope modes of decaying size, sign masks correlated with the weights), next to the
i.i.d. factors the benchmark configurations prescribe; and the HIP library's MSVID_l entry point (mdbf_msvid)
is compared with msvid() and with Theorem 1's closed form in tests/test_gpu_msvid.py.

Notation (paper -> here): W (N x M) ~ U V^T, U = S_a o (A Q^T) (N x R), V = S_b o (B G^T) (M x R).  The
forward oracle's layer uses m = N, n = M, k = R, SA = S_a, SB = S_b^T, and the same A, Q, G, B.

Readings of the paper taken here:
  * TSVD_l(|Z|) is returned as a pair of factors; the paper does not say how the singular values are
    split between them.  They are split evenly: A = U_l diag(sqrt(sigma)), Q = V_l diag(sqrt(sigma)).
  * sign(0) = +1 (Sec. 2, Notation).
  * One outer refinement sweep = `inner` iterations of the three-step update for U with V fixed, then the
    same for V on the transposed problem with U fixed (Sec. 4.3.2).  The scaled dual variable starts at
    zero at the beginning of every block of inner iterations.
  * The paper gives no value for rho.  `quantize` takes it relative to the mean eigenvalue of V^T V of
    the block being solved (rho = rho_rel * trace(V^T V) / R): with rho_rel between 1 and 10 the error of
    the test matrices falls sweep after sweep; far below, the sign-adaptive step undoes the fit.

Parity status: every function is pinned by tests/test_quantizer_pins.py (Theorem 1's closed-form error,
Eckart-Young for the initialisation, fixed points, first-order optimality of the least-squares step; the
refinement loop over several inner iterations and one full outer sweep against the three update
equations retyped with bare numpy calls, with planted mistakes -- a flipped dual update, a prox without
the dual variable, no U / V alternation -- shown to be caught).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def sign_pm1(Z):
    """Entrywise sign into {+1, -1}, sign(0) = +1 (Sec. 2, Notation)."""
    return np.where(np.asarray(Z) < 0, -1, 1).astype(np.int8)


def tsvd_factors(E, l):
    """Best rank-l approximation of E in Frobenius norm (Eckart-Young), as factors (A, Q), E_l = A Q^T."""
    E = np.asarray(E, dtype=F64)
    if not (1 <= l <= min(E.shape)):
        raise ValueError("need 1 <= l <= min(shape)")
    Uf, s, Vt = np.linalg.svd(E, full_matrices=False)
    r = np.sqrt(s[:l])
    return Uf[:, :l] * r, Vt[:l, :].T * r


def msvid(Z, l):
    """MSVID_l[Z] = sign(Z) o TSVD_l(|Z|)  (Eq. "msvid-def").  Returns (S, A, Q): the value is S o (A Q^T)."""
    Z = np.asarray(Z, dtype=F64)
    S = sign_pm1(Z)
    A, Q = tsvd_factors(np.abs(Z), l)
    return S, A, Q


def msvid_value(Z, l):
    S, A, Q = msvid(Z, l)
    return S.astype(F64) * (A @ Q.T)


def fixed_mask_optimum(U, S, l):
    """Best approximation of U in F_l(S) = {S o E : rank E <= l}: S o TSVD_l(S o U)  (Theorem 1, Eq. "Ustar")."""
    S = np.asarray(S, dtype=F64)
    A, Q = tsvd_factors(S * np.asarray(U, dtype=F64), l)
    return S * (A @ Q.T)


def balanced_factors(W, R):
    """U_0 = U_R Sigma_R^(1/2), V_0 = V_R Sigma_R^(1/2) from the rank-R truncated SVD of W (Eq. "mesvid-balanced")."""
    W = np.asarray(W, dtype=F64)
    if not (1 <= R <= min(W.shape)):
        raise ValueError("need 1 <= R <= min(shape)")
    Uf, s, Vt = np.linalg.svd(W, full_matrices=False)
    r = np.sqrt(s[:R])
    return Uf[:, :R] * r, Vt[:R, :].T * r


def least_squares_step(W, V, U, Lam, rho):
    """U~ = (W V + rho (U - Lam)) (V^T V + rho I)^(-1)  (Eq. "admm-U-tilde")."""
    W = np.asarray(W, dtype=F64)
    V = np.asarray(V, dtype=F64)
    R = V.shape[1]
    rhs = W @ V + rho * (np.asarray(U, dtype=F64) - np.asarray(Lam, dtype=F64))
    gram = V.T @ V + rho * np.eye(R)
    # X gram = rhs  <=>  gram^T X^T = rhs^T; gram is symmetric
    return np.linalg.solve(gram, rhs.T).T


def _value(f):
    S, A, Q = f
    return S.astype(F64) * (A @ Q.T)


def refine_factor(W, fU, V, l, rho, inner):
    """`inner` iterations of Eqs. "admm-U-tilde", "admm-U-prox", "admm-U-dual" for U with V fixed.
    fU = (S, A, Q) with U = S o (A Q^T); returns the refined factor in the same form."""
    U = _value(fU)
    Lam = np.zeros_like(U)
    for _ in range(inner):
        Ut = least_squares_step(W, V, U, Lam, rho)
        fU = msvid(Ut + Lam, l)
        U = _value(fU)
        Lam = Lam + Ut - U
    return fU


def quantize(W, R, l, rho_rel=1.0, outer=0, inner=3):
    """Initialise by MSVID_l of the balanced factors (Eq. "mesvid-init-compact"), then `outer` refinement
    sweeps (Sec. 4.3.2).  Returns the forward oracle's layer: dict with m, n, k, l, SA, SB, A, Q, G, B."""
    W = np.asarray(W, dtype=F64)
    U0, V0 = balanced_factors(W, R)
    fU = msvid(U0, l)
    fV = msvid(V0, l)
    for _ in range(outer):
        V = _value(fV)
        fU = refine_factor(W, fU, V, l, rho_rel * np.trace(V.T @ V) / R, inner)
        U = _value(fU)
        fV = refine_factor(W.T, fV, U, l, rho_rel * np.trace(U.T @ U) / R, inner)
    SA, A, Q = fU
    Sv, B, G = fV          # V = S_b o (B G^T), M x R
    N, M = W.shape
    return dict(m=N, n=M, k=R, l=l, SA=SA, SB=np.ascontiguousarray(Sv.T), A=A, Q=Q, G=G, B=B)


def relative_error(W, What):
    W = np.asarray(W, dtype=F64)
    return float(np.linalg.norm(W - np.asarray(What, dtype=F64)) / np.linalg.norm(W))
