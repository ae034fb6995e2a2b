"""CPU oracle for the Multi-Envelope Double Binary Factorization (MDBF) forward product.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
check and the CPU-baseline leg of the benchmark may import it.  It shares no
code, table, header or helper with the HIP library and never calls it.

Everything here is plain numpy in float64, written from the paper's equations.
No blocking, fusion or re-ordering beyond what each cited equation states.

Notation (paper -> this file)
-----------------------------
The paper approximates W in R^{N x M} by  W_l = U_l V_l^T  with
U_l = S_a o (A Q^T)  (N x R)   and   V_l = S_b o (B G^T)  (M x R)
(Sec. 4.2, Eq. "me-dbf-basis";  `o` is the Hadamard product).  Here

    m := N,  n := M,  k := R,  l := l,
    SA := S_a            (m x k, entries +-1)
    SB := S_b^T          (k x n, entries +-1)
    A (m x l), Q (k x l), G (k x l), B (n x l)   -- the real envelope factors
    What = U @ V,   U = SA o (A Q^T)  (m x k),   V = SB o (G B^T)  (k x n)

and the deployment product is  y = What x  for one token, Y[b,:] = What X[b,:]
for a batch X (T x n) -> Y (T x m).  The paper writes the row-vector form
Y = X What (Sec. 3.2, paragraph "Inference"); the format is symmetric under
transposition (swap A<->B, Q<->G, SA<->SB^T), so both describe one operation.

Parity status: every function below is pinned by tests/test_oracle_pins.py
(hand-worked fixture, closed forms, invariants, brute force); none is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


def _signs(S):
    S = np.asarray(S)
    if not np.all((S == 1) | (S == -1)):
        raise ValueError("sign matrix entries must be +1 or -1")
    return S.astype(F64)


# --------------------------------------------------------------------------
# sign convention
# --------------------------------------------------------------------------
def sign_pm1(Z):
    """Entrywise sign into {+1,-1} with sign(0) = +1 (Sec. 2, Notation)."""
    Z = np.asarray(Z)
    return np.where(Z < 0, -1, 1).astype(np.int8)


def demodulate(S, Z):
    """Demodulated envelope E_S(Z) = S o Z (Sec. 3.2, "Single-Envelope Constraint")."""
    return _signs(S) * _f64(Z)


# --------------------------------------------------------------------------
# the matrix the format denotes
# --------------------------------------------------------------------------
def factor_U(SA, A, Q):
    """U = S_a o (A Q^T), shape (m, k).  Eq. "me-dbf-basis"."""
    return _signs(SA) * (_f64(A) @ _f64(Q).T)


def factor_V(SB, G, B):
    """V = (S_b o (B G^T))^T = SB o (G B^T), shape (k, n).  Eq. "me-dbf-basis"."""
    return _signs(SB) * (_f64(G) @ _f64(B).T)


def dense_reconstruct(SA, SB, A, Q, G, B):
    """What = U V, shape (m, n).  Eq. "me-dbf-basis"."""
    return factor_U(SA, A, Q) @ factor_V(SB, G, B)


def forward_dense(SA, SB, A, Q, G, B, X):
    """Y[b,:] = What X[b,:] with What built densely first (the plain definition)."""
    W = dense_reconstruct(SA, SB, A, Q, G, B)
    X = np.atleast_2d(_f64(X))
    return X @ W.T


def forward_bruteforce(SA, SB, A, Q, G, B, X):
    """Entry-by-entry evaluation of the definition with Python loops (tiny shapes only).

    What[i,j] = sum_r  SA[i,r] (sum_t A[i,t] Q[r,t])  *  SB[r,j] (sum_s G[r,s] B[j,s])
    y[i]      = sum_j  What[i,j] x[j]                     (Eq. "me-dbf-basis")
    """
    SA = np.asarray(SA); SB = np.asarray(SB)
    A = _f64(A); Q = _f64(Q); G = _f64(G); B = _f64(B)
    X = np.atleast_2d(_f64(X))
    m, k = SA.shape
    n = SB.shape[1]
    l = A.shape[1]
    T = X.shape[0]
    Y = np.zeros((T, m), dtype=F64)
    for b in range(T):
        for i in range(m):
            acc = 0.0
            for j in range(n):
                w = 0.0
                for r in range(k):
                    eu = 0.0
                    ev = 0.0
                    for t in range(l):
                        eu += A[i, t] * Q[r, t]
                        ev += G[r, t] * B[j, t]
                    w += float(SA[i, r]) * eu * float(SB[r, j]) * ev
                acc += w * X[b, j]
            Y[b, i] = acc
    return Y


# --------------------------------------------------------------------------
# the method's own evaluation order
# --------------------------------------------------------------------------
def forward_factored(SA, SB, A, Q, G, B, X, return_intermediates=False):
    """y = U (V x) through the per-factor expansion of Eq. "me-dbf-expand":

        V = sum_s D_{g^(s)} SB D_{b^(s)},    U = sum_t D_{a^(t)} SA D_{q^(t)}

    i.e. per factor, l envelope-scaled binary products whose results are summed:
        xs[j,s] = B[j,s] x[j]                  scale in
        P1[r,s] = sum_j SB[r,j] xs[j,s]        binary product 1
        z[r]    = sum_s G[r,s] P1[r,s]         envelope accumulate 1
        zs[r,t] = Q[r,t] z[r]                  re-scale
        P2[i,t] = sum_r SA[i,r] zs[r,t]        binary product 2
        y[i]    = sum_t A[i,t] P2[i,t]         envelope accumulate 2
    No intermediate is rounded.
    """
    SAf = _signs(SA); SBf = _signs(SB)
    A = _f64(A); Q = _f64(Q); G = _f64(G); B = _f64(B)
    X = np.atleast_2d(_f64(X))
    T = X.shape[0]
    m = SAf.shape[0]
    Y = np.empty((T, m), dtype=F64)
    Z = np.empty((T, SAf.shape[1]), dtype=F64)
    for b in range(T):
        xs = B * X[b][:, None]            # (n, l)
        P1 = SBf @ xs                     # (k, l)
        z = np.sum(G * P1, axis=1)        # (k,)
        zs = Q * z[:, None]               # (k, l)
        P2 = SAf @ zs                     # (m, l)
        Y[b] = np.sum(A * P2, axis=1)     # (m,)
        Z[b] = z
    if return_intermediates:
        return Y, Z
    return Y


def forward_residual_stack(terms, X):
    """y = sum_p What^(p) x for a residual stack of independently factorised terms (the two-term form
    of Eq. "dbf-residual-comp", any number of terms, each an MDBF factorisation with its own sign bases
    and envelopes): the plain sum of the terms' products.  terms: sequence of (SA, SB, A, Q, G, B)."""
    X = np.atleast_2d(_f64(X))
    Y = None
    for (SA, SB, A, Q, G, B) in terms:
        Yp = forward_factored(SA, SB, A, Q, G, B, X)
        Y = Yp if Y is None else Y + Yp
    return Y


def dbf_forward(SA, SB, a, mvec, b, X):
    """Plain DBF, y = D_a SA D_m SB D_b x, in the printed evaluation order of
    Eq. "DBF-inference-form" (scale, binary product, scale, binary product, scale),
    transposed to the column-vector convention used here."""
    SAf = _signs(SA); SBf = _signs(SB)
    a = _f64(a); mvec = _f64(mvec); b = _f64(b)
    X = np.atleast_2d(_f64(X))
    Y = np.empty((X.shape[0], SAf.shape[0]), dtype=F64)
    for t in range(X.shape[0]):
        v = X[t] * b
        v = SBf @ v
        v = v * mvec
        v = SAf @ v
        Y[t] = v * a
    return Y


def forward_sum_of_dbf(SA, SB, A, Q, G, B, X):
    """l^2 plain-DBF forwards, summed.  Eq. "me-dbf-sum":
    What = sum_t sum_s D_{a^(t)} SA D_{q^(t) o g^(s)} SB D_{b^(s)}."""
    A = _f64(A); Q = _f64(Q); G = _f64(G); B = _f64(B)
    X = np.atleast_2d(_f64(X))
    l = A.shape[1]
    Y = np.zeros((X.shape[0], np.asarray(SA).shape[0]), dtype=F64)
    for t in range(l):
        for s in range(l):
            Y += dbf_forward(SA, SB, A[:, t], Q[:, t] * G[:, s], B[:, s], X)
    return Y


# --------------------------------------------------------------------------
# storage accounting and rank selection
# --------------------------------------------------------------------------
def bits_per_weight(m, n, k, l, env_bits=16, merge_inner=False):
    """Stored bits over the m*n entries of the matrix that is replaced.

    Sec. 3.2 ("Inference", last sentence) states the rule for DBF: bit-packed
    {S_a,S_b} plus the real vectors {a,b,m}, relative to the N*M entries.  For
    MDBF the stored real factors are A (m x l), Q (k x l), B (n x l), G (k x l)
    (Eq. "me-dbf-basis"), hence
        bpw = [ (m+n) k  +  env_bits * l * (m + n + 2k) ] / (m n).
    With merge_inner=True and l=1 the two inner vectors are stored as the one
    vector m = q o g, which is the DBF count  [(m+n)k + e(m+n+k)]/(mn).
    Padding bits of any packed layout are not counted.
    """
    sign_bits = (m + n) * k
    if merge_inner:
        if l != 1:
            raise ValueError("merge_inner only applies to l == 1 (plain DBF)")
        real_entries = m + n + k
    else:
        real_entries = l * (m + n + 2 * k)
    return (sign_bits + env_bits * real_entries) / float(m * n)


def rank_for_budget(m, n, l, bpw, env_bits=16, multiple=1):
    """Inner rank for a bits-per-weight budget.

    multiple == 1: the largest k whose bits_per_weight does not exceed the
    budget (Sec. 5.1, "largest inner rank that meets the budget").
    multiple  > 1: the real-valued solution of bits_per_weight(k) = bpw rounded
    to the NEAREST multiple (this is the rule that reproduces the word-aligned
    ranks 2656 and 4096 of the 1.5-bpw LLaMA-7B shapes; it may exceed the budget
    by a fraction of a percent).
    """
    k_real = (bpw * m * n - env_bits * l * (m + n)) / float((m + n) + 2 * env_bits * l)
    if multiple <= 1:
        k = int(np.floor(k_real + 1e-9))
        while k > 0 and bits_per_weight(m, n, k, l, env_bits) > bpw + 1e-12:
            k -= 1
        while bits_per_weight(m, n, k + 1, l, env_bits) <= bpw + 1e-12:
            k += 1
        return max(k, 0)
    return int(multiple * np.floor(k_real / multiple + 0.5))


# --------------------------------------------------------------------------
# logical reference bit layout (the bit-exactness contract for pack/unpack)
# --------------------------------------------------------------------------
def pack_ref(S):
    """Row-major reference packing: 32-bit little-endian words, entry c of a row
    in word c//32, bit c%32; bit value 1 <=> sign -1; rows padded with 0 bits
    (= +1) to a whole word.  Returns uint32 array (rows, ceil(cols/32))."""
    S = np.asarray(S)
    if not np.all((S == 1) | (S == -1)):
        raise ValueError("sign matrix entries must be +1 or -1")
    rows, cols = S.shape
    words = (cols + 31) // 32
    out = np.zeros((rows, words), dtype=np.uint32)
    for c in range(cols):
        neg = (S[:, c] < 0).astype(np.uint32)
        out[:, c // 32] |= neg << np.uint32(c % 32)
    return out


def unpack_ref(P, cols):
    """Inverse of pack_ref: uint32 (rows, words) -> int8 (rows, cols) of +-1."""
    P = np.asarray(P, dtype=np.uint32)
    rows = P.shape[0]
    S = np.empty((rows, cols), dtype=np.int8)
    for c in range(cols):
        bit = (P[:, c // 32] >> np.uint32(c % 32)) & np.uint32(1)
        S[:, c] = np.where(bit == 1, -1, 1)
    return S


# --------------------------------------------------------------------------
# error measure used by the parity gate
# --------------------------------------------------------------------------
def max_rel_error(Y, Yref):
    """max |Y - Yref| / max |Yref|  (norm-wise; element-wise relative error is
    unbounded because individual outputs are sums of thousands of +- terms)."""
    Y = _f64(Y); Yref = _f64(Yref)
    den = np.max(np.abs(Yref))
    if den == 0.0:
        return float(np.max(np.abs(Y)))
    return float(np.max(np.abs(Y - Yref)) / den)
