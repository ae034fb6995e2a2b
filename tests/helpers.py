"""Helpers shared by the test modules (not part of the product package)."""
import numpy as np


def concat_terms(terms):
    """Several layers of one shape (m, n), each with its own sign bases and envelope factors, written as ONE
    layer: inner dimension sum(k_p), envelope rank sum(l_p); sign bases side by side (S_A) resp. stacked
    (S_B), outer envelope factors A, B side by side, inner ones Q, G block-diagonal.  Pure data movement:
    the layer it returns denotes the sum of the terms' matrices."""
    m, n = terms[0]["m"], terms[0]["n"]
    ks, ls = [t["k"] for t in terms], [t["l"] for t in terms]
    K, Lr = sum(ks), sum(ls)
    dt = terms[0]["A"].dtype
    Q = np.zeros((K, Lr), dtype=dt)
    G = np.zeros((K, Lr), dtype=dt)
    r0 = c0 = 0
    for t, k, l in zip(terms, ks, ls):
        Q[r0:r0 + k, c0:c0 + l] = t["Q"]
        G[r0:r0 + k, c0:c0 + l] = t["G"]
        r0, c0 = r0 + k, c0 + l
    return dict(m=m, n=n, k=K, l=Lr, SA=np.hstack([t["SA"] for t in terms]), SB=np.vstack([t["SB"] for t in terms]),
                A=np.hstack([t["A"] for t in terms]), Q=Q, G=G, B=np.hstack([t["B"] for t in terms]),
                env_dtype=terms[0]["env_dtype"])
