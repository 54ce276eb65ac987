"""The simplified linear program of Sec. 3.2 for k = 2 drafts on a DENSE joint draft distribution
(test infrastructure, CPU only): the largest acceptance any verification rule can reach for a
given Q.  Variables pi(x1, x2 -> x1) and pi(x1, x2 -> x2) >= 0; a pair cannot give away more than
its mass, sum_i pi(x1, x2 -> x_i) <= Q(x1, x2); a token cannot receive more than its target
probability, sum over pairs and slots that hold y of pi(. -> y) <= p(y); maximise the total.
Q is q(x1) q(x2) for draws with replacement ("OTM" in the toy table of App. D) and
q(x1) q(x2) / (1 - q(x1)), x1 != x2, without ("OTMw"; Sec. 3.3 gives both)."""
import numpy as np
import scipy.optimize
import scipy.sparse as sp


def joint_draft(q, without_replacement):
    q = np.asarray(q, dtype=np.float64)
    if without_replacement:
        Q = np.outer(q, q) / (1.0 - q)[:, None]
        np.fill_diagonal(Q, 0.0)
        return Q
    return np.outer(q, q)


def optimal_acceptance(p, Q):
    """Optimum of the LP: 1 - (optimal transport cost with the membership cost)."""
    p = np.asarray(p, dtype=np.float64)
    V = p.size
    n = V * V
    idx = np.arange(n)
    x1, x2 = idx // V, idx % V
    eye = sp.identity(n, format="csr")
    ones = np.ones(n)
    pair_rows = sp.hstack([eye, eye])
    token_rows = sp.hstack([sp.csr_matrix((ones, (x1, idx)), shape=(V, n)),
                            sp.csr_matrix((ones, (x2, idx)), shape=(V, n))])
    res = scipy.optimize.linprog(-np.ones(2 * n), A_ub=sp.vstack([pair_rows, token_rows]).tocsr(),
                                 b_ub=np.concatenate([Q.ravel(), p]), bounds=(0, None), method="highs")
    assert res.status == 0, res.message
    return float(-res.fun)
