"""Graphs, Laplacian, chi_1, chi_2 and the hyper-parameter rule (test infrastructure, numpy fp64).

Definition 3.1 (instantaneous expected Laplacian), the two definitions that follow it
(chi_1: inverse of the smallest non-zero eigenvalue; chi_2: half the largest effective
resistance over the edges) and Proposition 3.2 (eta, alpha, alpha_tilde).
"""
import numpy as np


def complete(n):
    return [(i, j) for i in range(n) for j in range(i + 1, n)]


def ring(n):
    if n == 2:
        return [(0, 1)]
    return sorted({(min(i, (i + 1) % n), max(i, (i + 1) % n)) for i in range(n)})


def exponential(n):
    """Each node i is linked to i + 2^k (mod n) for every 2^k < n; undirected union, no duplicates."""
    edges = set()
    k = 1
    while k < n:
        for i in range(n):
            j = (i + k) % n
            if i != j:
                edges.add((min(i, j), max(i, j)))
        k *= 2
    return sorted(edges)


def laplacian(n, edges, rates):
    """Lambda = sum over edges of rate * (e_i - e_j)(e_i - e_j)^T  (Definition 3.1)."""
    lam = np.zeros((n, n))
    for (i, j), r in zip(edges, np.broadcast_to(rates, (len(edges),))):
        v = np.zeros(n); v[i] = 1.0; v[j] = -1.0
        lam += r * np.outer(v, v)
    return lam


def chi1(lam):
    """sup over unit x orthogonal to 1 of 1 / (x^T Lambda x) = 1 / (second smallest eigenvalue)."""
    w = np.linalg.eigvalsh(lam)
    return 1.0 / w[1]


def chi2(lam, edges):
    """1/2 * max over edges of (e_i - e_j)^T Lambda^+ (e_i - e_j)."""
    pinv = np.linalg.pinv(lam, hermitian=True)
    best = 0.0
    for i, j in edges:
        v = np.zeros(lam.shape[0]); v[i] = 1.0; v[j] = -1.0
        best = max(best, 0.5 * v @ pinv @ v)
    return best


def acid_params(n, edges, rates):
    """Proposition 3.2, accelerated setting: eta = 1/(2 sqrt(chi1 chi2)), alpha = 1/2,
    alpha_tilde = 1/2 sqrt(chi1 / chi2)."""
    lam = laplacian(n, edges, rates)
    c1, c2 = chi1(lam), chi2(lam, edges)
    return {"chi1": c1, "chi2": c2, "eta": 0.5 / np.sqrt(c1 * c2), "alpha": 0.5,
            "alpha_tilde": 0.5 * np.sqrt(c1 / c2)}


def baseline_params():
    """Proposition 3.2, non-accelerated setting."""
    return {"eta": 0.0, "alpha": 0.5, "alpha_tilde": 0.5}


def per_worker_to_edge_rate(n, edges, comm_per_grad):
    """Each worker does comm_per_grad p2p averagings per unit time, peers uniform over its
    neighbours: n * comm_per_grad / 2 communications per unit time spread evenly over the edges
    (regular graphs; the expected total matches Tr(Lambda)/2 of Proposition 3.2)."""
    return (n * comm_per_grad / 2.0) / len(edges)
