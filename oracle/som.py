"""Batch-SOM training epoch, written out plainly in float64 on the CPU.  TEST INFRASTRUCTURE ONLY.

This module is the yardstick the HIP path is compared against.  It is imported only by the tests, by the
smoke check and by the CPU-baseline leg of the benchmark; it shares no code with the GPU library.

What one epoch computes (paper Section 3.3.1, Eq. 3 and the paragraph after Eq. 4, with learning rate 1 and
no momentum):

  * every presented sample x gets its best-matching unit b(x): the node whose weight vector is nearest in
    squared Euclidean distance under the weights of the *start* of the epoch (lowest index on exact ties);
  * node j collects  Num_j = sum_x h(G[b(x), j]) x   and   Den_j = sum_x h(G[b(x), j]),
    where G is the node-to-node neighbourhood distance (lattice distance or graph hop count) and
    h(g) = exp(-g^2 / (2 sigma^2)) is the Gaussian influence at radius sigma;
  * w_j <- Num_j / Den_j, unless Den_j is below a fixed threshold (the "numerical safeguard"), in which
    case w_j is left as it was.

``epoch_definition`` is that statement written out sample by sample.  ``epoch_grouped`` is an algebraically
identical rearrangement (group the samples by BMU first) that uses a BLAS product for the distances; it
exists so that million-row inputs finish in seconds and is itself checked against ``epoch_definition``.

Pins (tests/test_oracle_*.py): hand-worked tiny cases under tests/golden/, scipy's cdist for the distances,
K = 1 gives the data mean, sigma -> 0 gives one Lloyd k-means step, sigma -> infinity gives the data mean
everywhere, every new weight is a convex combination of the presented samples, the Eq. 3 displacement form
w + U/H equals Num/Den, sample-order / chunk / shard invariance, node-relabelling equivariance.
"""
from __future__ import annotations

import math

import numpy as np

DEFAULT_EPS_H = 1e-30   # denominators below this leave the node unchanged


# ----------------------------------------------------------------------------------------------------
# Eq. 1: sampling budget
# ----------------------------------------------------------------------------------------------------
def sampling_budget(n: int, rho: float | None = None, m0: int | None = None) -> int:
    """Number of samples presented per iteration (Section 3.1, Eq. 1).

    A fixed budget m0 is used as given; a proportion rho gives max(1, floor(n * rho)).  A budget of n or
    more means the full dataset (text after Eq. 2).
    """
    if (rho is None) == (m0 is None):
        raise ValueError("give exactly one of rho, m0")
    m = int(m0) if m0 is not None else max(1, int(math.floor(n * rho)))
    return min(m, n)


# ----------------------------------------------------------------------------------------------------
# best-matching unit (Section 3.3.1, definition of b(x))
# ----------------------------------------------------------------------------------------------------
def sq_distances(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """d2[i, k] = sum_d (X[i, d] - W[k, d])^2 by direct differences in float64."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    diff = X[:, None, :] - W[None, :, :]
    return np.einsum("ikd,ikd->ik", diff, diff)


def bmu(X: np.ndarray, W: np.ndarray, block: int = 2048):
    """Best-matching unit of every row of X under weights W.

    Returns (b, d2_best, d2_second): b[i] is the lowest node index attaining the minimum squared distance,
    d2_best[i] that minimum and d2_second[i] the smallest distance among the *other* nodes (inf if K = 1).
    Rows are processed in blocks only to bound memory; each row's result does not depend on the blocking.
    """
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    m, K = X.shape[0], W.shape[0]
    b = np.empty(m, dtype=np.int64)
    best = np.empty(m, dtype=np.float64)
    second = np.full(m, np.inf, dtype=np.float64)
    for lo in range(0, m, block):
        hi = min(m, lo + block)
        d2 = sq_distances(X[lo:hi], W)
        bb = np.argmin(d2, axis=1)             # numpy's argmin returns the first (lowest) index of the minimum
        rows = np.arange(hi - lo)
        b[lo:hi] = bb
        best[lo:hi] = d2[rows, bb]
        if K > 1:
            d2[rows, bb] = np.inf
            second[lo:hi] = d2.min(axis=1)
    return b, best, second


def near_tie_mask(d2_best: np.ndarray, d2_second: np.ndarray, rel: float = 1e-5) -> np.ndarray:
    """True where the best two distances are closer than ``rel`` relative to the second best.

    For such samples more than one BMU is an acceptable answer in float32 arithmetic.
    """
    d2_second = np.asarray(d2_second, dtype=np.float64)
    finite = np.isfinite(d2_second)                      # K = 1 has no runner-up, hence no tie
    denom = np.where(finite, np.maximum(d2_second, np.finfo(np.float64).tiny), 1.0)
    gap = np.where(finite, d2_second - d2_best, np.inf)
    return gap / denom < rel


def quantization_error(d2_best: np.ndarray) -> float:
    """Mean Euclidean distance from each sample to its BMU (the quantisation error of Section 4.1.2)."""
    return float(np.mean(np.sqrt(d2_best))) if len(d2_best) else 0.0


# ----------------------------------------------------------------------------------------------------
# neighbourhood influence
# ----------------------------------------------------------------------------------------------------
def influence(G: np.ndarray, sigma: float) -> np.ndarray:
    """Gaussian influence h = exp(-G^2 / (2 sigma^2)); an infinite distance gives exactly 0."""
    G = np.asarray(G, dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        h = np.exp(-(G * G) / (2.0 * float(sigma) ** 2))
    h[np.isinf(G)] = 0.0
    return h


# ----------------------------------------------------------------------------------------------------
# one epoch, as defined
# ----------------------------------------------------------------------------------------------------
def epoch_definition(X, idx, W, G, sigma, eps_h: float = DEFAULT_EPS_H, chunk: int = 4096):
    """One batch epoch straight from the definition (Eq. 3 with learning rate 1, then U/H).

    X    (N, D) samples;   idx  presented row numbers or None for all rows
    W    (K, D) weights at the start of the epoch;   G (K, K) neighbourhood distances;   sigma radius
    Returns a dict: W (new weights), b, d2_best, d2_second, num, den, guarded (bool per node), qe, mean_d2.
    The sums run sample by sample; ``chunk`` only bounds the size of the temporary (chunk, K) influence rows,
    which is the chunk-wise accumulation the paper itself describes.
    """
    X = np.asarray(X)
    W0 = np.asarray(W, dtype=np.float64)
    K, D = W0.shape
    rows = np.arange(X.shape[0]) if idx is None else np.asarray(idx, dtype=np.int64)
    Xp = np.asarray(X[rows], dtype=np.float64)
    b, best, second = bmu(Xp, W0)
    h = influence(G, sigma)
    num = np.zeros((K, D), dtype=np.float64)
    den = np.zeros(K, dtype=np.float64)
    for lo in range(0, len(rows), chunk):
        hi = min(len(rows), lo + chunk)
        hx = h[b[lo:hi], :]                    # (chunk, K): influence of each sample's BMU on every node
        num += hx.T @ Xp[lo:hi]
        den += hx.sum(axis=0)
    guarded = ~(den >= eps_h)
    Wn = W0.copy()
    ok = ~guarded
    Wn[ok] = num[ok] / den[ok, None]
    return dict(W=Wn, b=b, d2_best=best, d2_second=second, num=num, den=den, guarded=guarded,
                qe=quantization_error(best), mean_d2=float(best.mean()) if len(best) else 0.0)


def displacement_form_update(X, b, W, G, sigma, eta: float = 1.0):
    """Eq. 3 as printed: U_j = sum eta h (x - w_j), H_j = sum h, new w_j = w_j + U_j / H_j (no safeguard)."""
    Xp = np.asarray(X, dtype=np.float64)
    W0 = np.asarray(W, dtype=np.float64)
    h = influence(G, sigma)
    K, D = W0.shape
    U = np.zeros((K, D))
    H = np.zeros(K)
    for i in range(Xp.shape[0]):
        for j in range(K):
            hij = h[j, b[i]]
            U[j] += eta * hij * (Xp[i] - W0[j])
            H[j] += hij
    return W0 + U / H[:, None]


# ----------------------------------------------------------------------------------------------------
# the grouped rearrangement (per-BMU sums first)
# ----------------------------------------------------------------------------------------------------
def accumulate(X, idx, b, K: int):
    """Per-node sample sums S[k] = sum_{i: b_i = k} x_i and counts n[k]."""
    X = np.asarray(X)
    rows = np.arange(X.shape[0]) if idx is None else np.asarray(idx, dtype=np.int64)
    D = X.shape[1]
    S = np.zeros((K, D), dtype=np.float64)
    np.add.at(S, np.asarray(b, dtype=np.int64), np.asarray(X[rows], dtype=np.float64))
    n = np.bincount(np.asarray(b, dtype=np.int64), minlength=K).astype(np.int64)
    return S, n


def neighborhood_update(S, n, G, sigma, W, eps_h: float = DEFAULT_EPS_H):
    """w_j <- (sum_k h(G[k, j]) S_k) / (sum_k h(G[k, j]) n_k), guarded nodes unchanged.

    Returns (W_new, guarded, den).
    """
    S = np.asarray(S, dtype=np.float64)
    nn = np.asarray(n, dtype=np.float64)
    W0 = np.asarray(W, dtype=np.float64)
    h = influence(G, sigma)
    num = h.T @ S
    den = h.T @ nn
    guarded = ~(den >= eps_h)
    Wn = W0.copy()
    ok = ~guarded
    Wn[ok] = num[ok] / den[ok, None]
    return Wn, guarded, den


def neighborhood_update_momentum(S, n, G, sigma, W, V, eta: float = 1.0, mu: float = 0.0,
                                 eps_h: float = DEFAULT_EPS_H):
    """General update of the paragraph after Eq. 4: learning rate inside U, optional momentum on the normalised update.

    u_j = eta * (Num_j / Den_j - w_j)  (= U_j / H_j of Eq. 3), or 0 where the denominator is below the threshold;
    delta_j = u_j + mu * V_j;  w_j <- w_j + delta_j;  the new velocity is delta_j.  Returns (W_new, V_new, guarded).
    """
    S = np.asarray(S, dtype=np.float64)
    nn = np.asarray(n, dtype=np.float64)
    W0 = np.asarray(W, dtype=np.float64)
    V0 = np.zeros_like(W0) if V is None else np.asarray(V, dtype=np.float64)
    h = influence(G, sigma)
    num = h.T @ S
    den = h.T @ nn
    guarded = ~(den >= eps_h)
    u = np.zeros_like(W0)
    ok = ~guarded
    u[ok] = eta * (num[ok] / den[ok, None] - W0[ok])
    delta = u + mu * V0
    return W0 + delta, delta, guarded


def neighborhood_update_shifted(S, n, G, sigma, W):
    """The update with the other possible reading of the guard that the paragraph after Eq. 4 asks for on U_j / H_j:
    instead of a threshold on the denominator, every updated node j has its exponents shifted by the smallest
    squared distance to an occupied node,

        m_j = min_{k: n_k > 0} G[k][j]^2,     h'_kj = exp(-(G[k][j]^2 - m_j) / (2 sigma^2))  for n_k > 0, else 0,

    and w_j = sum_k h'_kj S_k / sum_k h'_kj n_k.  The factor exp(m_j / 2 sigma^2) cancels in the ratio, so wherever
    the plain sums do not underflow the result is the same; where they do, the node follows its nearest occupied
    nodes instead of standing still.  A node that no occupied node reaches (m_j infinite) is left unchanged.
    Returns (W_new, unchanged) with ``unchanged`` the mask of such nodes.
    """
    S = np.asarray(S, dtype=np.float64)
    nn = np.asarray(n, dtype=np.float64)
    W0 = np.asarray(W, dtype=np.float64)
    g2 = np.asarray(G, dtype=np.float64) ** 2
    K = g2.shape[0]
    occupied = nn > 0
    Wn = W0.copy()
    unchanged = np.ones(K, dtype=bool)
    for j in range(K):
        col = g2[occupied, j]
        if col.size == 0 or not np.isfinite(col.min()):
            continue
        hj = np.exp(-(col - col.min()) / (2.0 * sigma * sigma))
        hj[~np.isfinite(col)] = 0.0
        Wn[j] = (hj @ S[occupied]) / (hj @ nn[occupied])
        unchanged[j] = False
    return Wn, unchanged


def bmu_gram(X, W, block: int = 65536, rel_tol: float = 1e-9):
    """BMU through |x|^2 - 2 x.w + |w|^2 with a float64 BLAS product; checked against ``bmu`` in the tests.

    The Gram form only shortlists: the two nodes with the smallest Gram values are re-evaluated by direct
    differences and ordered by (distance, node index), so the returned distances carry no cancellation error and
    an exact tie between them goes to the lower index whatever order the rounded Gram values put them in.  A
    row in which a third node's Gram value lies within ``rel_tol`` (|x|^2 + max |w|^2) of the smallest one - a
    margin some 10^5 times the rounding error of the float64 Gram form - could have its lowest-index minimum
    outside that pair; such rows are decided by ``bmu``, i.e. by the definition over all nodes.
    """
    X = np.asarray(X)
    W = np.asarray(W, dtype=np.float64)
    m, K = X.shape[0], W.shape[0]
    wn = np.einsum("kd,kd->k", W, W)
    b = np.empty(m, dtype=np.int64)
    best = np.empty(m, dtype=np.float64)
    second = np.full(m, np.inf, dtype=np.float64)
    for lo in range(0, m, block):
        hi = min(m, lo + block)
        Xb = np.asarray(X[lo:hi], dtype=np.float64)
        if K == 1:
            b[lo:hi] = 0
            best[lo:hi] = np.einsum("id,id->i", Xb - W[0], Xb - W[0])
            continue
        g = wn[None, :] - 2.0 * (Xb @ W.T)
        rows = np.arange(hi - lo)
        c0 = np.argmin(g, axis=1)
        g0 = g[rows, c0]
        g[rows, c0] = np.inf
        c1 = np.argmin(g, axis=1)
        g[rows, c1] = np.inf
        tol = rel_tol * (np.einsum("id,id->i", Xb, Xb) + wn.max())
        crowded = np.nonzero(g.min(axis=1) <= g0 + tol)[0] if K > 2 else np.empty(0, dtype=np.int64)
        d0 = np.einsum("id,id->i", Xb - W[c0], Xb - W[c0])
        d1 = np.einsum("id,id->i", Xb - W[c1], Xb - W[c1])
        swap = (d1 < d0) | ((d1 == d0) & (c1 < c0))
        b[lo:hi] = np.where(swap, c1, c0)
        best[lo:hi] = np.where(swap, d1, d0)
        second[lo:hi] = np.where(swap, d0, d1)
        if crowded.size:
            bb, db, ds = bmu(Xb[crowded], W)
            b[lo + crowded] = bb
            best[lo + crowded] = db
            second[lo + crowded] = ds
        del g, rows
    return b, best, second


def epoch_grouped(X, idx, W, G, sigma, eps_h: float = DEFAULT_EPS_H, b=None):
    """The same epoch as ``epoch_definition``, rearranged: BMUs, per-node sums, then one K x K contraction."""
    X = np.asarray(X)
    W0 = np.asarray(W, dtype=np.float64)
    K = W0.shape[0]
    rows = np.arange(X.shape[0]) if idx is None else np.asarray(idx, dtype=np.int64)
    Xp = X[rows]
    if b is None:
        b, best, second = bmu_gram(Xp, W0)
    else:
        best = second = None
    S, n = accumulate(Xp, None, b, K)
    Wn, guarded, den = neighborhood_update(S, n, G, sigma, W0, eps_h)
    out = dict(W=Wn, b=b, S=S, n=n, den=den, guarded=guarded)
    if best is not None:
        out.update(d2_best=best, d2_second=second, qe=quantization_error(best),
                   mean_d2=float(best.mean()) if len(best) else 0.0)
    return out
