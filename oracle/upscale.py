"""CPU oracle of the any-precision quantiser (incremental upscaling, Any-Precision LLM Section 4).

Test infrastructure only; numpy, float64, one output channel at a time, no blocking.  Shares no
code with the HIP package and never imports it.

Steps, in the paper's order (Section 4.1, Section 4.2):
  1. seed model: cluster the weights of a channel into 2^n_seed groups by weighted k-means, the
     weight of an element being its sensitivity (SqueezeLLM-style non-uniform quantisation);
  2. upscale n_seed -> n one bit at a time: divide every cluster in two sub-clusters by a weighted
     2-means over its members; a member's new index is the old index with one bit appended;
  3. the table of the b-bit model holds the centroids of the clusters at level b.

The paper leaves the clustering details open.  The reading taken here: one-dimensional Lloyd
iterations that start from the values found at the weighted quantiles (q + 0.5)/k, run `iters`
rounds at most (stop when nothing moves), send a point to the nearest centroid (ties to the lower
index), leave the centroid of an empty cluster where it was; clusters are numbered by ascending
centroid, so the sub-cluster with the smaller centroid gets bit 0; a cluster whose 2-means puts all
members on one side passes its centroid to both children and its members to child 0.
"""
import numpy as np


def weighted_kmeans_1d(v, s, k, iters):
    """Lloyd's algorithm on scalars v with weights s; returns (centroids[k], assignment[len(v)])."""
    v = np.asarray(v, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    m = v.size
    if m == 0:
        return np.zeros(k), np.zeros(0, dtype=np.int64)
    order = np.argsort(v, kind="stable")
    cum = np.zeros(m)
    acc = 0.0
    for r, i in enumerate(order):          # running sum in sorted order
        acc = acc + s[i]
        cum[r] = acc
    total = cum[-1]
    centroids = np.empty(k)
    for q in range(k):
        target = (q + 0.5) / k * total
        r = int(np.searchsorted(cum, target, side="left"))   # first rank with cum >= target
        centroids[q] = v[order[min(r, m - 1)]]
    assign = np.zeros(m, dtype=np.int64)
    for it in range(iters + 1):
        dist = np.abs(v[:, None] - centroids[None, :])
        new_assign = np.argmin(dist, axis=1)                 # first minimum = lower index on ties
        changed = bool(np.any(new_assign != assign))
        assign = new_assign
        if it == iters or (not changed and it > 0):
            break
        num = np.bincount(assign, weights=s * v, minlength=k)   # sums run in element order
        den = np.bincount(assign, weights=s, minlength=k)
        for q in range(k):
            if den[q] > 0.0:
                centroids[q] = num[q] / den[q]
    return centroids, assign


def upscale_channel(w, s, n_seed, n, iters):
    """One output channel: returns (codes[K] at n bits, {b: centroids[2^b]} for n_seed <= b <= n)."""
    w = np.asarray(w, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    c, a = weighted_kmeans_1d(w, s, 1 << n_seed, iters)
    by = np.argsort(c, kind="stable")
    rank = np.empty_like(by)
    rank[by] = np.arange(by.size)
    code = rank[a]
    cent = c[by]
    tables = {n_seed: cent.copy()}
    for b in range(n_seed, n):
        nxt = np.empty(2 << b)
        nxt_code = np.empty_like(code)
        for parent in range(1 << b):
            members = np.nonzero(code == parent)[0]
            c2, a2 = weighted_kmeans_1d(w[members], s[members], 2, iters)
            if members.size == 0 or np.all(a2 == a2[0]):
                nxt[2 * parent] = nxt[2 * parent + 1] = cent[parent]
                nxt_code[members] = 2 * parent
            else:
                lo = 1 if c2[1] < c2[0] else 0
                nxt[2 * parent] = c2[lo]
                nxt[2 * parent + 1] = c2[1 - lo]
                nxt_code[members] = 2 * parent + (a2 ^ lo)
        cent, code = nxt, nxt_code
        tables[b + 1] = cent.copy()
    return code, tables


def upscale(W, S, n_seed, n, iters):
    """Whole matrix: (idx uint8 (M, K), {b: float16 (M, 2^b)}); tables rounded to binary16 at the end."""
    W = np.asarray(W, dtype=np.float64)
    M, K = W.shape
    S = np.ones_like(W) if S is None else np.asarray(S, dtype=np.float64)
    idx = np.empty((M, K), dtype=np.uint8)
    luts = {b: np.empty((M, 1 << b), dtype=np.float16) for b in range(n_seed, n + 1)}
    for i in range(M):
        code, tables = upscale_channel(W[i], S[i], n_seed, n, iters)
        idx[i] = code
        for b, t in tables.items():
            luts[b][i] = t.astype(np.float16)
    return idx, luts
