"""Incremental upscaling (Section 4): pins of the numpy oracle, then the host C-ABI quantiser
against it.  No GPU involved: the quantiser is host code."""
import itertools

import numpy as np
import pytest

from oracle import upscale as O
from paper_2402_10517_amd import binding as B


def _channel(seed, K, heavy=False):
    rng = np.random.default_rng([20240210, 77, seed])
    w = rng.normal(0.0, 0.02, K)
    if heavy:
        w[rng.integers(0, K, max(1, K // 64))] *= 8.0          # a few outliers, as LLM weights have
    s = rng.gamma(0.5, 1.0, K) + 1e-6                          # skewed positive sensitivities
    return w, s


def _wsse(w, s, cent, code):
    return float(np.sum(s * (w - cent[code]) ** 2))


# ---- pins of the oracle against what the mathematics fixes -------------------------------------

def test_two_means_matches_exhaustive_split_on_tiny_inputs():
    # In one dimension the optimal 2-clustering is a split of the sorted values; Lloyd must end in
    # a split whose cost no single-boundary move improves, and on well separated data it is the optimum.
    rng = np.random.default_rng(5)
    for _ in range(40):
        m = int(rng.integers(3, 9))
        v = np.concatenate([rng.normal(-1, 0.1, m // 2), rng.normal(1, 0.1, m - m // 2)])
        s = rng.uniform(0.5, 2.0, m)
        c, a = O.weighted_kmeans_1d(v, s, 2, 50)
        best = min(
            (sum(s[g] @ (v[g] - (s[g] @ v[g]) / s[g].sum()) ** 2 for g in (np.argsort(v)[:cut], np.argsort(v)[cut:])), cut)
            for cut in range(1, m))
        assert _wsse(v, s, c, a) == pytest.approx(best[0], rel=1e-12, abs=1e-15)


def test_kmeans_fixed_point_properties():
    # After convergence every centroid is the weighted mean of its members and every point sits
    # with its nearest centroid (the two Lloyd conditions), checked from their definitions.
    w, s = _channel(1, 700, heavy=True)
    c, a = O.weighted_kmeans_1d(w, s, 8, 500)
    for q in range(8):
        g = a == q
        assert g.any()
        assert c[q] == pytest.approx(np.sum(s[g] * w[g]) / np.sum(s[g]), rel=1e-12)
    d = np.abs(w[:, None] - c[None, :])
    assert np.all(d[np.arange(w.size), a] <= d.min(axis=1))


def test_weights_matter_and_uniform_weights_give_plain_mean():
    v = np.array([0.0, 1.0, 10.0, 11.0])
    c, a = O.weighted_kmeans_1d(v, np.ones(4), 2, 20)
    assert list(a) == [0, 0, 1, 1] and list(c) == [0.5, 10.5]
    c, a = O.weighted_kmeans_1d(v, np.array([3.0, 1.0, 1.0, 3.0]), 2, 20)
    assert list(c) == [0.25, 10.75]                      # (3*0 + 1*1)/4, (1*10 + 3*11)/4


def test_upscale_nesting_and_prefix_property():
    # Section 4.1: the b-bit model's index is the prefix of the parent index, i.e. the members of a
    # level-b cluster are exactly the members of its two children at level b+1.
    w, s = _channel(2, 1024, heavy=True)
    code, tables = O.upscale_channel(w, s, 3, 8, 30)
    assert code.min() >= 0 and code.max() < 256
    for b in range(3, 8):
        cb, cb1 = code >> (8 - b), code >> (8 - b - 1)
        assert np.array_equal(cb1 >> 1, cb)
        for parent in range(1 << b):
            g = cb == parent
            if not g.any():
                continue
            lo, hi = tables[b + 1][2 * parent], tables[b + 1][2 * parent + 1]
            assert lo <= hi                               # child with the smaller centroid gets bit 0
            # children lie inside the parent's range of values
            assert w[g].min() - 1e-15 <= lo and hi <= w[g].max() + 1e-15


def test_seed_level_equals_direct_kmeans_and_is_independent_of_n():
    # The seed model is the plain weighted clustering; upscaling further never changes lower levels.
    w, s = _channel(3, 512)
    c, a = O.weighted_kmeans_1d(w, s, 8, 30)
    code5, t5 = O.upscale_channel(w, s, 3, 5, 30)
    code8, t8 = O.upscale_channel(w, s, 3, 8, 30)
    assert np.array_equal(np.sort(c), t8[3])
    assert np.array_equal(code8 >> 3, code5)
    for b in (3, 4, 5):
        assert np.array_equal(t5[b], t8[b])


def test_error_never_increases_with_bit_width_and_centroids_are_weighted_means():
    w, s = _channel(4, 2048, heavy=True)
    code, tables = O.upscale_channel(w, s, 3, 8, 100)
    errs = [_wsse(w, s, tables[b], code >> (8 - b)) for b in range(3, 9)]
    assert all(e1 <= e0 * (1 + 1e-12) for e0, e1 in zip(errs, errs[1:]))
    assert errs[-1] < errs[0] / 100                      # roughly 4x per bit on smooth data
    for b in range(3, 9):
        cb = code >> (8 - b)
        for q in range(1 << b):
            g = cb == q
            if g.sum() >= 2 and (b == 3 or tables[b][q] != tables[b - 1][q >> 1]):
                assert tables[b][q] == pytest.approx(np.sum(s[g] * w[g]) / np.sum(s[g]), rel=1e-9)


def test_degenerate_channels():
    # constant channel: nothing can be divided; every table entry used is that constant
    w = np.full(64, 0.125)
    code, tables = O.upscale_channel(w, np.ones(64), 3, 8, 10)
    assert np.all(tables[8][code] == 0.125)
    for b in range(3, 9):
        assert np.all(tables[b][code >> (8 - b)] == 0.125)
    # fewer distinct values than clusters: exact representation at every level that has enough entries
    w = np.tile(np.array([-1.0, -0.5, 0.25, 2.0]), 16)
    code, tables = O.upscale_channel(w, np.ones(64), 3, 8, 10)
    assert np.array_equal(tables[8][code], w)
    assert np.array_equal(tables[3][code >> 5], w)


def test_zero_weight_elements_do_not_move_centroids():
    v = np.array([0.0, 1.0, 5.0, 100.0])
    c, a = O.weighted_kmeans_1d(v, np.array([1.0, 1.0, 1.0, 0.0]), 2, 20)
    # the zero-sensitivity outlier joins a cluster without shifting its mean
    assert sorted(c) == [0.5, 5.0] and a[3] == int(np.argmax(c))


# ---- the C-ABI quantiser against the oracle -----------------------------------------------------

@pytest.mark.parametrize("M,K,n_seed,n,use_sens", [
    (8, 256, 3, 8, True), (5, 96, 3, 8, False), (4, 512, 4, 6, True), (3, 64, 3, 3, True),
    (6, 1000, 2, 8, True), (2, 33, 1, 4, False)])
def test_ap_quantize_matches_oracle(M, K, n_seed, n, use_sens):
    rng = np.random.default_rng([20240210, 78, M, K])
    W = rng.normal(0.0, 0.02, (M, K)).astype(np.float32)
    W[rng.integers(0, M, 3), rng.integers(0, K, 3)] *= 10.0
    S = (rng.gamma(0.5, 1.0, (M, K)) + 1e-6).astype(np.float32) if use_sens else None
    idx, luts = B.ap_quantize(W, S, n_seed=n_seed, n=n, iters=25)
    ridx, rluts = O.upscale(W, S, n_seed, n, 25)
    assert np.array_equal(idx, ridx)
    assert set(luts) == set(rluts)
    for b in luts:
        assert np.array_equal(luts[b].view(np.uint16), rluts[b].view(np.uint16)), b


def test_ap_quantize_degenerate_rows_and_errors():
    W = np.zeros((3, 64), dtype=np.float32)
    W[1] = 0.5
    W[2, ::2] = -1.0
    idx, luts = B.ap_quantize(W, None, 3, 8, 5)
    ridx, rluts = O.upscale(W, None, 3, 8, 5)
    assert np.array_equal(idx, ridx)
    for b in luts:
        assert np.array_equal(luts[b].view(np.uint16), rluts[b].view(np.uint16))
    deq = np.take_along_axis(luts[8].astype(np.float32), idx.astype(np.int64), axis=1)
    assert np.array_equal(deq, W)
    for bad in (dict(n_seed=0, n=8), dict(n_seed=5, n=4), dict(n_seed=3, n=9)):
        with pytest.raises(B.ApError):
            B.ap_quantize(W, None, iters=5, **bad)
    with pytest.raises(B.ApError):
        B.ap_quantize(W, None, 3, 8, 0)


def test_half_rounding_of_tables_is_nearest_even():
    # rows holding a single value v: every used table entry is v rounded to binary16; values sit on
    # and around rounding boundaries, in the subnormal range and beyond the largest finite value
    vals = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20, 6.0e-8, 2.9e-8,
                     3.1e-8, 65504.0, 65519.0, 65520.0, -1.0e-5, 6.1e-5, 2.0 ** -14 - 2.0 ** -26], dtype=np.float32)
    W = np.repeat(vals[:, None], 32, axis=1)
    idx, luts = B.ap_quantize(W, None, 3, 4, 3)
    got = np.take_along_axis(luts[4], idx.astype(np.int64), axis=1)[:, 0]
    with np.errstate(over="ignore"):
        want = vals.astype(np.float64).astype(np.float16)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_quantize_pack_round_trip_feeds_the_packer():
    rng = np.random.default_rng(9)
    W = rng.normal(0, 0.02, (8, 128)).astype(np.float32)
    idx, luts = B.ap_quantize(W, None, 3, 8, 10)
    blob = B.ap_pack_host(idx, {b: t for b, t in luts.items()}, 8)
    assert np.array_equal(B.ap_unpack_host(blob, 8, 128), idx)


# ---- the C-ABI quantiser against the definitions of Section 4 themselves (not against its oracle) ----

def _f16(v):
    return np.asarray(v, dtype=np.float64).astype(np.float16).astype(np.float64)


def test_ap_quantize_output_satisfies_the_definitions():
    # What Section 4.1 / 4.2 fix, checked on the product's own output: (1) the members of a level-b
    # cluster are the members of its two children (prefix property of the indices); (2) a level-b
    # table entry is the sensitivity-weighted mean of the members of its cluster (binary16-rounded),
    # unless the cluster could not be divided and inherited its parent's centroid; (3) the weighted
    # squared error does not grow with b; (4) the models below n do not depend on n.
    rng = np.random.default_rng([20240210, 78])
    M, K = 6, 1536
    W = (rng.standard_t(5, (M, K)) * 0.02).astype(np.float32)
    S = (rng.gamma(0.5, 1.0, (M, K)) + 1e-6).astype(np.float32)
    idx8, luts8 = B.ap_quantize(W, S, 3, 8, 60)
    idx6, luts6 = B.ap_quantize(W, S, 3, 6, 60)
    assert np.array_equal(idx8 >> 2, idx6)                                   # (4)
    for b in range(3, 7):
        assert np.array_equal(luts8[b].view(np.uint16), luts6[b].view(np.uint16))
    w64, s64 = W.astype(np.float64), S.astype(np.float64)
    for i in range(M):
        errs = []
        for b in range(3, 9):
            code = idx8[i].astype(np.int64) >> (8 - b)
            tab = luts8[b][i].astype(np.float64)
            errs.append(float(np.sum(s64[i] * (w64[i] - tab[code]) ** 2)))
            for q in range(1 << b):
                g = code == q
                if not g.any():
                    continue
                mean = np.sum(s64[i][g] * w64[i][g]) / np.sum(s64[i][g])
                inherited = b > 3 and tab[q] == luts8[b - 1][i].astype(np.float64)[q >> 1]
                if not inherited:
                    # (2): equal after rounding to binary16, or one binary16 step away when the mean
                    # sits on a rounding boundary (sums are taken in a different order here)
                    assert abs(tab[q] - _f16(mean)) <= np.spacing(np.float16(abs(tab[q]))).astype(np.float64), (i, b, q)
                if b < 8:                                                    # (1)
                    child = idx8[i][g].astype(np.int64) >> (8 - b - 1)
                    assert set(np.unique(child)) <= {2 * q, 2 * q + 1}
        # (3), with the slack of rounding every table to binary16
        assert all(e1 <= e0 * 1.001 + 1e-12 for e0, e1 in zip(errs, errs[1:])), errs
        assert errs[-1] < errs[0] / 50


def _optimal_by_enumeration(v, s, k):
    """Exact optimum of weighted 1-D k-means by brute force: some optimal clustering consists of k runs
    of the sorted values, so trying every way to cut the sorted order into k runs finds it."""
    order = np.argsort(v, kind="stable")
    v, s = v[order], s[order]
    m = v.size
    best = np.inf
    for cuts in itertools.combinations(range(1, m), k - 1):
        edges = (0,) + cuts + (m,)
        cost = 0.0
        for lo, hi in zip(edges, edges[1:]):
            mean = np.sum(s[lo:hi] * v[lo:hi]) / np.sum(s[lo:hi])
            cost += float(np.sum(s[lo:hi] * (v[lo:hi] - mean) ** 2))
        best = min(best, cost)
    return best


def _optimal_by_dynamic_programming(v, s, k):
    """The same optimum for channels too long to enumerate: best[j][i] = cheapest way to cover the first
    i sorted values with j runs = min over l of best[j-1][l] + cost of the run l..i (prefix sums)."""
    order = np.argsort(v, kind="stable")
    v, s = v[order], s[order]
    m = v.size
    S0 = np.concatenate([[0.0], np.cumsum(s)])
    S1 = np.concatenate([[0.0], np.cumsum(s * v)])
    S2 = np.concatenate([[0.0], np.cumsum(s * v * v)])

    def run_cost(lo, hi):
        w, a, q = S0[hi] - S0[lo], S1[hi] - S1[lo], S2[hi] - S2[lo]
        return np.maximum(q - a * a / w, 0.0)

    prev = np.concatenate([[0.0], run_cost(0, np.arange(1, m + 1))])
    for j in range(2, k + 1):
        cur = np.full(m + 1, np.inf)
        for i in range(j, m + 1):
            lo = np.arange(j - 1, i)
            cur[i] = np.min(prev[lo] + run_cost(lo, i))
        prev = cur
    return float(prev[m])


def test_seed_level_against_the_exact_optimum():
    # Lloyd's iteration promises a local optimum only, and where it lands depends on the start, the
    # tie rule and the empty-cluster rule (readings Q3-Q5): nothing the paper prints fixes those.  What
    # the mathematics fixes is the optimum of the weighted k-means objective itself, which in one
    # dimension can be computed exactly.  Pins: (a) the exact solver, by enumeration on tiny channels;
    # (b) the seed model is never cheaper than the optimum and is a Lloyd fixed point; (c) how far above
    # the optimum it ends, on channels of realistic length, for the oracle and for the product alike.
    rng = np.random.default_rng([20240210, 79])
    for trial in range(30):                                   # (a) + (b) on tiny channels
        K = int(rng.integers(9, 13))
        n_seed = 2 if trial % 2 else 3
        k = 1 << n_seed
        v = rng.normal(0, 1, K)
        s = rng.gamma(0.5, 1.0, K) + 1e-3
        opt = _optimal_by_enumeration(v, s, k)
        assert _optimal_by_dynamic_programming(v, s, k) == pytest.approx(opt, rel=1e-9, abs=1e-12)
        c, a = O.weighted_kmeans_1d(v, s, k, 100)
        assert _wsse(v, s, c, a) >= opt * (1 - 1e-9) - 1e-15
        d = np.abs(v[:, None] - c[None, :])
        assert np.all(d[np.arange(K), a] <= d.min(axis=1) + 1e-15)
    ratios = []
    for seed in range(8):                                     # (c) realistic lengths, 8 clusters
        for K in (256, 1024):
            w, s = _channel(seed, K, heavy=seed % 2 == 1)
            opt = _optimal_by_dynamic_programming(w, s, 8)
            c, a = O.weighted_kmeans_1d(w, s, 8, 200)
            cost = _wsse(w, s, c, a)
            assert cost >= opt * (1 - 1e-9)
            idx, luts = B.ap_quantize(w[None, :].astype(np.float32), s[None, :].astype(np.float32), 3, 3, 200)
            tab = luts[3][0].astype(np.float64)
            pcost = float(np.sum(s * (w - tab[idx[0]]) ** 2))
            assert pcost >= opt * (1 - 1e-3)                  # binary32 inputs, binary16 table
            assert pcost == pytest.approx(cost, rel=2e-2)     # the product lands where its oracle lands
            ratios.append(cost / opt)
    # Measured spread of the quantile start on these channels: 1.02 .. 2.7 times the optimal cost (the
    # heavy-tailed channels, whose outliers would each need a cluster of their own, are the far ones).
    # The bound documents that spread; it is not a quality claim.
    assert 1.0 <= min(ratios) and max(ratios) < 3.5, ratios


def test_two_means_split_against_the_best_cut():
    # The upscaling step divides a cluster in two (Section 4.2).  The optimal weighted 2-means of scalars
    # is the best single cut of the sorted values; Lloyd from the quantile start must not beat it and, on
    # the members of real clusters, ends close to it.
    w, s = _channel(11, 4096, heavy=True)
    code, tables = O.upscale_channel(w, s, 3, 4, 100)
    worst = 1.0
    for parent in range(8):
        g = (code >> 1) == parent
        if g.sum() < 3:
            continue
        opt = _optimal_by_dynamic_programming(w[g], s[g], 2)
        c, a = O.weighted_kmeans_1d(w[g], s[g], 2, 100)
        cost = _wsse(w[g], s[g], c, a)
        assert cost >= opt * (1 - 1e-9)
        worst = max(worst, cost / opt)
    assert worst < 1.5, worst        # measured 1.29 on this channel (the cluster that holds the outliers)
