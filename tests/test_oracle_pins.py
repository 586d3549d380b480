"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the HIP path.  Each test names the passage of the paper
(arXiv 2410.13056) or the textbook fact it checks the oracle against, and is
chosen so that a plausible slip in the oracle (dropped term, wrong sign or
index, transposed operand, wrong tie rule) fails it.
"""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


# ----------------------------------------------------------------------------- fp16 codec

def test_half_codec_matches_numpy_on_every_pattern(orc):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.f16_bits_to_f64(int(b)) for b in bits])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


def test_float_to_half_rounds_to_nearest_even_like_numpy(orc):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.normal(0, 1, 4000), rng.normal(0, 1e-3, 2000), rng.normal(0, 1e-6, 2000),
        rng.normal(0, 3e4, 1000), np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -25,
                                             2.0 ** -25 * 1.0001, 2.0 ** -24 * 1.5, 2.0 ** -24 * 2.5])
    ]).astype(np.float32)
    # exact half-way cases between neighbouring halves
    h = rng.integers(0, 0x7BFF, 3000).astype(np.uint16)
    mid = ((h.view(np.float16).astype(np.float64) + (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)) / 2)
    xs = np.concatenate([xs, mid.astype(np.float32), -mid.astype(np.float32)])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([orc.f32_to_f16_bits(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ----------------------------------------------------------------------------- Sec. 3.2.1 statistics

def test_act_stats_is_squared_column_norm(orc):
    rng = np.random.default_rng(2)
    for dt in (np.float16, np.float32):
        X = rng.normal(0, 1, (301, 77)).astype(dt)
        acc, sumsq = orc.act_stats(X)
        ref = np.linalg.norm(X.astype(np.float64), axis=0) ** 2
        assert np.allclose(acc, ref, rtol=1e-12, atol=0)
        assert np.array_equal(sumsq, acc.astype(np.float32))


def test_act_stats_constant_column_chunks_and_permutation(orc):
    rng = np.random.default_rng(3)
    n, d = 500, 33
    X = rng.normal(0, 2, (n, d)).astype(np.float32)
    X[:, 5] = 0.75                                   # closed form n * v^2
    acc, _ = orc.act_stats(X)
    assert acc[5] == n * 0.75 ** 2
    a1, _ = orc.act_stats(X[:123])
    a2, s2 = orc.act_stats(X[123:], acc=a1)          # streaming tokens
    assert np.allclose(a2, acc, rtol=1e-14)
    accp, _ = orc.act_stats(X[rng.permutation(n)])   # token order is irrelevant
    assert np.allclose(accp, acc, rtol=1e-13)
    accs, _ = orc.act_stats((X * 4).astype(np.float32))
    assert np.allclose(accs, 16 * acc, rtol=1e-14)   # power-of-two scaling is exact
    # a transposed-operand slip would reduce over the wrong axis
    assert acc.shape == (d,)


# ----------------------------------------------------------------------------- Sec. 3.2.2 O_act

def _rank_order(keys):
    """indices sorted by (key descending, index ascending) - the textbook definition."""
    return sorted(range(len(keys)), key=lambda i: (-float(keys[i]), i))


def test_top_channels_equals_full_sort_with_ties(orc):
    rng = np.random.default_rng(4)
    d = 400
    s = rng.integers(0, 40, d).astype(np.float32)      # many ties
    for k in (0, 1, 7, 123, d):
        idx, mask = orc.top_channels(s, k)
        ref = sorted(_rank_order(s)[:k])
        assert list(idx) == ref
        assert mask.sum() == k and set(np.flatnonzero(mask)) == set(ref)


def test_outlier_counts_follow_printed_fractions(orc):
    ppm = {r[0]: int(r[1]) for r in _rows("sec3_2_2_outlier_fractions.txt")}
    assert ppm["rho_act"] + ppm["rho_q"] == ppm["rho_total"]
    # counts the scope table quotes for the LLaMA shapes
    for d_in, k in [(256, 1), (4096, 18), (11008, 50), (5120, 23), (13824, 62), (8192, 37), (28672, 129)]:
        assert orc.count_ppm(ppm["rho_act"], d_in) == k
    assert orc.count_ppm(5000, 512 * 256) == 655
    assert orc.count_ppm(ppm["rho_q"], 4096 * 4096) == 8389
    assert orc.count_ppm(5000, 4096 * 4096) == 83886


# ----------------------------------------------------------------------------- Algorithm 1

def _literal_alg1(a, b):
    """Algorithm 1 as printed, with numpy's linearly interpolated quantile."""
    c = np.full(a.shape, 3)
    if b > 3:
        c[a > np.quantile(a, 1 - (b - 3))] = 4
    elif b < 3:
        c[a < np.quantile(a, 3 - b)] = 2
    else:
        c[a < np.quantile(a, 0.01)] = 2
        c[a > np.quantile(a, 0.99)] = 4
    return c


def test_allocation_against_printed_algorithm_rows(orc):
    rng = np.random.default_rng(5)
    for b, d, n2, n3, n4 in _rows("alg1_branches.txt"):
        b, d, want = float(b), int(d), (int(n2), int(n3), int(n4))
        a = rng.permutation(d).astype(np.float32) + 1.0          # tie free
        lit = _literal_alg1(a.astype(np.float64), b)
        assert tuple(int((lit == w).sum()) for w in (2, 3, 4)) == want   # the fixture is Algorithm 1
        bits, counts = orc.allocate_bits(a, None, (2, 3, 4), b)
        got = tuple(int((bits == w).sum()) for w in (2, 3, 4))
        assert tuple(counts) == got
        assert all(abs(g - w) <= 1 for g, w in zip(got, want)), (got, want)
        # same channels, not just same counts: at most one channel differs per threshold
        assert int((bits != lit).sum()) <= 2


@pytest.mark.parametrize("bit_set", [(2, 3), (2, 3, 4), (3, 4), (1, 2, 3, 4)])
def test_allocation_budget_is_exact_and_monotone(orc, bit_set):
    rng = np.random.default_rng(6)
    for d in (7, 256, 1000, 4096):
        a = rng.lognormal(0, 1, d).astype(np.float32)
        a[rng.integers(0, d, d // 10)] = a[0]                    # ties
        for b in np.linspace(bit_set[0], bit_set[-1], 23):
            bits, counts = orc.allocate_bits(a, None, bit_set, float(b))
            assert counts.sum() == d and set(np.unique(bits)) <= set(bit_set)
            total = int(bits.astype(np.int64).sum())
            if abs(b - round(b)) < 1e-9:
                assert total == round(b) * d                     # symmetric branch: average exactly b
                assert len(np.unique(bits)) in (1, 3)
            else:
                T = int(np.floor(b * d + 1e-9))
                assert total == T and T / d <= b < T / d + 1.0 / d
                assert len(np.unique(bits)) <= 2
            order = _rank_order(a)                               # more salient => never fewer bits
            assert all(bits[order[j]] >= bits[order[j + 1]] for j in range(d - 1))


def test_allocation_closed_forms_and_protection(orc):
    a = np.arange(1, 257, dtype=np.float32)
    bits, counts = orc.allocate_bits(a, None, (2, 3), 2.5)
    assert list(counts) == [128, 128] and (bits[128:] == 3).all() and (bits[:128] == 2).all()
    a = np.arange(1, 4097, dtype=np.float32)
    _, mask = orc.top_channels(a, 18)
    bits, counts = orc.allocate_bits(a, mask, (2, 3, 4), 3.0)    # d_eff = 4078
    assert list(counts) == [41, 3996, 41]
    assert (bits[mask == 1] == orc.PROTECTED).all() and (bits[-18:] == orc.PROTECTED).all()
    assert (bits[:41] == 2).all() and (bits[4096 - 18 - 41:4096 - 18] == 4).all()
    for b, w in ((2.0, 2), (4.0, 4)):                            # ends of the range: uniform
        bits, _ = orc.allocate_bits(a, None, (2, 3, 4), b)
        assert (bits == w).all()
    bits, _ = orc.allocate_bits(a, None, (2, 3), 3.0)            # no neighbour above: uniform
    assert (bits == 3).all()
    with pytest.raises(ValueError):
        orc.allocate_bits(a, None, (2, 3), 3.5)
    with pytest.raises(ValueError):
        orc.allocate_bits(a, None, (2, 4), 3.0)


def test_scaling_activations_leaves_integer_outputs_unchanged(orc):
    rng = np.random.default_rng(7)
    X = rng.normal(0, 1, (64, 300)).astype(np.float32) * rng.lognormal(0, 1, 300).astype(np.float32)
    _, s1 = orc.act_stats(X)
    _, s2 = orc.act_stats(X * np.float32(8.0))
    for b in (2.3, 3.0, 3.7):
        i1, m1 = orc.top_channels(s1, 3)
        i2, m2 = orc.top_channels(s2, 3)
        assert np.array_equal(i1, i2)
        assert np.array_equal(orc.allocate_bits(s1, m1, (2, 3, 4), b)[0],
                              orc.allocate_bits(s2, m2, (2, 3, 4), b)[0])


# ----------------------------------------------------------------------------- K-means (Sec. 3.2.1)

def _optimal_sse(x, K):
    """Exact optimum of 1-D K-clustering by dynamic programming over the sorted values."""
    x = np.sort(np.asarray(x, np.float64))
    m = len(x)
    p1 = np.concatenate([[0.0], np.cumsum(x)])
    p2 = np.concatenate([[0.0], np.cumsum(x * x)])

    def cost(i, j):  # cluster x[i:j]
        s, q, n = p1[j] - p1[i], p2[j] - p2[i], j - i
        return max(q - s * s / n, 0.0)

    INF = float("inf")
    D = np.full((K + 1, m + 1), INF)
    D[0, 0] = 0.0
    for k in range(1, K + 1):
        for j in range(1, m + 1):
            D[k, j] = min([D[k - 1, i] + cost(i, j) for i in range(k - 1, j) if D[k - 1, i] < INF],
                          default=INF)
    return min(D[k, m] for k in range(1, K + 1))


def _sorted_lloyd(x, w, K, iters):
    """Independent second implementation of the oracle's K-means: works on the
    sorted values with prefix sums; a cell is the run of values closer to its
    level than to any other (ties to the smaller level index)."""
    x = np.asarray(x, np.float64).copy()
    x[x == 0] = 0.0
    w = np.asarray(w, np.float64)
    inc = np.sort(x[w > 0])
    M = len(inc)
    c = np.array([inc[((2 * j + 1) * M) // (2 * K)] if M else 0.0 for j in range(K)], np.float32)
    order = np.argsort(x, kind="stable")
    xs, ws = x[order], w[order]
    pw = np.concatenate([[0.0], np.cumsum(ws)])

    def assign(c):
        # distinct level values, each owned by its smallest index
        cd = c.astype(np.float64)
        owners = {}
        for j in range(K):
            owners.setdefault(cd[j], j)
        vals = sorted(owners)
        edges = [0]
        for lo, hi in zip(vals[:-1], vals[1:]):
            mid = (lo + hi) / 2.0
            side = "right" if owners[lo] < owners[hi] else "left"   # tie -> smaller index
            edges.append(int(np.searchsorted(xs, mid, side=side)))
        edges.append(len(xs))
        code_sorted = np.empty(len(xs), np.int64)
        for t, v in enumerate(vals):
            code_sorted[edges[t]:edges[t + 1]] = owners[v]
        return code_sorted

    for _ in range(iters):
        cs = assign(c)
        for j in range(K):
            sel = cs == j
            mass = ws[sel].sum()
            if mass > 0:
                # same summation order as index order is not needed: these test inputs are fp16-exact
                c[j] = np.float32((ws[sel] * xs[sel]).sum() / mass)
    cs = assign(c)
    codes = np.empty(len(x), np.int64)
    codes[order] = cs
    return c, codes


def test_kmeans_never_beats_and_sometimes_reaches_the_optimum(orc):
    rng = np.random.default_rng(8)
    d_in, d_out = 24, 48
    W = rng.normal(0, 1, (d_in, d_out)).astype(np.float16)
    bits = rng.integers(1, 4, d_in).astype(np.uint8)            # K in {2,4,8}
    cent, codes, sse = orc.kmeans(W, bits, iters=30, trace=True)
    for i in range(d_in):
        K = 1 << int(bits[i])
        opt = _optimal_sse(W[i].astype(np.float64), K)
        assert sse[i, -1] >= opt - 1e-9
    # well separated planted clusters: Lloyd from quantile starts lands on the optimum
    K = 4
    centers = np.array([-3.0, -1.0, 1.0, 3.0])
    # equal-sized groups so that the order-statistic start hits every group
    Wp = np.stack([np.concatenate([c + rng.normal(0, 0.01, 16) for c in centers]) for _ in range(6)]).astype(np.float16)
    cent, codes, sse = orc.kmeans(Wp, np.full(6, 2, np.uint8), iters=5, trace=True)
    for i in range(6):
        assert abs(sse[i, -1] - _optimal_sse(Wp[i].astype(np.float64), K)) < 1e-9


def test_kmeans_lloyd_invariants(orc):
    rng = np.random.default_rng(9)
    d_in, d_out = 40, 333
    W = (rng.standard_t(3, (d_in, d_out)) * 0.05).astype(np.float32)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    cent, codes, sse = orc.kmeans(W, bits, iters=60, trace=True)
    # the error never goes up from one assignment to the next
    assert (np.diff(sse, axis=1) <= 1e-12 * (1 + sse[:, :-1])).all()
    for i in range(d_in):
        K = 1 << int(bits[i])
        c = cent[i, :K].astype(np.float64)
        assert np.isinf(cent[i, K:]).all() and (cent[i, K:] > 0).all()
        assert (np.diff(c) >= 0).all()                            # levels stay ordered
        x = W[i].astype(np.float64)
        d = np.abs(x[:, None] - c[None, :])
        assert np.array_equal(codes[i], d.argmin(axis=1))          # nearest level, first on ties
    # after convergence every level is the mean of its members (fixed point)
    cent2, codes2 = orc.kmeans(W, bits, iters=61)
    conv = np.flatnonzero(sse[:, -1] == sse[:, -2])
    assert len(conv) > d_in // 2
    for i in conv:
        K = 1 << int(bits[i])
        for j in range(K):
            mem = W[i][codes2[i] == j].astype(np.float64)
            if len(mem):
                assert abs(mem.mean() - cent2[i, j]) <= 2e-7 * max(1e-3, abs(mem.mean()))


def test_kmeans_matches_independent_sorted_implementation(orc):
    rng = np.random.default_rng(10)
    d_in, d_out = 30, 257
    W = (rng.normal(0, 0.02, (d_in, d_out))).astype(np.float16)
    W[rng.random((d_in, d_out)) < 0.01] *= 20
    W[3, :] = W[3, 0]                                 # one distinct value
    W[4, 100:] = 0.0                                  # heavy duplicates -> duplicate starts
    W[5, ::2] = -W[5, ::2]
    W[6, :40] = np.float16(-0.0)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    excl = np.sort(rng.choice(d_in * d_out, 200, replace=False)).astype(np.int64)
    for out_idx in (None, excl):
        cent, codes = orc.kmeans(W, bits, out_idx=out_idx, iters=12)
        for i in range(d_in):
            K = 1 << int(bits[i])
            w = np.ones(d_out)
            if out_idx is not None:
                loc = out_idx[(out_idx >= i * d_out) & (out_idx < (i + 1) * d_out)] - i * d_out
                w[loc] = 0.0
            c_ref, code_ref = _sorted_lloyd(W[i].astype(np.float64), w, K, 12)
            assert np.array_equal(cent[i, :K], c_ref), i
            assert np.array_equal(codes[i], code_ref), i


def test_kmeans_importance_weights(orc):
    rng = np.random.default_rng(11)
    d_in, d_out = 12, 200
    W = rng.normal(0, 1, (d_in, d_out)).astype(np.float16)
    bits = np.full(d_in, 3, np.uint8)
    ew = rng.integers(0, 4, (d_in, d_out)).astype(np.float32)         # integer weights = repeated points
    cent, codes = orc.kmeans(W, bits, elem_weight=ew, iters=8)
    for i in range(d_in):
        c_ref, code_ref = _sorted_lloyd(W[i].astype(np.float64), ew[i].astype(np.float64), 8, 8)
        assert np.allclose(cent[i, :8], c_ref, rtol=1e-6, atol=0)
        assert np.array_equal(codes[i], code_ref)
    # weight 0 == listing the entry as excluded
    zero = np.flatnonzero(ew.reshape(-1) == 0).astype(np.int64)
    ones = (ew > 0).astype(np.float32)
    c1, k1 = orc.kmeans(W, bits, elem_weight=ones, iters=8)
    c2, k2 = orc.kmeans(W, bits, out_idx=zero, iters=8)
    assert np.array_equal(c1, c2) and np.array_equal(k1, k2)


def test_kmeans_few_distinct_values_and_affine_equivariance(orc):
    rng = np.random.default_rng(12)
    vals = np.array([-0.5, -0.125, 0.0, 0.25, 0.375, 1.0, 2.0], np.float32)
    # 16 copies of each value: the order-statistic start then lands on all seven
    W = np.stack([rng.permutation(np.repeat(vals, 16)) for _ in range(10)])
    cent, codes, sse = orc.kmeans(W, np.full(10, 3, np.uint8), iters=20, trace=True)
    assert (sse[:, -1] == 0).all()                     # #distinct <= K: exact representation
    for i in range(10):
        assert np.array_equal(cent[i][codes[i]], W[i])
    # x -> 4x + 0.5 (exact in fp32 for these inputs): levels follow, codes unchanged
    Wn = (rng.integers(-2000, 2000, (6, 90)) / 1024.0).astype(np.float32)
    c1, k1 = orc.kmeans(Wn, np.full(6, 2, np.uint8), iters=1)
    c2, k2 = orc.kmeans((4 * Wn + 0.5).astype(np.float32), np.full(6, 2, np.uint8), iters=1)
    assert np.array_equal(k1, k2)
    assert np.allclose(c2[:, :4], 4 * c1[:, :4].astype(np.float64) + 0.5, rtol=3e-7)


def test_kmeans_protected_channels_and_empty_channel(orc):
    W = np.linspace(-1, 1, 5 * 64).reshape(5, 64).astype(np.float16)
    bits = np.array([2, 16, 3, 0, 4], np.uint8)
    cent, codes = orc.kmeans(W, bits, iters=3)
    assert np.isinf(cent[1]).all() and np.isinf(cent[3]).all()
    assert (codes[1] == 0).all() and (codes[3] == 0).all()
    all_out = np.arange(64, dtype=np.int64)            # channel 0 entirely excluded
    cent, codes = orc.kmeans(W, bits, out_idx=all_out, iters=3)
    assert (cent[0, :4] == 0).all() and (codes[0] == 0).all()


# ----------------------------------------------------------------------------- O_q (Sec. 3.2.2)

def test_weight_outliers_equal_full_sort(orc):
    rng = np.random.default_rng(13)
    d_in, d_out = 20, 96
    W = (rng.integers(-30, 30, (d_in, d_out)) / 64.0).astype(np.float16)   # coarse grid: many tied residuals
    bits = rng.integers(2, 4, d_in).astype(np.uint8)
    bits[[2, 11]] = orc.PROTECTED
    cent, codes = orc.kmeans(W, bits, iters=5)
    w64 = W.astype(np.float64)
    resid = np.abs(w64 - np.take_along_axis(cent.astype(np.float64), codes.astype(np.int64), axis=1)).astype(np.float32)
    keep = np.repeat((bits <= 4)[:, None], d_out, axis=1).reshape(-1)
    for score, key in ((orc.SCORE_RESIDUAL, resid), (orc.SCORE_MAGNITUDE, np.abs(W).astype(np.float32))):
        flat = key.reshape(-1)
        cand = [i for i in range(d_in * d_out) if keep[i]]
        order = sorted(cand, key=lambda i: (-float(flat[i]), i))
        for k in (0, 1, 10, 97, len(cand)):
            idx, val = orc.weight_outliers(W, cent, codes, bits, k, score)
            assert list(idx) == sorted(order[:k])
            assert np.array_equal(val, W.reshape(-1)[idx].view(np.uint16))
            assert not set(idx // d_out) & {2, 11}            # nothing from O_act channels
    with pytest.raises(ValueError):
        orc.weight_outliers(W, cent, codes, bits, len(cand) + 1)


def test_weight_outliers_without_codes_rank_distance_to_nearest_level(orc):
    """Sec. 3.2.2 with Q(x) of Sec. 3: the preliminary quantization puts each weight on its
    nearest level, so the residual is the distance to the nearest level.  With codes left out
    both selections rank exactly that: equal to a full sort of min_j |w - q_j| (levels that did
    not come from a clustering, so that nothing but the definition is used), and equal to the
    selection with the clustering's own codes."""
    rng = np.random.default_rng(131)
    d_in, d_out = 14, 120
    W = (rng.integers(-30, 30, (d_in, d_out)) / 64.0).astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[3, 9]] = orc.PROTECTED
    live = [i for i in range(d_in) if bits[i] <= 4]
    cent = np.full((d_in, 16), np.inf, np.float32)
    for i in live:                                      # arbitrary levels, unsorted, some repeated
        K = 1 << bits[i]
        cent[i, :K] = rng.choice(np.arange(-28, 28) / 64.0 + 1 / 256.0, K).astype(np.float32)
    dist = np.abs(W.astype(np.float64)[:, :, None] - cent.astype(np.float64)[:, None, :])
    key = np.where(np.isfinite(cent)[:, None, :], dist, np.inf).min(axis=2).astype(np.float32)
    cand = [i * d_out + o for i in live for o in range(d_out)]
    flat = key.reshape(-1)
    order = sorted(cand, key=lambda t: (-float(flat[t]), t))
    for k in (0, 1, 33, len(cand) // 2, len(cand)):
        idx, val = orc.weight_outliers(W, cent, None, bits, k)
        assert list(idx) == sorted(order[:k])
        assert np.array_equal(val, W.reshape(-1)[idx].view(np.uint16))
    for k in (0, 1, 7, d_out):
        idx, _ = orc.weight_outliers_per_channel(W, cent, None, bits, k)
        want = []
        for i in live:
            row = sorted(range(d_out), key=lambda o: (-float(key[i, o]), o))
            want += [i * d_out + o for o in sorted(row[:k])]
        assert list(idx) == want
    # with a clustering's levels and codes: the same selection either way
    c1, k1 = orc.kmeans(W, bits, iters=4)
    for k in (1, 50, len(cand) // 3):
        assert np.array_equal(orc.weight_outliers(W, c1, None, bits, k)[0], orc.weight_outliers(W, c1, k1, bits, k)[0])
    assert np.array_equal(orc.weight_outliers_per_channel(W, c1, None, bits, 5)[0],
                          orc.weight_outliers_per_channel(W, c1, k1, bits, 5)[0])


def test_residual_score_finds_planted_distorters_not_just_big_weights(orc):
    """Sec. 3.2.2: the criterion is the quantization residual, not the magnitude.  A lone
    far value in a tight channel has a large residual; a channel whose values are
    all large but exactly representable has none."""
    rng = np.random.default_rng(14)
    d_in, d_out = 8, 256
    W = rng.normal(0, 0.01, (d_in, d_out)).astype(np.float32)
    W[7] = np.float32(5.0) * np.sign(rng.normal(size=d_out)).astype(np.float32)     # big, two exact levels
    planted = [(0, 17), (1, 200), (3, 3)]
    for i, o in planted:
        W[i, o] = 0.4
    bits = np.full(d_in, 1, np.uint8)                   # two levels: a lone point cannot own one
    cent, codes = orc.kmeans(W, bits, iters=3)
    idx, _ = orc.weight_outliers(W, cent, codes, bits, 3, orc.SCORE_RESIDUAL)
    assert sorted(idx) == sorted(i * d_out + o for i, o in planted)
    idxm, _ = orc.weight_outliers(W, cent, codes, bits, 3, orc.SCORE_MAGNITUDE)
    assert all(i // d_out == 7 for i in idxm)


def test_weight_outliers_per_channel_equal_row_sorts(orc):
    """The per-channel variant of O_q: in every channel outside O_act, the k first entries of
    that row's full (score descending, output index ascending) sort - with a coarse grid so that
    tied scores decide membership; count per channel as the fraction of d_out, half rounded up."""
    rng = np.random.default_rng(113)
    d_in, d_out = 12, 200
    W = (rng.integers(-30, 30, (d_in, d_out)) / 64.0).astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[0, 7]] = orc.PROTECTED
    live = [i for i in range(d_in) if bits[i] <= 4]
    cent, codes = orc.kmeans(W, bits, iters=4)
    resid = np.abs(W.astype(np.float64) - np.take_along_axis(cent.astype(np.float64), codes.astype(np.int64),
                                                            axis=1)).astype(np.float32)
    for score, key in ((orc.SCORE_RESIDUAL, resid), (orc.SCORE_MAGNITUDE, np.abs(W).astype(np.float32))):
        for k in (0, 1, 7, d_out):
            idx, val = orc.weight_outliers_per_channel(W, cent, codes, bits, k, score)
            want = []
            for i in live:
                order = sorted(range(d_out), key=lambda o: (-float(key[i, o]), o))
                want += [i * d_out + o for o in sorted(order[:k])]
            assert list(idx) == want                                   # ascending as a whole, too
            assert np.array_equal(val, W.reshape(-1)[idx].view(np.uint16))
    with pytest.raises(ValueError):
        orc.weight_outliers_per_channel(W, cent, codes, bits, d_out + 1)
    # the count: 0.5 % of 200 outputs is exactly 1, 0.74 % rounds to 1, 0.75 % to 2
    assert [orc.count_ppm(p, d_out) for p in (5000, 7400, 7500)] == [1, 1, 2]
    # a single channel: the two scopes are the same selection
    one = np.full(1, 3, np.uint8)
    c1, k1 = orc.kmeans(W[:1], one, iters=4)
    a, _ = orc.weight_outliers_per_channel(W[:1], c1, k1, one, 9)
    b, _ = orc.weight_outliers(W[:1], c1, k1, one, 9)
    assert np.array_equal(a, b)


def test_per_channel_and_layer_scope_agree_when_outliers_are_spread_evenly(orc):
    """With exactly k far entries planted in every channel (all larger than anything else in
    the layer; magnitude score, so that the clustering plays no part), the layer-wide top
    (k * d_in) of Sec. 3.2.2 and the per-channel top k are the same set; moving one planted
    entry to another channel makes them differ in exactly the way the definitions say."""
    rng = np.random.default_rng(114)
    d_in, d_out, k = 6, 128, 3
    W = rng.normal(0, 0.01, (d_in, d_out)).astype(np.float32)
    spots = {i: sorted(rng.choice(d_out, k, replace=False)) for i in range(d_in)}
    for i, os_ in spots.items():
        for t, o in enumerate(os_):
            W[i, o] = (1.0 + 0.01 * (i * k + t)) * (-1) ** t
    bits = np.full(d_in, 2, np.uint8)
    planted = sorted(i * d_out + o for i, os_ in spots.items() for o in os_)
    a, _ = orc.weight_outliers_per_channel(W, None, None, bits, k, orc.SCORE_MAGNITUDE)
    b, _ = orc.weight_outliers(W, None, None, bits, k * d_in, orc.SCORE_MAGNITUDE)
    assert list(a) == planted and list(b) == planted
    # channel 0 loses one far entry, channel 1 gains one
    o_from = spots[0][0]
    o_to = next(o for o in range(d_out) if o not in spots[1])
    W2 = W.copy()
    W2[0, o_from] = 0.0
    W2[1, o_to] = 2.0
    a2, _ = orc.weight_outliers_per_channel(W2, None, None, bits, k, orc.SCORE_MAGNITUDE)
    b2, _ = orc.weight_outliers(W2, None, None, bits, k * d_in, orc.SCORE_MAGNITUDE)
    per = lambda idx, i: sum(1 for x in idx if x // d_out == i)
    assert [per(a2, i) for i in range(d_in)] == [k] * d_in            # the count per channel is fixed
    assert per(b2, 1) == k + 1 and 1 * d_out + o_to in b2             # the layer-wide rule follows the values
    assert 1 * d_out + o_to in a2 and per(b2, 0) + per(b2, 1) >= 2 * k - 1


# ----------------------------------------------------------------------------- storage (Sec. 5.1, Fig. 4)

def _unpack(row_words, b, d_out):
    """Independent reader of the packed layout: big Python integer as the bit stream."""
    stream = 0
    for w, word in enumerate(row_words):
        stream |= int(word) << (32 * w)
    return [(stream >> (o * b)) & ((1 << b) - 1) for o in range(d_out)], stream >> (d_out * b)


@pytest.mark.parametrize("d_out", [1, 31, 32, 33, 100, 512])
def test_pack_roundtrip_layout_and_padding(orc, d_out):
    rng = np.random.default_rng(15)
    d_in = 37
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[4, 9]] = orc.PROTECTED
    codes = np.stack([rng.integers(0, 1 << min(int(b), 4), d_out) for b in bits]).astype(np.uint8)
    cent = rng.normal(0, 1, (d_in, 16)).astype(np.float32)
    seen = 0
    for b in (1, 2, 3, 4):
        packed, chan, lut = orc.pack(codes, bits, cent, b)
        want = np.flatnonzero(bits == b)
        assert np.array_equal(chan, want)                          # ascending channel index
        assert packed.shape == (len(want), (d_out * b + 31) // 32)
        for r, i in enumerate(want):
            got, pad = _unpack(packed[r], b, d_out)
            assert got == list(codes[i]) and pad == 0
            assert np.array_equal(lut[r], cent[i, :1 << b].astype(np.float16).view(np.uint16))
        seen += len(want)
    assert seen == d_in - 2                                         # protected channels store no row


def test_storage_overhead_reproduces_printed_example(orc):
    for d, b, lut_bits, kind, printed in _rows("sec5_1_storage_overhead.txt"):
        d, b, lut_bits, printed = int(d), int(b), int(lut_bits), float(printed)
        codes = np.zeros((1, d), np.uint8)
        packed, chan, lut = orc.pack(codes, np.array([b], np.uint8), np.zeros((1, 16), np.float32), b)
        assert packed.size * 32 == d * b                            # payload: exactly b bits per weight
        meta_bits = 4 + lut.shape[1] * lut_bits                     # one 4-bit width + 2^b table entries
        per_weight = meta_bits / d
        if kind == "approx":
            assert lut.dtype == np.uint16 and lut_bits == 16
            assert abs(per_weight - printed) < 0.005 and round(per_weight, 2) == printed
        else:
            assert per_weight < printed


# ----------------------------------------------------------------------------- reconstruction / error

def test_error_is_zero_with_all_outliers_restored(orc):
    rng = np.random.default_rng(16)
    W = rng.normal(0, 1, (9, 70)).astype(np.float16)
    bits = np.full(9, 2, np.uint8)
    cent, codes = orc.kmeans(W, bits, iters=2)
    err, tot = orc.dequant_error(W, cent, codes, bits, np.arange(9 * 70, dtype=np.int64), None)
    assert (err == 0).all() and (tot == 0).all()
    err, tot = orc.dequant_error(W, cent, codes, np.full(9, orc.PROTECTED, np.uint8), None, None)
    assert (err == 0).all()
    # fp32 weights restored through FP16 keep exactly the FP16 rounding error
    W32 = rng.normal(0, 1, (4, 50)).astype(np.float32)
    b4 = np.full(4, 2, np.uint8)
    c, k = orc.kmeans(W32, b4, iters=1)
    err, _ = orc.dequant_error(W32, c, k, b4, np.arange(200, dtype=np.int64), None)
    ref = ((W32.astype(np.float64) - W32.astype(np.float16).astype(np.float64)) ** 2).sum(axis=1)
    assert np.allclose(err, ref, rtol=1e-12)


def test_error_matches_dense_definition_and_delta_y(orc):
    rng = np.random.default_rng(17)
    d_in, d_out, n = 16, 40, 64
    W = rng.normal(0, 1, (d_in, d_out)).astype(np.float32)
    # orthogonal columns: scaled columns of a random orthogonal matrix
    Q, _ = np.linalg.qr(rng.normal(size=(n, d_in)))
    X = (Q * rng.lognormal(0, 1, d_in)).astype(np.float32)
    _, sumsq = orc.act_stats(X)
    bits = rng.integers(2, 4, d_in).astype(np.uint8)
    bits[5] = orc.PROTECTED
    cent, codes = orc.kmeans(W, bits, iters=4)
    out_idx = np.sort(rng.choice(d_in * d_out, 25, replace=False)).astype(np.int64)
    err, tot = orc.dequant_error(W, cent, codes, bits, out_idx, sumsq)
    What = np.take_along_axis(cent.astype(np.float64), codes.astype(np.int64), axis=1)
    w16 = W.astype(np.float16).astype(np.float64)
    What[5] = w16[5]
    What.reshape(-1)[out_idx] = w16.reshape(-1)[out_idx]
    dW = W.astype(np.float64) - What
    assert np.allclose(err, (dW ** 2).sum(axis=1), rtol=1e-12)
    assert np.isclose(tot[1], (dW ** 2).sum(), rtol=1e-12)
    assert np.isclose(tot[0], (sumsq.astype(np.float64)[:, None] * dW ** 2).sum(), rtol=1e-12)
    # App. B.3: Delta Y = X (W - W_hat); for orthogonal columns its squared norm is the weighted sum
    dY = X.astype(np.float64) @ dW
    assert np.isclose(tot[0], (dY ** 2).sum(), rtol=1e-5)


def test_more_levels_never_hurt_and_outlier_removal_helps(orc):
    """End-to-end sanity of the path of Sec. 3.2 on a small layer."""
    rng = np.random.default_rng(18)
    d_in, d_out = 64, 128
    W = rng.normal(0, 0.02, (d_in, d_out)).astype(np.float16)
    W[rng.random(W.shape) < 0.005] = np.float16(0.3)
    X = (rng.normal(0, 1, (96, d_in)) * rng.lognormal(0, 0.5, d_in)).astype(np.float16)
    e = {}
    for b in (2.0, 2.5, 3.0):
        e[b] = orc.quantize_layer(W.copy(), X, (2, 3), b, 4500, 5000, 15)["totals"][0]
    assert e[2.0] > e[2.5] > e[3.0]
    r0 = orc.quantize_layer(W.copy(), X, (2, 3), 2.5, 0, 0, 15)
    r1 = orc.quantize_layer(W.copy(), X, (2, 3), 2.5, 4500, 5000, 15)
    assert r1["totals"][0] < r0["totals"][0]
    assert len(r1["out_idx"]) == orc.count_ppm(5000, d_in * d_out)
    assert r1["chan_mask"].sum() == orc.count_ppm(4500, d_in) == len(r1["act_idx"])
    assert not set(r1["out_idx"] // d_out) & set(r1["act_idx"])


# ------------------------------------------------------------------ Fig. 4: product with the deployed weight

def _deployed_weight(W, cent, codes, bits, out_idx):
    """W_hat of Fig. 4 built with numpy only: FP16 table levels, outliers as FP16 weights."""
    lut = cent.astype(np.float16).astype(np.float64)
    what = np.take_along_axis(lut, codes.astype(np.int64), axis=1)
    w16 = W.astype(np.float16).astype(np.float64)
    keep = np.zeros(W.shape, bool)
    keep[(bits < 1) | (bits > 4), :] = True
    if out_idx is not None and len(out_idx):
        keep.reshape(-1)[out_idx] = True
    return np.where(keep, w16, what)


def test_lut_matvec_hand_example(orc):
    # 2 channels x 2 outputs: channel 0 has two levels {-1, 3}, channel 1 is protected
    W = np.array([[0.3, 2.9], [0.5, -0.25]], np.float32)
    cent = np.zeros((2, 16), np.float32)
    cent[0, :2] = [-1.0, 3.0]
    codes = np.array([[0, 1], [0, 0]], np.uint8)
    bits = np.array([1, orc.PROTECTED], np.uint8)
    X = np.array([[2.0, 4.0], [1.0, 0.0]], np.float32)
    Y = orc.lut_matvec(X, W, cent, codes, bits)
    # y = x0 * level + x1 * w1:  [2*(-1) + 4*0.5, 2*3 + 4*(-0.25)] and [-1, 3]
    assert np.array_equal(Y, np.array([[0.0, 5.0], [-1.0, 3.0]]))
    # entry (0, 0) as an outlier: the weight 0.3 (as FP16) replaces the level -1
    Y = orc.lut_matvec(X, W, cent, codes, bits, out_idx=np.array([0]))
    w = float(np.float16(0.3))
    assert np.allclose(Y, [[2 * w + 2.0, 5.0], [w, 3.0]], rtol=0, atol=1e-15)


def test_lut_matvec_equals_dense_product_with_rebuilt_weight(orc):
    rng = np.random.default_rng(31)
    d_in, d_out, m = 45, 70, 3
    W = rng.normal(0, 0.05, (d_in, d_out)).astype(np.float16)
    X = rng.normal(0, 1, (m, d_in)).astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[3, 30]] = orc.PROTECTED
    cent, codes = orc.kmeans(W, bits, iters=4)
    out_idx = np.sort(rng.choice(d_in * d_out, 60, replace=False))
    out_idx = out_idx[~np.isin(out_idx // d_out, [3, 30])]
    for oi in (None, out_idx):
        Y = orc.lut_matvec(X, W, cent, codes, bits, oi)
        ref = X.astype(np.float64) @ _deployed_weight(W, cent, codes, bits, oi)
        assert np.allclose(Y, ref, rtol=1e-13, atol=1e-13)
    # every entry restored: the product with the FP16 weight itself
    all_prot = np.full(d_in, orc.PROTECTED, np.uint8)
    Y = orc.lut_matvec(X, W, cent, codes, all_prot)
    assert np.allclose(Y, X.astype(np.float64) @ W.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_lut_matvec_agrees_with_the_packed_format(orc):
    """The product computed from the stored streams (unpacked here bit by bit, Sec. 5.1) equals the
    product computed from codes and levels: packing loses nothing the kernel needs."""
    rng = np.random.default_rng(32)
    d_in, d_out = 29, 50
    W = rng.normal(0, 0.05, (d_in, d_out)).astype(np.float32)
    x = rng.normal(0, 1, (1, d_in)).astype(np.float32)
    bits = rng.integers(2, 5, d_in).astype(np.uint8)
    cent, codes = orc.kmeans(W, bits, iters=3)
    y = np.zeros(d_out)
    for b in (2, 3, 4):
        packed, chan, lut = orc.pack(codes, bits, cent, b)
        for r, i in enumerate(chan):
            row_codes, _ = _unpack(packed[r], b, d_out)
            y += float(x[0, i]) * lut[r].view(np.float16).astype(np.float64)[row_codes]
    assert np.allclose(orc.lut_matvec(x, W, cent, codes, bits)[0], y, rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ Tab. 13: other norms as the statistic

def test_act_stats_other_norms_match_numpy_and_chunking(orc):
    rng = np.random.default_rng(41)
    X = (rng.normal(0, 1, (300, 37)) * np.exp(rng.normal(0, 1, 37))).astype(np.float16)
    X64 = X.astype(np.float64)
    want = {0: (X64 ** 2).sum(0), 1: np.abs(X64).sum(0), 2: np.abs(X64).max(0)}
    for norm, ref in want.items():
        acc, stat = orc.act_stats_norm(X, norm)
        assert np.allclose(acc, ref, rtol=1e-14, atol=0)
        assert np.array_equal(stat, acc.astype(np.float32))
        a1, _ = orc.act_stats_norm(X[:111], norm)                 # tokens arriving in two chunks
        a2, _ = orc.act_stats_norm(X[111:], norm, acc=a1)
        assert np.allclose(a2, ref, rtol=1e-14, atol=0)
    assert np.array_equal(orc.act_stats_norm(X, 0)[0], orc.act_stats(X)[0])
    # the norms are different criteria: one spike outranks a steady channel only under l-infinity
    Y = np.zeros((100, 2), np.float32)
    Y[:, 0] = 1.0
    Y[7, 1] = 5.0
    s2, s1, si = (orc.act_stats_norm(Y, k)[1] for k in (0, 1, 2))
    assert s2[0] > s2[1] and s1[0] > s1[1] and si[1] > si[0]
    # a channel that holds a NaN (or an infinity) comes out non-finite under every norm, also
    # when the bad token arrives in an earlier chunk; the other channels are untouched
    for bad in (np.nan, np.inf):
        Z = Y.copy()
        Z[3, 1] = bad
        for norm in (0, 1, 2):
            acc = orc.act_stats_norm(Z, norm)[0]
            assert not np.isfinite(acc[1]) and acc[0] == orc.act_stats_norm(Y, norm)[0][0]
            a1 = orc.act_stats_norm(Z[:50], norm)[0]
            assert not np.isfinite(orc.act_stats_norm(Z[50:], norm, acc=a1)[0][1])


# ----------------------------------------------------------------------------- App. A.2: uniform quantizer

def test_rtn_hand_examples(orc):
    """Sec. 3, uniform quantizer: a ramp 0..7 at 3 bits has Delta = 1 and is its own code; the
    same ramp shifted to 8..15 at 2 bits has Delta = 7/3 and the codes worked out by hand
    (quotients 0, .43, .86, 1.29, 1.71, 2.14, 2.57, 3)."""
    W = np.arange(16, dtype=np.float32).reshape(2, 8)
    codes, scale, zero, err = orc.rtn_quantize(W, np.array([3, 2], np.uint8), group=8)
    assert codes[0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert codes[1].tolist() == [0, 0, 1, 1, 2, 2, 3, 3]
    assert scale[:, 0].tolist() == [1.0, np.float32(7) / np.float32(3)] and zero[:, 0].tolist() == [0.0, 8.0]
    assert err[0] == 0.0
    # row 1: distances to the levels 8, 10.33, 12.67, 15 are 0, 1, 1/3, 2/3, 2/3, 1/3, 1, 0
    assert abs(err[1] - (2 * 1.0 + 2 * (1 / 9) + 2 * (4 / 9))) < 1e-6


def test_rtn_code_is_the_nearest_level_and_error_is_within_half_a_step(orc):
    """Sec. 3: round-to-nearest on a uniform grid is the nearest of the 2^N levels
    min + k Delta (checked by brute force over the levels in fp64), so no weight moves by
    more than Delta / 2, and the ends of the range are kept exactly."""
    rng = np.random.default_rng(3)
    for N in (1, 2, 3, 4):
        W = (rng.standard_t(4, size=(6, 300)) * 0.02).astype(np.float16)
        bits = np.full(6, N, np.uint8)
        codes, scale, zero, err = orc.rtn_quantize(W, bits, group=128)
        assert scale.shape == (6, 3)
        w = W.astype(np.float64)
        for i in range(6):
            for g in range(3):
                sl = slice(128 * g, min(300, 128 * (g + 1)))
                lo, d = float(zero[i, g]), float(scale[i, g])
                assert lo == w[i, sl].min() and codes[i, sl].max() == 2 ** N - 1 and codes[i, sl].min() == 0
                levels = lo + d * np.arange(2 ** N)
                dist = np.abs(w[i, sl][:, None] - levels[None, :])
                best = dist.min(axis=1)
                mine = dist[np.arange(dist.shape[0]), codes[i, sl]]
                assert np.all(mine <= best + 1e-6 * d)          # nearest, up to a rounding of the quotient
                assert np.all(mine <= d / 2 * (1 + 1e-6))
                assert abs(levels[-1] - w[i, sl].max()) <= 1e-6 * max(abs(levels[-1]), d)
            rebuilt = np.concatenate([float(zero[i, g]) + float(scale[i, g]) * codes[i, 128 * g:128 * (g + 1)]
                                      for g in range(3)])
            assert abs(err[i] - np.sum((w[i] - rebuilt) ** 2)) <= 1e-12 * max(err[i], 1e-30)


def test_rtn_groups_are_independent_and_ragged_tail_is_its_own_group(orc):
    """App. A.2: group-wise ranges.  Two groups of very different spread must each use their
    own step; a quantizer that ignored the group boundary would give the narrow group one
    code only."""
    rng = np.random.default_rng(5)
    wide = rng.uniform(-8, 8, 128)
    narrow = rng.uniform(-0.01, 0.01, 40)                     # a ragged last group of 40
    W = np.concatenate([wide, narrow])[None, :].astype(np.float32)
    codes, scale, zero, _ = orc.rtn_quantize(W, np.array([4], np.uint8), group=128)
    assert scale.shape == (1, 2) and scale[0, 0] > 100 * scale[0, 1] > 0
    assert len(set(codes[0, 128:].tolist())) > 8               # the narrow group uses its own 16 levels
    alone = orc.rtn_quantize(W[:, 128:].copy(), np.array([4], np.uint8), group=128)
    assert np.array_equal(alone[0][0], codes[0, 128:]) and alone[1][0, 0] == scale[0, 1]


def test_rtn_invariances_and_degenerate_groups(orc):
    """Facts any min/max uniform quantizer obeys: scaling by a power of two keeps the codes
    and scales Delta (and the error by its square); quantizing the rebuilt weights again
    changes nothing; codes are monotone in the weight; a constant group has Delta = 0 and is
    exact; channels kept in FP16 get no codes and only the FP16 rounding error."""
    rng = np.random.default_rng(7)
    W = rng.normal(0, 0.05, size=(5, 256)).astype(np.float32)
    W[3, :128] = 0.125                                          # a constant group
    bits = np.array([2, 3, 4, 3, 16], np.uint8)
    codes, scale, zero, err = orc.rtn_quantize(W, bits, group=128)
    c4, s4, z4, e4 = orc.rtn_quantize(W * 4, bits, group=128)
    assert np.array_equal(c4, codes) and np.array_equal(s4, scale * 4) and np.array_equal(z4, zero * 4)
    assert np.allclose(e4[:4], err[:4] * 16, rtol=1e-12)
    assert scale[3, 0] == 0 and zero[3, 0] == np.float32(0.125) and not codes[3, :128].any()
    assert not codes[4].any() and not scale[4].any()
    w16 = W[4].astype(np.float16).astype(np.float64)
    assert abs(err[4] - np.sum((W[4].astype(np.float64) - w16) ** 2)) <= 1e-12 * err[4]
    for i in range(4):
        for g in range(2):
            sl = slice(128 * g, 128 * (g + 1))
            order = np.argsort(W[i, sl], kind="stable")
            assert np.all(np.diff(codes[i, sl][order].astype(int)) >= 0)
    rebuilt = np.zeros_like(W)
    for g in range(2):
        sl = slice(128 * g, 128 * (g + 1))
        rebuilt[:, sl] = (zero[:, g:g + 1].astype(np.float64) + scale[:, g:g + 1].astype(np.float64) * codes[:, sl]).astype(np.float32)
    again = orc.rtn_quantize(rebuilt, bits, group=128)
    assert (again[0][:4] != codes[:4]).mean() < 1e-3           # fp32 rounding of a rebuilt level may flip a tie
    assert np.all(again[3][:4] <= 1e-10 + 1e-3 * err[:4])


def test_rtn_more_bits_never_hurt_and_kmeans_is_no_worse_on_heavy_tails(orc):
    """App. A.2 / Tab. 10: the uniform grid wastes levels on heavy-tailed weights, so the
    K-means levels of Sec. 3.2.1 give a smaller error at the same width; and for either
    quantizer the error falls as the width grows."""
    rng = np.random.default_rng(11)
    W = (rng.standard_t(3, size=(4, 512)) * 0.02).astype(np.float16)
    prev = None
    for N in (2, 3, 4):
        bits = np.full(4, N, np.uint8)
        e_rtn = orc.rtn_quantize(W, bits, group=512)[3]
        cent, codes = orc.kmeans(W, bits, iters=20)
        e_km = orc.dequant_error(W, cent, codes, bits)[0]
        assert np.all(e_km < e_rtn)
        if prev is not None:
            assert np.all(e_rtn < prev)
        prev = e_rtn


# ----------------------------------------------------------------------------- Sec. 5.1 / Tab. 7: 4-bit tables

def test_lut4_hand_example_and_textbook_properties(orc):
    """One uniform 16-level grid per layer (Sec. 3's quantizer with N = 4 over all centres): a
    table that already lies on such a grid is kept exactly; otherwise no centre moves by more
    than half a step, the smallest and largest centre of the layer are kept, codes are
    monotone in the centre, unused slots and FP16 channels stay +infinity, and doing it again
    changes nothing."""
    cent = np.full((3, 16), np.inf, np.float32)
    cent[0, :4] = [-1.5, -0.5, 0.5, 1.5]                       # a 2-bit channel on the grid -1.5 + 0.2 k
    cent[1, :8] = np.array([-1.5, -1.1, -0.7, -0.3, 0.1, 0.5, 0.9, 1.3], np.float32)
    cent[2, :4] = [7, 8, 9, 10]                                # a channel kept in FP16: ignored
    bits = np.array([2, 3, 16], np.uint8)
    codes4, rng, cq = orc.lut4(cent, bits)
    assert rng[0] == np.float32(-1.5) and abs(rng[1] - 0.2) < 1e-7
    assert codes4[0, :4].tolist() == [0, 5, 10, 15] and codes4[1, :8].tolist() == [0, 2, 4, 6, 8, 10, 12, 14]
    assert np.allclose(cq[0, :4], cent[0, :4], atol=1e-6) and np.allclose(cq[1, :8], cent[1, :8], atol=1e-6)
    assert np.all(np.isposinf(cq[0, 4:])) and np.all(np.isposinf(cq[2])) and not codes4[2].any()

    r = np.random.default_rng(3)
    cent = np.full((40, 16), np.inf, np.float32)
    bits = r.choice(np.array([1, 2, 3, 4, 16], np.uint8), 40)
    for i, b in enumerate(bits):
        if b <= 4:
            cent[i, :1 << b] = np.sort(r.normal(0, 0.03, 1 << b)).astype(np.float32)
    codes4, rng, cq = orc.lut4(cent, bits)
    live = np.isfinite(cq)
    assert np.array_equal(live, np.isfinite(cent) & (bits[:, None] <= 4))
    step = float(rng[1])
    assert np.all(np.abs(cq[live].astype(np.float64) - cent[live]) <= step / 2 * (1 + 1e-5))
    assert cq[live].min() == cent[live].min() and abs(cq[live].max() - cent[live].max()) <= 1e-6 * step
    assert codes4[live].min() == 0 and codes4[live].max() == 15
    order = np.argsort(cent[live], kind="stable")
    assert np.all(np.diff(codes4[live][order].astype(int)) >= 0)
    again = orc.lut4(cq, bits)
    assert np.array_equal(again[0], codes4) and np.allclose(again[2][live], cq[live], rtol=0, atol=1e-4 * step)
    # a layer whose centres all coincide, and a layer without quantized channels
    same = np.full((2, 16), np.inf, np.float32)
    same[:, :4] = 0.25
    c, g, q = orc.lut4(same, np.array([2, 2], np.uint8))
    assert g.tolist() == [0.25, 0.0] and not c.any() and np.all(q[:, :4] == 0.25)
    c, g, q = orc.lut4(same, np.array([16, 16], np.uint8))
    assert g.tolist() == [0.0, 0.0] and np.all(np.isposinf(q))


def test_lut4_costs_little_error_on_a_quantized_layer(orc):
    """Tab. 7 reports a small loss from 4-bit tables.  On a layer whose channels share one
    scale the 16-level grid moves every level by at most half a step of the layer's range / 15,
    so the reconstruction error grows, but stays far below that of dropping one bit of width."""
    r = np.random.default_rng(5)
    W = (r.standard_t(5, size=(24, 512)) * 0.02).astype(np.float16)
    bits3, bits2 = np.full(24, 3, np.uint8), np.full(24, 2, np.uint8)
    cent, codes = orc.kmeans(W, bits3, iters=10)
    e16 = orc.dequant_error(W, cent, codes, bits3)[1][1]
    _, _, cq = orc.lut4(cent, bits3)
    e4 = orc.dequant_error(W, cq, codes, bits3)[1][1]
    cent2, codes2 = orc.kmeans(W, bits2, iters=10)
    e_2bit = orc.dequant_error(W, cent2, codes2, bits2)[1][1]
    assert e16 <= e4 < e_2bit


def _heavy_tailed_quantized_layer(orc, d_in=48, d_out=1024, seed=6):
    """A layer in the image of the synthetic workloads (narrow Gaussian bulk, 0.5 % of the entries
    from a heavy tail), widths 2..4, quantized by the oracle."""
    r = np.random.default_rng(seed)
    W = r.normal(0, 0.02, (d_in, d_out))
    tail = r.random(W.shape) < 0.005
    W[tail] = 0.1 * r.standard_t(3, size=int(tail.sum()))
    W = W.astype(np.float16)
    bits = r.choice(np.array([2, 3, 4], np.uint8), d_in)
    cent, codes = orc.kmeans(W, bits, iters=20)
    return W, bits, cent, codes


def test_lut4_codebook_is_a_16_level_table_per_layer(orc):
    """Sec. 5.1 / Tab. 7, the storage side: after the call every table entry of the layer is one
    of at most 16 FP16 values (4 bits per entry, nothing per channel: the printed (1*4 + 8*4)/4096
    for a 3-bit channel of 4096 outputs, below 0.01 bit per weight), codes4 names it, unused
    slots and FP16 channels stay +infinity."""
    W, bits, cent, codes = _heavy_tailed_quantized_layer(orc)
    bits[5] = orc.PROTECTED
    cent[5] = np.inf
    codes4, table, cq = orc.lut4_codebook(cent, bits)
    K = np.where(bits <= 4, 1 << np.minimum(bits, 4).astype(int), 0)
    used = np.arange(16)[None, :] < K[:, None]
    assert np.array_equal(np.isfinite(cq), used) and not codes4[~used].any()
    table16 = table.astype(np.float16).astype(np.float32)                 # the stored FP16 table
    assert np.array_equal(cq[used], table16[codes4[used]])
    assert len(np.unique(cq[used])) <= 16
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sec5_1_storage_overhead.txt")) if not l.startswith("#")]
    d, b, entry_bits, kind, printed = next(r for r in rows if r[2] == "4")
    per_weight = (1 * 4 + (1 << int(b)) * int(entry_bits)) / int(d)
    assert kind == "below" and per_weight < float(printed)
    layer_table_bits = 16 * 16                                            # one FP16 table per layer
    assert layer_table_bits / (int(d) * int(d)) < 1e-4                    # does not change the figure


def test_lut4_codebook_is_lloyds_algorithm_on_the_fp16_centres(orc):
    """The clustering side, against numpy: every code is the nearest table level in exact
    arithmetic (ties to the smaller index); run to convergence, every level with members is
    the mean of its members (Lloyd's fixed point); the squared error over the centres is at
    least the optimum of the exact 1-D dynamic programme and reaches it on planted groups."""
    r = np.random.default_rng(9)
    cent = np.full((30, 16), np.inf, np.float32)
    bits = r.choice(np.array([1, 2, 3, 16], np.uint8), 30)
    for i, b in enumerate(bits):
        if b <= 4:
            cent[i, :1 << b] = np.sort(r.standard_t(3, 1 << b) * 0.03).astype(np.float32)
    codes4, table, cq = orc.lut4_codebook(cent, bits, iters=200)
    used = np.isfinite(cq)
    v = cent[used].astype(np.float16).astype(np.float64)
    c = codes4[used]
    d = np.abs(v[:, None] - table.astype(np.float64)[None, :])
    assert np.array_equal(c, d.argmin(1))                                 # argmin takes the first of equals
    for j in range(16):
        if (c == j).any():
            assert table[j] == np.float32(v[c == j].mean())
    sse = float(((v - table.astype(np.float64)[c]) ** 2).sum())
    assert sse >= _optimal_sse(v, 16) * (1 - 1e-9) - 1e-18
    # 16 well separated groups of equal size: the optimum, whatever the channel they sit in
    centres = np.arange(16) * 1.0 - 7.5
    vals = (centres[:, None] + r.normal(0, 1e-3, (16, 8))).astype(np.float16).astype(np.float32)
    flat = r.permutation(vals.reshape(-1))
    cent = flat.reshape(8, 16)
    _, table, cq = orc.lut4_codebook(cent, np.full(8, 4, np.uint8), iters=10)
    assert np.allclose(np.sort(table), vals.astype(np.float64).mean(1), rtol=0, atol=1e-6)
    # a layer whose channels share one 16-level table keeps it exactly; no quantized channel: zeros
    one = np.sort(r.normal(0, 0.05, 16)).astype(np.float16).astype(np.float32)
    same = np.tile(one, (11, 1))
    c4, table, cq = orc.lut4_codebook(same, np.full(11, 4, np.uint8))
    assert np.array_equal(cq, same) and np.array_equal(table, one) and np.array_equal(c4, np.tile(np.arange(16), (11, 1)))
    c4, table, cq = orc.lut4_codebook(same, np.full(11, 16, np.uint8))
    assert not table.any() and not c4.any() and np.all(np.isposinf(cq))


def test_lut4_codebook_costs_what_tab7_says_where_the_uniform_grid_does_not(orc):
    """Tab. 7: 4-bit centres cost at most 1.5 % (perplexity).  On a heavy-tailed layer the
    per-layer table keeps the reconstruction error within a factor 1.5 of the FP16 tables' and
    far below that of one bit less per weight, while the uniform 16-level grid - whose step is
    set by the few far centres - multiplies it many times over."""
    W, bits, cent, codes = _heavy_tailed_quantized_layer(orc)
    e16 = orc.dequant_error(W, cent, codes, bits)[1][1]
    e4 = orc.dequant_error(W, orc.lut4_codebook(cent, bits)[2], codes, bits)[1][1]
    e4_uniform = orc.dequant_error(W, orc.lut4(cent, bits)[2], codes, bits)[1][1]
    less = np.maximum(bits - 1, 1).astype(np.uint8)
    cl, kl = orc.kmeans(W, less, iters=20)
    e_less = orc.dequant_error(W, cl, kl, less)[1][1]
    assert e16 * (1 - 1e-3) <= e4 <= 1.5 * e16
    assert e4 < e_less
    assert e4_uniform > 10 * e16 and e4_uniform > 10 * e4


# ------------------------------------------------------------------ K-means from given levels (variant)

def test_kmeans_from_given_levels_continues_the_same_iteration(orc):
    """r rounds from the quantile start, then s more from where they ended, are r + s rounds:
    the given-start path is the cold path (pinned above) entered later.  0 rounds return the
    start itself, so the quantile levels are available to start from."""
    rng = np.random.default_rng(77)
    W = rng.normal(0, 0.05, (9, 300)).astype(np.float16)
    W[3, :40] = W[3, 0]                                   # ties and a short run of equal values
    bits = np.array([1, 2, 3, 4, 2, 3, 4, 16, 4], np.uint8)
    excl = np.sort(rng.choice(9 * 300, 60, replace=False)).astype(np.int64)
    for oi in (None, excl):
        c0, k0 = orc.kmeans(W, bits, out_idx=oi, iters=0)
        c7, k7 = orc.kmeans(W, bits, out_idx=oi, iters=7)
        g0, h0 = orc.kmeans(W, bits, out_idx=oi, iters=0, start=c0)
        assert np.array_equal(g0, c0) and np.array_equal(h0, k0)
        g7, h7 = orc.kmeans(W, bits, out_idx=oi, iters=7, start=c0)
        assert np.array_equal(g7, c7) and np.array_equal(h7, k7)
        c3, _ = orc.kmeans(W, bits, out_idx=oi, iters=3)
        g4, h4 = orc.kmeans(W, bits, out_idx=oi, iters=4, start=c3)
        assert np.array_equal(g4, c7) and np.array_equal(h4, k7)


def test_kmeans_from_given_levels_keeps_level_indices_and_fixed_points(orc):
    """Level j stays level j: a permuted start gives the permuted result.  A start that is a
    fixed point (levels = means of their own cells) comes back unchanged after any number of
    rounds.  The objective never rises from one round to the next."""
    rng = np.random.default_rng(78)
    x = np.concatenate([rng.normal(m, 0.01, 50) for m in (-0.3, -0.1, 0.2, 0.5)]).astype(np.float32)
    W = x[None, :]
    bits = np.array([2], np.uint8)
    c, k = orc.kmeans(W, bits, iters=30)                  # well separated: converged long before
    again, k2 = orc.kmeans(W, bits, iters=5, start=c)
    assert np.array_equal(again, c) and np.array_equal(k2, k)
    perm = np.array([2, 0, 3, 1])
    start = c.copy()
    start[0, :4] = c[0, perm]
    cp, kp = orc.kmeans(W, bits, iters=5, start=start)
    assert np.array_equal(cp[0, :4], c[0, perm])
    assert np.array_equal(perm[kp[0]], k[0])              # code j of the permuted run is level perm[j]
    rough = np.full((1, 16), np.inf, np.float32)
    rough[0, :4] = [-1.0, 0.0, 0.01, 1.0]
    _, _, sse = orc.kmeans(W, bits, iters=12, start=rough, trace=True)
    assert (np.diff(sse[0]) <= 1e-12 * sse[0, 0]).all() and sse[0, -1] < sse[0, 0]
    # a level that gets no member keeps the value it was given; -0 is taken as +0
    lone = np.full((1, 16), np.inf, np.float32)
    lone[0, :4] = [-0.0, 100.0, -0.3, 0.3]
    cl, kl = orc.kmeans(W, bits, iters=3, start=lone)
    assert cl[0, 1] == 100.0 and not (kl == 1).any()
    z, _ = orc.kmeans(W, bits, iters=0, start=lone)
    assert z[0, 0] == 0.0 and not np.signbit(z[0, 0])


def test_whole_path_with_final_levels_started_from_the_preliminary_ones(orc):
    """The variant of the whole path: same O_act, widths, preliminary quantization and O_q as the
    default; the final levels are those of K-means started at the preliminary levels."""
    rng = np.random.default_rng(79)
    W = rng.normal(0, 0.02, (40, 256)).astype(np.float16)
    X = rng.normal(0, 1, (64, 40)).astype(np.float16)
    a = orc.quantize_layer(W, X, (2, 3, 4), 3.0, 45000, 10000, iters=6)
    b = orc.quantize_layer(W, X, (2, 3, 4), 3.0, 45000, 10000, iters=6, iters_final_from_prelim=4)
    for f in ("act_idx", "bits", "cent1", "codes1", "out_idx", "out_val"):
        assert np.array_equal(a[f], b[f]), f
    want, wk = orc.kmeans(W, a["bits"], out_idx=a["out_idx"], iters=4, start=a["cent1"])
    assert np.array_equal(b["centroids"], want) and np.array_equal(b["codes"], wk)
