"""GPU-vs-oracle parity of every step of the path, element by element, through the C ABI.

Bars (stated where used): integer outputs - bits, outlier index sets and values, codes
given identical levels, packed words - are bit-exact.  Levels agree within 1e-5 relative
(they are in fact bit-identical for fp16 inputs, whose fp64 sums are exact); per-layer
activation-weighted error within 1e-4 relative; the activation statistic within 1e-5
relative of the fp64 oracle (observed: ~1e-15).
"""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.fixture(scope="module")
def env(orc):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_13056_amd import binding as B, pipeline as P, synth
    B.lib()                                   # fails loudly when the library has not been built
    return dict(B=B, P=P, synth=synth, ws=B.Workspace(DEV), orc=orc)


def _np(t):
    return t.detach().cpu().numpy()


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.to(DEV) if dtype is None else t.to(DEV).to(dtype)


def _rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    fin = np.isfinite(a) & np.isfinite(b)
    assert np.array_equal(np.isfinite(a), np.isfinite(b))
    if not fin.any():
        return 0.0
    den = np.maximum(np.abs(b[fin]), 1e-30)
    return float(np.max(np.abs(a[fin] - b[fin]) / den))


# ------------------------------------------------------------------ statistics

@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("n,d_in", [(1, 8), (7, 77), (300, 512), (1031, 1000), (4096, 1536), (33, 8200)])
def test_act_stats_parity(env, dtype, n, d_in):
    rng = np.random.default_rng(n * 131 + d_in)
    X = (rng.normal(0, 1, (n, d_in)) * rng.lognormal(0, 1, d_in)).astype(dtype)
    acc, sumsq = env["P"].activation_stats(_dev(X), env["ws"])
    oacc, osum = env["orc"].act_stats(X)
    assert _rel(_np(acc), oacc) < 1e-12
    assert _rel(_np(sumsq), osum) <= 1e-5          # the stated bar; in practice bit-identical
    assert np.array_equal(_np(sumsq), osum)


def test_act_stats_strided_chunked_empty_and_status(env):
    B, P, ws, orc = env["B"], env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(0)
    big = rng.normal(0, 2, (500, 640)).astype(np.float16)
    Xd = _dev(big)[:, 64:64 + 264]                  # leading dimension 640 > d_in, 16-byte aligned start
    acc, sumsq = P.activation_stats(Xd, ws)
    oacc, _ = orc.act_stats(big[:, 64:64 + 264])
    assert _rel(_np(acc), oacc) < 1e-12
    Xo = _dev(big)[:, 3:3 + 100]                    # odd offset: the unaligned path
    acc, _ = P.activation_stats(Xo, ws)
    assert _rel(_np(acc), orc.act_stats(big[:, 3:103])[0]) < 1e-12
    # tokens arriving in chunks give the one-shot result
    full = _dev(big)
    a1, _ = P.activation_stats(full[:123], ws)
    a2, s2 = P.activation_stats(full[123:], ws, acc=a1)
    a0, s0 = P.activation_stats(full, ws)
    assert _rel(_np(a2), _np(a0)) < 1e-13 and np.array_equal(_np(s2), _np(s0))
    # no tokens: accumulator untouched when adding, zero when starting
    a3 = a0.clone()
    B.act_stats(full[:0], a3, None, True, ws)
    assert torch.equal(a3, a0)
    B.act_stats(full[:0], a3, None, False, ws)
    assert (a3 == 0).all()
    # NaN / infinity in X raises the status flag
    bad = big.copy()
    bad[17, 5] = np.inf
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    P.activation_stats(_dev(bad), ws, status=st)
    assert st.item() & B.STATUS_NONFINITE
    st.zero_()
    P.activation_stats(full, ws, status=st)
    assert st.item() == 0


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("norm", [0, 1, 2])
def test_act_stats_other_norms_parity(env, dtype, norm):
    """Tab. 13: l2 (squared), l1 and l-infinity statistics, in two chunks of tokens.  Sums of
    magnitudes and maxima of fp16 inputs are exact in fp64: compared bit for bit.  Squares, and
    fp32 inputs, within 1e-12 relative (the order of the fp64 additions differs)."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(17 + norm)
    n, d_in = 777, 1000 + 8
    X = (rng.normal(0, 1, (n, d_in)) * np.exp(rng.normal(0, 1, d_in))).astype(dtype)
    Xd = _dev(X)
    acc = torch.empty(d_in, dtype=torch.float64, device=DEV)
    stat = torch.empty(d_in, dtype=torch.float32, device=DEV)
    B.act_stats_norm(Xd[:300], norm, acc, stat, False, ws)
    B.act_stats_norm(Xd[300:], norm, acc, stat, True, ws)
    oacc, ostat = orc.act_stats_norm(X, norm)
    if dtype == np.float16 and norm != 0:
        assert np.array_equal(_np(acc), oacc) and np.array_equal(_np(stat), ostat)
    else:
        assert _rel(_np(acc), oacc) <= 1e-12 and _rel(_np(stat), ostat) <= 1e-6
    # the statistic drives the same ranking calls
    k = 9
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    mask = torch.empty(d_in, dtype=torch.uint8, device=DEV)
    B.extract_channel_outliers(stat, k, idx, mask, ws)
    assert np.array_equal(_np(idx), orc.top_channels(_np(stat), k)[0])        # same input on both sides


@pytest.mark.parametrize("norm", [0, 1, 2])
@pytest.mark.parametrize("bad", [np.nan, np.inf])
def test_act_stats_norms_flag_nonfinite_input(env, norm, bad):
    """A NaN or an infinity in X raises the status flag under every norm (a maximum must not
    drop the NaN), in the first chunk of tokens or a later one, on the aligned and the unaligned
    kernel; the flag stays clear on finite input."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(5)
    X = rng.normal(0, 1, (200, 256)).astype(np.float16)
    for cols in (slice(0, 256), slice(3, 103)):
        Z = X.copy()
        Z[150, 40] = bad
        Zd = _dev(Z)[:, cols]
        d_in = Zd.shape[1]
        for split in (0, 100, 180):
            acc = torch.empty(d_in, dtype=torch.float64, device=DEV)
            st = torch.zeros(1, dtype=torch.int32, device=DEV)
            if split:
                B.act_stats_norm(Zd[:split], norm, acc, None, False, ws, st)
            B.act_stats_norm(Zd[split:], norm, acc, None, bool(split), ws, st)
            assert st.item() & B.STATUS_NONFINITE
            oacc = orc.act_stats_norm(Z[:, cols], norm)[0]
            assert np.array_equal(np.isfinite(_np(acc)), np.isfinite(oacc))
        st = torch.zeros(1, dtype=torch.int32, device=DEV)
        acc = torch.empty(d_in, dtype=torch.float64, device=DEV)
        B.act_stats_norm(_dev(X)[:, cols], norm, acc, None, False, ws, st)
        assert st.item() == 0


def test_act_stats_is_reproducible(env):
    X = env["synth"].make_activations(20000, 2048, "f16", 5, DEV)
    a1, _ = env["P"].activation_stats(X, env["ws"])
    a2, _ = env["P"].activation_stats(X, env["ws"])
    assert torch.equal(a1, a2)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("rows,cols", [(1, 1), (64, 64), (65, 63), (512, 256), (1000, 3), (7, 900), (100, 260), (4, 8), (68, 4), (1024, 8192)])
def test_transpose(env, dtype, rows, cols):
    src = torch.randn(rows, cols, device=DEV).to(dtype)
    dst = torch.empty(cols, rows, dtype=dtype, device=DEV)
    env["B"].transpose(src, dst)
    assert torch.equal(dst, src.t().contiguous())
    wide = torch.zeros(cols, rows + 5, dtype=dtype, device=DEV)
    env["B"].transpose(src, wide[:, :rows])          # leading dimension of dst > rows
    assert torch.equal(wide[:, :rows], src.t()) and (wide[:, rows:] == 0).all()


# ------------------------------------------------------------------ rankings

@pytest.mark.parametrize("d_in", [1, 5, 256, 1000, 4096, 28672])
def test_channel_outliers_and_allocation_parity(env, d_in):
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in)
    s = rng.lognormal(0, 1, d_in).astype(np.float32)
    if d_in > 4:
        s[rng.integers(0, d_in, d_in // 5)] = s[0]          # exact ties
        s[rng.integers(0, d_in, 3)] = 0.0
    sd = _dev(s)
    for k in sorted({0, 1, B.count_ppm(4500, d_in), d_in // 3, d_in}):
        idx = torch.full((max(k, 1),), -7, dtype=torch.int32, device=DEV)
        mask = torch.empty(d_in, dtype=torch.uint8, device=DEV)
        B.extract_channel_outliers(sd, k, idx, mask, ws)
        oidx, omask = orc.top_channels(s, k)
        assert np.array_equal(_np(idx)[:k], oidx) and np.array_equal(_np(mask), omask)
        for bit_set in ((2, 3), (2, 3, 4), (1, 2, 3, 4)):
            for b in (bit_set[0], bit_set[0] + 0.2, 2.5, 3.0, bit_set[-1] - 0.37, bit_set[-1]):
                if not bit_set[0] <= b <= bit_set[-1]:
                    continue
                bits = torch.empty(d_in, dtype=torch.uint8, device=DEV)
                counts = B.allocate_bits(sd, mask, k, bit_set, b, bits, ws)
                obits, ocounts = orc.allocate_bits(s, omask, bit_set, b)
                assert np.array_equal(_np(bits), obits), (d_in, k, bit_set, b)
                assert counts == list(ocounts)
    bits = torch.empty(d_in, dtype=torch.uint8, device=DEV)          # no mask at all
    B.allocate_bits(sd, None, 0, (2, 3, 4), 3.3, bits, ws)
    assert np.array_equal(_np(bits), orc.allocate_bits(s, None, (2, 3, 4), 3.3)[0])


# ------------------------------------------------------------------ k-means

def _kmeans_gpu(env, W, bits, out_idx=None, ew=None, iters=20, status=None, start=None, algorithm=None):
    B, ws = env["B"], env["ws"]
    Wd = _dev(W)
    d_in, d_out = W.shape
    if start is None:
        cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV)
    else:
        cent = _dev(np.ascontiguousarray(start, np.float32))
    codes = torch.full((d_in, d_out), 255, dtype=torch.uint8, device=DEV)
    oi = None if out_idx is None else _dev(out_idx.astype(np.int32))
    B.kmeans_quantize(Wd, _dev(bits), oi, 0 if out_idx is None else len(out_idx),
                      None if ew is None else _dev(ew), iters, cent, codes, ws, status,
                      init=B.INIT_QUANTILE if start is None else B.INIT_GIVEN, algorithm=algorithm)
    return _np(cent), _np(codes)


def _check_kmeans(cent, codes, ocent, ocodes, exact):
    if exact:
        assert np.array_equal(cent, ocent)
        assert np.array_equal(codes, ocodes)
    else:
        assert _rel(cent, ocent) <= 1e-5                       # bar on levels
        assert (codes != ocodes).mean() <= 1e-4                # bar on assignments


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("d_out", [1, 2, 63, 64, 257, 1000, 4096 + 7])
def test_kmeans_parity_ragged_sizes(env, dtype, d_out):
    rng = np.random.default_rng(d_out)
    d_in = 40
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 15
    W = W.astype(dtype)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[3, 17]] = 16
    bits[5] = 0
    cent, codes = _kmeans_gpu(env, W, bits, iters=12)
    ocent, ocodes = env["orc"].kmeans(W, bits, iters=12)
    _check_kmeans(cent, codes, ocent, ocodes, exact=dtype == np.float16)


def test_kmeans_parity_degenerate_channels(env):
    rng = np.random.default_rng(1)
    d_in, d_out = 24, 300
    W = rng.normal(0, 1, (d_in, d_out)).astype(np.float16)
    W[0, :] = W[0, 0]                                   # one distinct value
    W[1, 50:] = 0.0                                     # most of the channel equal: duplicate starts
    W[2, :] = np.float16(-0.0)
    W[3, ::2] = np.float16(-0.0)
    W[3, 1::2] = np.float16(0.0)
    W[4] = np.repeat(np.array([-1, 0.5, 2], np.float16), 100)     # fewer values than levels
    W[5, :150] = 1.0
    W[5, 150:] = -1.0
    W[6] = np.float16(65504.0) * np.sign(rng.normal(size=d_out)).astype(np.float16)   # largest finite halves
    W[7] = (rng.integers(0, 3, d_out) * 2.0 ** -24).astype(np.float16)               # subnormals
    W[8, :4] = [3.0, 1.0, 2.0, 1.0]
    for nb in (1, 2, 3, 4):
        bits = np.full(d_in, nb, np.uint8)
        for iters in (0, 1, 7):
            cent, codes = _kmeans_gpu(env, W, bits, iters=iters)
            ocent, ocodes = env["orc"].kmeans(W, bits, iters=iters)
            _check_kmeans(cent, codes, ocent, ocodes, exact=True)


@pytest.mark.parametrize("d_out", [512, 2048, 8192, 28672])
def test_kmeans_parity_signed_zeros_and_boundaries_at_zero(env, d_out):
    # +0 and -0 are one value: they share a cell whatever boundary lands on or next to zero
    rng = np.random.default_rng(d_out + 11)
    d_in = 12
    W = rng.normal(0, 0.02, (d_in, d_out)).astype(np.float16)
    z = rng.random(W.shape)
    W[z < 0.15] = np.float16(0.0)
    W[z < 0.075] = np.float16(-0.0)
    W[0] = rng.choice(np.array([-1.0, -0.0, 0.0, 1.0], np.float16), d_out)        # symmetric: midpoint exactly 0
    W[1] = rng.choice(np.array([-2.0 ** -24, -0.0, 0.0], np.float16), d_out)      # midpoint just below zero
    W[2] = rng.choice(np.array([-0.0, 0.0, 2.0 ** -24], np.float16), d_out)
    W[3] = rng.choice(np.array([-3.0, -0.0, 0.0, 1.0], np.float16), d_out)
    for nb in (1, 2, 3, 4):
        bits = np.full(d_in, nb, np.uint8)
        cent, codes = _kmeans_gpu(env, W, bits, iters=20)
        ocent, ocodes = env["orc"].kmeans(W, bits, iters=20)
        _check_kmeans(cent, codes, ocent, ocodes, exact=True)


@pytest.mark.parametrize("dtype,d_out", [(np.float16, 32768), (np.float32, 16384)])
def test_kmeans_parity_at_the_largest_channel_length(env, dtype, d_out):
    """The documented limits of cmpq_kmeans_quantize: 32768 outputs per channel for fp16
    weights, 16384 for fp32; with removed entries and every width."""
    rng = np.random.default_rng(d_out)
    d_in = 6
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.005] *= 20
    W = W.astype(dtype)
    bits = np.array([1, 2, 3, 4, 16, 4], np.uint8)
    excl = np.sort(rng.choice(d_in * d_out, 1500, replace=False)).astype(np.int64)
    for out_idx in (None, excl):
        cent, codes = _kmeans_gpu(env, W, bits, out_idx=out_idx, iters=6)
        ocent, ocodes = env["orc"].kmeans(W, bits, out_idx=out_idx, iters=6)
        _check_kmeans(cent, codes, ocent, ocodes, exact=dtype == np.float16)


def test_kmeans_direct_kernel_agrees(env):
    """The brute-force kernel (CMPQ_KMEANS_DIRECT) is a second implementation: same bits as
    the bucket kernel and as the oracle, with and without removed entries."""
    B, orc = env["B"], env["orc"]
    rng = np.random.default_rng(21)
    d_in, d_out = 48, 4096
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 12
    W = W.astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[7] = 16
    excl = np.sort(rng.choice(d_in * d_out, 2000, replace=False)).astype(np.int64)
    for out_idx in (None, excl):
        ocent, ocodes = orc.kmeans(W, bits, out_idx=out_idx, iters=11)
        for algo in (B.KMEANS_DIRECT, B.KMEANS_HISTOGRAM):       # named per call (the job form of the call)
            cent, codes = _kmeans_gpu(env, W, bits, out_idx=out_idx, iters=11, algorithm=algo)
            _check_kmeans(cent, codes, ocent, ocodes, exact=True)


def test_kmeans_parity_with_removed_entries_and_weights(env):
    rng = np.random.default_rng(2)
    d_in, d_out = 32, 777
    W = (rng.standard_t(3, (d_in, d_out)) * 0.03).astype(np.float16)
    bits = rng.integers(2, 5, d_in).astype(np.uint8)
    bits[9] = 16
    excl = np.sort(rng.choice(d_in * d_out, 600, replace=False)).astype(np.int64)
    excl = np.concatenate([excl, np.arange(4 * d_out, 5 * d_out)])      # channel 4 removed entirely
    excl = np.unique(excl)
    cent, codes = _kmeans_gpu(env, W, bits, out_idx=excl, iters=9)
    ocent, ocodes = env["orc"].kmeans(W, bits, out_idx=excl, iters=9)
    _check_kmeans(cent, codes, ocent, ocodes, exact=True)
    assert (cent[4, :1 << bits[4]] == 0).all()
    # importance weights: integer weights keep the fp64 sums exact -> still bit-identical
    ew = rng.integers(0, 5, (d_in, d_out)).astype(np.float32)
    cent, codes = _kmeans_gpu(env, W, bits, ew=ew, iters=9)
    ocent, ocodes = env["orc"].kmeans(W, bits, elem_weight=ew, iters=9)
    _check_kmeans(cent, codes, ocent, ocodes, exact=True)
    # real-valued weights and both mechanisms together: within the stated bars
    ew = rng.lognormal(0, 1, (d_in, d_out)).astype(np.float32)
    cent, codes = _kmeans_gpu(env, W, bits, out_idx=excl, ew=ew, iters=9)
    ocent, ocodes = env["orc"].kmeans(W, bits, out_idx=excl, elem_weight=ew, iters=9)
    _check_kmeans(cent, codes, ocent, ocodes, exact=False)


def test_kmeans_flags_nonfinite_weights_and_is_reproducible(env):
    rng = np.random.default_rng(3)
    W = rng.normal(0, 1, (8, 500)).astype(np.float16)
    bits = np.full(8, 3, np.uint8)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    c1, k1 = _kmeans_gpu(env, W, bits, status=st)
    c2, k2 = _kmeans_gpu(env, W, bits, status=st)
    assert st.item() == 0 and np.array_equal(c1, c2) and np.array_equal(k1, k2)
    W[2, 7] = np.nan
    c3, k3 = _kmeans_gpu(env, W, bits, status=st)
    assert st.item() & env["B"].STATUS_NONFINITE
    ok = np.arange(8) != 2                       # the other channels are not affected
    assert np.array_equal(c3[ok], c1[ok]) and np.array_equal(k3[ok], k1[ok])
    assert k3[2].max() < 8


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("d_in,d_out", [(6, 64), (9, 300), (11, 4096 + 24), (5, 8192), (4, 28672)])
def test_kmeans_from_given_levels_parity(env, dtype, d_in, d_out):
    """CMPQ_INIT_GIVEN: rounds started from the caller's levels (the preliminary ones, a shuffled
    copy with a repeat, levels far outside the data), with and without removed entries."""
    orc = env["orc"]
    if dtype == np.float32:
        d_out = min(d_out, 16384)                        # the limit of the entry point for fp32
    rng = np.random.default_rng(d_in * 17 + d_out)
    W = rng.normal(0, 0.03, (d_in, d_out)).astype(dtype)
    W[0, : d_out // 3] = W[0, 0]
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[d_in // 2] = 16
    n_q = max(1, d_in * d_out // 80)
    excl = np.sort(rng.choice(d_in * d_out, n_q, replace=False)).astype(np.int64)
    prelim, _ = orc.kmeans(W, bits, iters=3)
    odd = prelim.copy()
    for i in range(d_in):
        K = 1 << int(bits[i]) if bits[i] <= 4 else 0
        if K >= 2:
            odd[i, :K] = rng.permutation(odd[i, :K])
            odd[i, K - 1] = odd[i, 0]                    # a repeated level
        if K >= 4:
            odd[i, 1] = 50.0                             # beyond every weight: stays without members
            odd[i, 2] = -0.0
    for start in (prelim, odd):
        for oi in (None, excl):
            for iters in (0, 4):
                ocent, ocodes = orc.kmeans(W, bits, out_idx=oi, iters=iters, start=start)
                cent, codes = _kmeans_gpu(env, W, bits, out_idx=oi, iters=iters, start=start)
                _check_kmeans(cent, codes, ocent, ocodes, exact=dtype == np.float16)


def test_kmeans_from_given_levels_weighted_and_flags(env):
    """The general kernel (importance per entry) from given levels; a non-finite starting level
    raises the status flag and leaves the other channels as they are."""
    orc, B = env["orc"], env["B"]
    rng = np.random.default_rng(5)
    d_in, d_out = 7, 700
    W = rng.normal(0, 0.03, (d_in, d_out)).astype(np.float16)
    bits = np.array([2, 3, 4, 16, 1, 4, 3], np.uint8)
    ew = rng.lognormal(0, 1, (d_in, d_out)).astype(np.float32)
    start, _ = orc.kmeans(W, bits, iters=2)
    ocent, ocodes = orc.kmeans(W, bits, elem_weight=ew, iters=5, start=start)
    cent, codes = _kmeans_gpu(env, W, bits, ew=ew, iters=5, start=start)
    _check_kmeans(cent, codes, ocent, ocodes, exact=False)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    good, gk = _kmeans_gpu(env, W, bits, iters=5, start=start, status=st)
    assert st.item() == 0
    bad = start.copy()
    bad[2, 3] = np.nan
    c, k = _kmeans_gpu(env, W, bits, iters=5, start=bad, status=st)
    assert st.item() & B.STATUS_NONFINITE
    ok = np.arange(d_in) != 2
    assert np.array_equal(c[ok], good[ok]) and np.array_equal(k[ok], gk[ok]) and k[2].max() < 16


@pytest.mark.parametrize("d_in,d_out", [(40, 512), (9, 4096 + 8), (5, 28672), (33, 1024 + 4)])
def test_kmeans_levels_alone(env, d_in, d_out):
    """cmpq_kmeans_quantize without codes (what the preliminary quantization of Sec. 3.2.2 asks
    for): the levels the call with codes leaves, bit for bit, on every launch shape of the
    histogram kernel, with entries removed, from given levels, and with tables kept; the status
    word still reports a non-finite weight; inputs other kernels take are refused."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in + d_out)
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 8
    W = W.astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[1] = 16
    dW, db = _dev(W), _dev(bits)
    ocent, _ = orc.kmeans(W, bits, iters=4)
    want, _ = _kmeans_gpu(env, W, bits, iters=4)
    cent = torch.full((d_in, 16), -3.0, dtype=torch.float32, device=DEV)
    B.kmeans_quantize(dW, db, None, 0, None, 4, cent, None, ws)
    assert _np(cent).tobytes() == want.tobytes()
    assert _rel(_np(cent)[bits <= 4][:, :2], ocent[bits <= 4][:, :2]) <= 1e-5
    # with removed entries, from given levels
    excl = np.sort(rng.choice(d_in * d_out, d_in * d_out // 50, replace=False)).astype(np.int32)
    want2, _ = _kmeans_gpu(env, W, bits, out_idx=excl, iters=3, start=want)
    cent2 = _dev(want.copy())
    B.kmeans_quantize(dW, db, _dev(excl), len(excl), None, 3, cent2, None, ws, init=B.INIT_GIVEN)
    assert _np(cent2).tobytes() == want2.tobytes()
    # tables kept by a run without codes serve a later run
    tables = torch.zeros(B.arrangement_bytes(d_in, d_out), dtype=torch.uint8, device=DEV)
    cent3 = torch.empty_like(cent)
    B.kmeans_quantize(dW, db, None, 0, None, 4, cent3, None, ws, arrangement=tables, arrangement_use=B.ARRANGEMENT_KEEP)
    assert _np(cent3).tobytes() == want.tobytes()
    want4, codes4 = _kmeans_gpu(env, W, bits, out_idx=excl, iters=4)
    cent4 = torch.empty_like(cent)
    k4 = torch.empty((d_in, d_out), dtype=torch.uint8, device=DEV)
    B.kmeans_quantize(dW, db, _dev(excl), len(excl), None, 4, cent4, k4, ws, arrangement=tables,
                      arrangement_use=B.ARRANGEMENT_REUSE)
    assert _np(cent4).tobytes() == want4.tobytes() and np.array_equal(_np(k4), codes4)
    # a non-finite weight is still reported
    Wbad = W.copy()
    Wbad[0, 3] = np.inf
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.kmeans_quantize(_dev(Wbad), db, None, 0, None, 2, cent, None, ws, st)
    assert st.item() & B.STATUS_NONFINITE
    # fp32 weights and importance weights go to kernels that always code
    with pytest.raises(B.CmpqError):
        B.kmeans_quantize(_dev(W.astype(np.float32)), db, None, 0, None, 2, cent, None, ws)
    with pytest.raises(B.CmpqError):
        B.kmeans_quantize(dW, db, None, 0, _dev(np.ones((d_in, d_out), np.float32)), 2, cent, None, ws)


# ------------------------------------------------------------------ O_q

@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("d_in,d_out", [(3, 5), (20, 96), (16, 2048 + 40), (70, 333)])
def test_weight_outliers_parity(env, dtype, d_in, d_out):
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in * 7 + d_out)
    W = (rng.integers(-40, 40, (d_in, d_out)) / 64.0).astype(dtype)      # coarse grid: tied scores
    bits = rng.integers(1, 4, d_in).astype(np.uint8)
    bits[rng.integers(0, d_in)] = 16
    ocent, ocodes = orc.kmeans(W, bits, iters=3)
    live = int((bits <= 4).sum()) * d_out
    Wd, cd, kd, bd = _dev(W), _dev(ocent), _dev(ocodes), _dev(bits)
    for score in (B.SCORE_RESIDUAL, B.SCORE_MAGNITUDE):
        for k in sorted({0, 1, 9, live // 50 + 1, live // 2, live}):
            idx = torch.full((max(k, 1),), -7, dtype=torch.int32, device=DEV)
            val = torch.zeros(max(k, 1), dtype=torch.float16, device=DEV)
            B.extract_weight_outliers(Wd, cd, kd, bd, k, idx, val, ws, score)
            oidx, oval = orc.weight_outliers(W, ocent, ocodes, bits, k, score)
            assert np.array_equal(_np(idx)[:k].astype(np.int64), oidx), (score, k)
            assert np.array_equal(_np(val)[:k].view(np.uint16), oval)
            if score == B.SCORE_RESIDUAL:        # without codes: the distance to the nearest level
                idx.fill_(-7)
                B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws, score)
                assert np.array_equal(_np(idx)[:k].astype(np.int64), oidx), ("no codes", k)
                assert np.array_equal(_np(val)[:k].view(np.uint16), oval)
    # asking for more than the candidates: every candidate, then -1
    k = live + 5
    idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
    B.extract_weight_outliers(Wd, cd, kd, bd, k, idx, None, ws)
    got = _np(idx)
    assert (got[live:] == -1).all() and len(np.unique(got[:live])) == live and (got[:live] >= 0).all()


@pytest.mark.parametrize("case", ["spread", "ties", "concentrated", "ragged"])
def test_weight_outliers_staging_and_full_path(env, case):
    # large enough that a unit's share of the staging list is smaller than the unit: "spread"
    # is answered from the list, "ties" and "concentrated" overflow it and take the full path
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(len(case))
    d_in, d_out = (300, 16384) if case != "ragged" else (523, 9000 + 4)
    W = rng.normal(0, 0.02, (d_in, d_out))
    if case == "ties":
        W = np.round(W * 64) / 64
    if case == "concentrated":
        W[7] *= 50
    W = W.astype(np.float16)
    bits = rng.integers(2, 5, d_in).astype(np.uint8)
    bits[5] = 16
    ocent, ocodes = orc.kmeans(W, bits, iters=2)
    live = int((bits <= 4).sum()) * d_out
    Wd, cd, kd, bd = _dev(W), _dev(ocent), _dev(ocodes), _dev(bits)
    for score in (B.SCORE_RESIDUAL, B.SCORE_MAGNITUDE):
        for k in (live // 100, 17):
            idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
            val = torch.zeros(k, dtype=torch.float16, device=DEV)
            B.extract_weight_outliers(Wd, cd, kd, bd, k, idx, val, ws, score)
            oidx, oval = orc.weight_outliers(W, ocent, ocodes, bits, k, score)
            assert np.array_equal(_np(idx).astype(np.int64), oidx), (case, score, k)
            assert np.array_equal(_np(val).view(np.uint16), oval)
            if score == B.SCORE_RESIDUAL:
                idx.fill_(-7)
                B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws, score)
                assert np.array_equal(_np(idx).astype(np.int64), oidx), (case, "no codes", k)
                assert np.array_equal(_np(val).view(np.uint16), oval)


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_weight_outliers_sampled_guess(env, dtype):
    # enough wave-chunks (17 per channel x 1536) that the first guess comes from a sample
    # (every 3rd chunk); ragged channel tail, both dtypes and both scores
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(5)
    d_in, d_out = 1536, 8192 + 8
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.005] *= 8
    W = W.astype(dtype)
    bits = rng.integers(3, 5, d_in).astype(np.uint8)
    bits[[11, 700]] = 16
    ocent, ocodes = orc.kmeans(W, bits, iters=2)
    live = int((bits <= 4).sum()) * d_out
    Wd, cd, kd, bd = _dev(W), _dev(ocent), _dev(ocodes), _dev(bits)
    for score in (B.SCORE_RESIDUAL, B.SCORE_MAGNITUDE):
        for k in (live // 100, live // 2000):
            idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
            val = torch.zeros(k, dtype=torch.float16, device=DEV)
            B.extract_weight_outliers(Wd, cd, kd, bd, k, idx, val, ws, score)
            oidx, oval = orc.weight_outliers(W, ocent, ocodes, bits, k, score)
            assert np.array_equal(_np(idx).astype(np.int64), oidx), (score, k)
            assert np.array_equal(_np(val).view(np.uint16), oval)
            if score == B.SCORE_RESIDUAL:
                idx.fill_(-7)
                B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws, score)
                assert np.array_equal(_np(idx).astype(np.int64), oidx), ("no codes", k)
                assert np.array_equal(_np(val).view(np.uint16), oval)


@pytest.mark.parametrize("d_in,d_out", [(1536, 8192 + 8), (600, 28672), (96, 1000), (130, 1001)])
def test_weight_outliers_without_codes_edge_values(env, d_in, d_out):
    """O_q without codes on FP16 weights, where the staging pass tells candidates from the
    channel's intervals of "close to some level": levels that did not come from a clustering
    (unsorted, repeated, outside the weights' range, not FP16 values, equal to weights), weights
    at the ends of the FP16 range, zeros of both signs and subnormals, channel lengths with a
    ragged last wave-chunk and rows that rule out vector loads; from a handful of outliers
    (a threshold wider than the gaps between levels: one interval) to a tenth of the layer (a
    threshold below the FP16 spacing at some levels: no interval there).  Bit-exact against the
    oracle's ranking of the distance to the nearest level."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in + 3 * d_out)
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.005] *= 8
    W = W.astype(np.float16)
    flat = W.reshape(-1)
    special = np.array([65504, -65504, 0.0, -0.0, 6e-8, -6e-8, 6e-5, -6.1e-5, 1.0, -2.5], np.float16)
    flat[rng.choice(flat.size, 400, replace=False)] = rng.choice(special, 400)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[[5, d_in - 1]] = 16
    cent = np.full((d_in, 16), np.inf, np.float32)
    for i in range(d_in):
        if bits[i] > 4:
            continue
        K = 1 << bits[i]
        lv = rng.normal(0, 0.03, K).astype(np.float32)
        if i % 7 == 0:
            lv[0] = lv[K - 1]                                   # a repeated level
        if i % 11 == 0:
            lv[K // 2] = np.float32(W[i, 3])                    # a level that is one of the weights
        if i % 13 == 0:
            lv[0] = np.float32(3.0e4)                           # far outside the weights
        if i % 17 == 0:
            lv[K - 1] = np.float32(-1e-7)                       # among the subnormals
        cent[i, :K] = lv
    live = int((bits <= 4).sum()) * d_out
    Wd, cd, bd = _dev(W), _dev(cent), _dev(bits)
    for k in (7, live // 2000, live // 100, live // 10):
        idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
        val = torch.zeros(k, dtype=torch.float16, device=DEV)
        B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws)
        oidx, oval = orc.weight_outliers(W, cent, None, bits, k)
        assert np.array_equal(_np(idx).astype(np.int64), oidx), k
        assert np.array_equal(_np(val).view(np.uint16), oval)


@pytest.mark.parametrize("seed", range(12))
def test_weight_outliers_without_codes_random_levels_and_counts(env, seed):
    """The same route over random draws: weight scale, number and spread of the levels (from
    levels packed closer than the FP16 spacing to levels whole binades apart), channel length and
    the count asked for all vary, so the threshold falls anywhere from far above the gaps
    between levels (one interval per channel) to below them (one per level, or none)."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(1000 + seed)
    d_in = int(rng.integers(40, 200))
    d_out = int(rng.choice([512, 1000, 2048 + 24, 4096, 5000]))
    scale = float(10.0 ** rng.uniform(-4, 1))
    W = (rng.standard_t(3, (d_in, d_out)) * scale).astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[rng.integers(0, d_in)] = 16
    cent = np.full((d_in, 16), np.inf, np.float32)
    for i in range(d_in):
        if bits[i] <= 4:
            K = 1 << bits[i]
            spread = float(10.0 ** rng.uniform(-3, 1))
            cent[i, :K] = (rng.normal(0, scale * spread, K)).astype(np.float32)
    live = int((bits <= 4).sum()) * d_out
    Wd, cd, bd = _dev(W), _dev(cent), _dev(bits)
    for frac in (1e-4, 3e-3, 0.05, 0.4):
        k = max(1, int(live * frac))
        idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
        val = torch.zeros(k, dtype=torch.float16, device=DEV)
        B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws)
        oidx, oval = orc.weight_outliers(W, cent, None, bits, k)
        assert np.array_equal(_np(idx).astype(np.int64), oidx), (seed, k)
        assert np.array_equal(_np(val).view(np.uint16), oval)


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("d_in,d_out", [(3, 5), (20, 96), (16, 2048 + 40), (70, 333), (40, 8192)])
def test_weight_outliers_per_channel_parity(env, dtype, d_in, d_out):
    """The per-channel scope of O_q: k entries in every quantized channel, bit-exact against the
    oracle's per-row sorts - tied scores (coarse grid), channels of O_act in between, ragged
    channel lengths, every k from none to the whole channel, both scores."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in * 11 + d_out)
    W = (rng.integers(-40, 40, (d_in, d_out)) / 64.0).astype(dtype)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    bits[rng.integers(0, d_in, 2)] = 16
    ocent, ocodes = orc.kmeans(W, bits, iters=3)
    n_live = int((bits <= 4).sum())
    Wd, cd, kd, bd = _dev(W), _dev(ocent), _dev(ocodes), _dev(bits)
    for score in (B.SCORE_RESIDUAL, B.SCORE_MAGNITUDE):
        for k in sorted({0, 1, 3, d_out // 100 + 1, d_out // 2, d_out}):
            idx = torch.full((max(k * n_live, 1),), -7, dtype=torch.int32, device=DEV)
            val = torch.zeros(max(k * n_live, 1), dtype=torch.float16, device=DEV)
            B.extract_weight_outliers(Wd, cd, kd, bd, k, idx, val, ws, score, B.SCOPE_CHANNEL)
            oidx, oval = orc.weight_outliers_per_channel(W, ocent, ocodes, bits, k, score)
            assert np.array_equal(_np(idx)[:k * n_live].astype(np.int64), oidx), (score, k)
            assert np.array_equal(_np(val)[:k * n_live].view(np.uint16), oval)
            if score == B.SCORE_RESIDUAL:
                idx.fill_(-7)
                B.extract_weight_outliers(Wd, cd, None, bd, k, idx, val, ws, score, B.SCOPE_CHANNEL)
                assert np.array_equal(_np(idx)[:k * n_live].astype(np.int64), oidx), ("no codes", k)
                assert np.array_equal(_np(val)[:k * n_live].view(np.uint16), oval)


def test_layer_with_per_channel_outliers_end_to_end(env):
    """The whole path with O_q taken per channel (count = the fraction of d_out, half rounded
    up), free running against the oracle's same chain: every integer output identical."""
    P, ws, orc = env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(31)
    d_in, d_out = 96, 1200
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 9
    W = W.astype(np.float16)
    X = (rng.normal(0, 1, (64, d_in)) * np.exp(rng.normal(0, 0.7, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(X), ws)
    r = P.quantize_layer(_dev(W), sumsq, (2, 3, 4), 3.2, 20000, 7500, 8, ws, with_error=True, transposed=True,
                         oq_per_channel=True)
    o = orc.quantize_layer(W, X, (2, 3, 4), 3.2, 20000, 7500, 8, per_channel=True)
    assert len(o["out_idx"]) == 9 * int((o["bits"] <= 4).sum())           # 0.75 % of 1200
    assert np.array_equal(_np(r.bits), o["bits"]) and np.array_equal(_np(r.out_idx).astype(np.int64), o["out_idx"])
    assert np.array_equal(_np(r.out_val).view(np.uint16), o["out_val"])
    assert np.array_equal(_np(r.centroids), o["centroids"]) and np.array_equal(_np(r.codes), o["codes"])
    assert abs(_np(r.err_total)[0] - o["totals"][0]) <= 1e-9 * o["totals"][0]


# ------------------------------------------------------------------ storage and error

@pytest.mark.parametrize("d_out", [1, 31, 32, 33, 100, 512, 4096 + 16])
def test_pack_parity(env, d_out):
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_out)
    d_in = 53
    for bit_set in ((2, 3), (2, 3, 4), (1, 2, 3, 4)):
        bits = rng.choice(np.array(bit_set + (16,), np.uint8), d_in)
        codes = np.stack([rng.integers(0, 1 << min(int(b), 4), d_out) for b in bits]).astype(np.uint8)
        cent = rng.normal(0, 1, (d_in, 16)).astype(np.float32)
        counts = [int((bits == b).sum()) for b in bit_set]
        packed = [torch.full((c, (d_out * b + 31) // 32), -1, dtype=torch.int32, device=DEV) if c else None
                  for b, c in zip(bit_set, counts)]
        chan = [torch.empty(c, dtype=torch.int32, device=DEV) if c else None for c in counts]
        lut = [torch.empty((c, 1 << b), dtype=torch.float16, device=DEV) if c else None
               for b, c in zip(bit_set, counts)]
        B.pack(_dev(codes), _dev(bits), _dev(cent), bit_set, counts, packed, chan, lut, ws)
        for j, b in enumerate(bit_set):
            opk, och, olut = orc.pack(codes, bits, cent, b)
            if counts[j] == 0:
                assert opk.shape[0] == 0
                continue
            assert np.array_equal(_np(packed[j]).view(np.uint32), opk)
            assert np.array_equal(_np(chan[j]), och)
            assert np.array_equal(_np(lut[j]).view(np.uint16), olut)


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_dequant_error_parity(env, dtype):
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(4)
    d_in, d_out = 45, 1234
    W = rng.normal(0, 0.05, (d_in, d_out)).astype(dtype)
    bits = rng.integers(2, 5, d_in).astype(np.uint8)
    bits[[1, 30]] = 16
    cent, codes = orc.kmeans(W, bits, iters=4)
    sumsq = rng.lognormal(3, 1, d_in).astype(np.float32)
    out_idx = np.sort(rng.choice(d_in * d_out, 500, replace=False)).astype(np.int64)
    for oi in (None, out_idx):
        for ss in (None, sumsq):
            err = torch.empty(d_in, dtype=torch.float64, device=DEV)
            tot = torch.empty(2, dtype=torch.float64, device=DEV)
            B.dequant_error(_dev(W), _dev(cent), _dev(codes), _dev(bits),
                            None if oi is None else _dev(oi.astype(np.int32)), 0 if oi is None else len(oi),
                            None if ss is None else _dev(ss), err, tot, ws)
            oerr, otot = orc.dequant_error(W, cent, codes, bits, oi, ss)
            assert _rel(_np(err), oerr) < 1e-12
            assert _rel(_np(tot), otot) < 1e-12                 # bar: 1e-4 relative on the layer total
    # every entry restored: zero error for fp16 weights ("reconstruction with all outliers restored")
    if dtype == np.float16:
        all_idx = _dev(np.arange(d_in * d_out, dtype=np.int32))
        err = torch.empty(d_in, dtype=torch.float64, device=DEV)
        tot = torch.empty(2, dtype=torch.float64, device=DEV)
        B.dequant_error(_dev(W), _dev(cent), _dev(codes), _dev(bits), all_idx, d_in * d_out, None, err, tot, ws)
        assert (err == 0).all() and (tot == 0).all()


@pytest.mark.parametrize("d_out", [4, 36, 252, 1000, 2052, 4100, 8192, 11008, 16388, 28672])
@pytest.mark.parametrize("bit_set", [(1, 2, 3, 4), (2, 3)])
def test_kmeans_with_stored_format_from_its_coding_pass(env, d_out, bit_set):
    """The job form of the K-means call with the stored format and the error asked for (the
    coding pass of the histogram kernel writes them): levels and codes identical to the plain
    call and to the oracle, packed rows / channel lists / tables bit for bit those of
    cmpq_pack_with_error and of the oracle, errors to 1e-12 - for every launch shape of the
    kernel, every width, channels of O_act in between, with and without removed entries, with
    the dense codes written or left out, and from given starting levels."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_out * 7 + len(bit_set))
    d_in = 24 if d_out > 4096 else 40
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = W.astype(np.float16)
    bits = rng.choice(np.array(bit_set + (16,), np.uint8), d_in)
    bits[:len(bit_set)] = bit_set                                   # every width present
    counts = [int((bits == b).sum()) for b in bit_set]
    sumsq = rng.lognormal(3, 1, d_in).astype(np.float32)
    n_q = max(1, d_in * d_out // 80)
    excl = np.sort(rng.choice(d_in * d_out, n_q, replace=False)).astype(np.int64)
    dW, db, dss = _dev(W), _dev(bits), _dev(sumsq)

    def outputs():
        packed = [torch.full((c, (d_out * b + 31) // 32), -1, dtype=torch.int32, device=DEV) if c else None
                  for b, c in zip(bit_set, counts)]
        chan = [torch.full((c,), -1, dtype=torch.int32, device=DEV) if c else None for c in counts]
        lut = [torch.full((c, 1 << b), -1, dtype=torch.float16, device=DEV) if c else None
               for b, c in zip(bit_set, counts)]
        return packed, chan, lut, torch.full((d_in,), -1.0, dtype=torch.float64, device=DEV), \
            torch.full((2,), -1.0, dtype=torch.float64, device=DEV)

    for oi, start_iters in ((None, None), (excl, None), (excl, 3)):
        iters = 5
        ostart = None
        if start_iters is not None:
            ostart, _ = orc.kmeans(W, bits, iters=start_iters)
        ocent, ocodes = orc.kmeans(W, bits, out_idx=oi, iters=iters, start=ostart)
        oerr, otot = orc.dequant_error(W, ocent, ocodes, bits, oi, sumsq)
        d_oi = None if oi is None else _dev(oi.astype(np.int32))
        n_oi = 0 if oi is None else len(oi)
        init = B.INIT_QUANTILE if ostart is None else B.INIT_GIVEN
        for with_codes in (True, False):
            cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV) if ostart is None else _dev(ostart)
            codes = torch.full((d_in, d_out), 255, dtype=torch.uint8, device=DEV) if with_codes else None
            packed, chan, lut, err, tot = outputs()
            B.kmeans_quantize_pack(dW, db, d_oi, n_oi, iters, cent, codes, bit_set, counts, packed, chan, lut, dss,
                                   err, tot, ws, init=init)
            assert np.array_equal(_np(cent), ocent)
            if with_codes:
                assert np.array_equal(_np(codes), ocodes)
            assert _rel(_np(err), oerr) < 1e-12 and _rel(_np(tot), otot) < 1e-12
            # the two-call route on the same levels and codes
            p2, c2, l2, e2, t2 = outputs()
            B.pack_with_error(dW, _dev(ocodes), db, _dev(ocent), bit_set, counts, p2, c2, l2, d_oi, n_oi, dss, e2, t2, ws)
            assert _rel(_np(err), _np(e2)) < 1e-12 and _rel(_np(tot), _np(t2)) < 1e-12
            for j, b in enumerate(bit_set):
                opk, och, olut = orc.pack(ocodes, bits, ocent, b)
                assert np.array_equal(_np(packed[j]).view(np.uint32), opk), (b, with_codes)
                assert np.array_equal(_np(chan[j]), och)
                assert np.array_equal(_np(lut[j]).view(np.uint16), olut)
                assert torch.equal(packed[j], p2[j]) and torch.equal(chan[j], c2[j])
                assert torch.equal(lut[j].view(torch.int16), l2[j].view(torch.int16))


@pytest.mark.parametrize("d_out", [4, 36, 252, 1000, 2052, 4100, 8192, 11008, 16388, 28672, 32768])
def test_final_kmeans_from_the_preliminary_runs_tables(env, d_out):
    """Sec. 3.2.2 runs the quantizer twice on the same channels.  With the preliminary run's
    per-channel tables kept (`arrangement`), the final run - which takes the entries of O_q out
    of them instead of building them again - gives the oracle's levels and codes bit for bit,
    with or without the stored format asked for: every launch shape, channels of O_act in
    between, removed entries that repeat one value many times, a channel with everything
    removed, another width in the second run, and given starting levels."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_out + 1)
    d_in = 12 if d_out > 4096 else 24
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = W.astype(np.float16)
    W[3, : max(1, d_out // 3)] = np.float16(0.0371)                 # one value many times ...
    W[4, ::2] = np.float16(-0.0)                                    # ... and both zeros
    W[4, 1::2] = np.float16(0.0) if d_out < 64 else W[4, 1::2]
    bit_set = (2, 3, 4)
    bits = rng.choice(np.array(bit_set + (16,), np.uint8), d_in)
    bits[:3] = bit_set
    bits[3], bits[4], bits[5] = 3, 2, 4
    counts = [int((bits == b).sum()) for b in bit_set]
    n_q = max(1, d_in * d_out // 60)
    excl = set(rng.choice(d_in * d_out, n_q, replace=False).tolist())
    excl |= {3 * d_out + o for o in range(0, max(1, d_out // 3), 2)}    # many removed entries of one value
    excl |= {4 * d_out + o for o in range(0, d_out, 3)}
    excl |= {5 * d_out + o for o in range(d_out)}                       # a whole channel
    excl = np.array(sorted(excl), np.int64)
    dW, db = _dev(W), _dev(bits)
    tables = torch.zeros(B.arrangement_bytes(d_in, d_out), dtype=torch.uint8, device=DEV)
    assert tables.numel() > 0
    cent1 = torch.empty((d_in, 16), dtype=torch.float32, device=DEV)
    codes1 = torch.empty((d_in, d_out), dtype=torch.uint8, device=DEV)
    B.kmeans_quantize(dW, db, None, 0, None, 4, cent1, codes1, ws, arrangement=tables,
                      arrangement_use=B.ARRANGEMENT_KEEP)
    o1, k1 = orc.kmeans(W, bits, iters=4)
    assert np.array_equal(_np(cent1), o1) and np.array_equal(_np(codes1), k1)     # keeping changes nothing
    d_oi = _dev(excl.astype(np.int32))
    bits2 = bits.copy()
    bits2[bits2 == 2] = 3                                           # the tables do not depend on the width
    for bb, start in ((bits, None), (bits, o1), (bits2, None)):
        ocent, ocodes = orc.kmeans(W, bb, out_idx=excl, iters=5, start=start)
        init = B.INIT_QUANTILE if start is None else B.INIT_GIVEN
        # plain call from the kept tables
        cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV) if start is None else _dev(start)
        codes = torch.full((d_in, d_out), 255, dtype=torch.uint8, device=DEV)
        B.kmeans_quantize(dW, _dev(bb), d_oi, len(excl), None, 5, cent, codes, ws, init=init, arrangement=tables,
                          arrangement_use=B.ARRANGEMENT_REUSE)
        assert np.array_equal(_np(cent), ocent) and np.array_equal(_np(codes), ocodes)
        # and with the stored format from the coding pass
        cnt = [int((bb == b).sum()) for b in bit_set]
        packed = [torch.full((c, (d_out * b + 31) // 32), -1, dtype=torch.int32, device=DEV) if c else None
                  for b, c in zip(bit_set, cnt)]
        chan = [torch.full((c,), -1, dtype=torch.int32, device=DEV) if c else None for c in cnt]
        lut = [torch.full((c, 1 << b), -1, dtype=torch.float16, device=DEV) if c else None for b, c in zip(bit_set, cnt)]
        err = torch.full((d_in,), -1.0, dtype=torch.float64, device=DEV)
        tot = torch.full((2,), -1.0, dtype=torch.float64, device=DEV)
        cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV) if start is None else _dev(start)
        codes = torch.full((d_in, d_out), 255, dtype=torch.uint8, device=DEV)
        B.kmeans_quantize_pack(dW, _dev(bb), d_oi, len(excl), 5, cent, codes, bit_set, cnt, packed, chan, lut, None, err,
                               tot, ws, init=init, arrangement=tables, arrangement_use=B.ARRANGEMENT_REUSE)
        assert np.array_equal(_np(cent), ocent) and np.array_equal(_np(codes), ocodes)
        oerr, otot = orc.dequant_error(W, ocent, ocodes, bb, excl, None)
        assert _rel(_np(err), oerr) < 1e-12 and _rel(_np(tot), otot) < 1e-12
        for j, b in enumerate(bit_set):
            if cnt[j]:
                opk, och, olut = orc.pack(ocodes, bb, ocent, b)
                assert np.array_equal(_np(packed[j]).view(np.uint32), opk) and np.array_equal(_np(chan[j]), och)
                assert np.array_equal(_np(lut[j]).view(np.uint16), olut)


def test_kept_tables_flags(env):
    """A channel that held a non-finite weight when the tables were kept is flagged again by the
    run that starts from them; a buffer that holds no kept tables raises the arrangement flag;
    either way the other channels and the caller's memory are left in order."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(8)
    d_in, d_out = 6, 2048
    W = rng.normal(0, 0.02, (d_in, d_out)).astype(np.float16)
    W[2, 100] = np.nan
    bits = np.full(d_in, 3, np.uint8)
    dW, db = _dev(W), _dev(bits)
    tables = torch.zeros(B.arrangement_bytes(d_in, d_out), dtype=torch.uint8, device=DEV)
    cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV)
    codes = torch.empty((d_in, d_out), dtype=torch.uint8, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.kmeans_quantize(dW, db, None, 0, None, 3, cent, codes, ws, st, arrangement=tables, arrangement_use=B.ARRANGEMENT_KEEP)
    assert st.item() == B.STATUS_NONFINITE
    st.zero_()
    c2, k2 = torch.empty_like(cent), torch.empty_like(codes)
    B.kmeans_quantize(dW, db, None, 0, None, 3, c2, k2, ws, st, arrangement=tables, arrangement_use=B.ARRANGEMENT_REUSE)
    assert st.item() == B.STATUS_NONFINITE
    assert torch.equal(c2, cent) and torch.equal(k2, codes)        # flagged channel included: zeros both times
    keep = np.arange(d_in) != 2
    oc, ok = orc.kmeans(W[keep], bits[keep], iters=3)
    assert np.array_equal(_np(c2)[keep], oc) and np.array_equal(_np(k2)[keep], ok)
    st.zero_()
    blank = torch.zeros_like(tables)
    B.kmeans_quantize(dW, db, None, 0, None, 3, c2, k2, ws, st, arrangement=blank, arrangement_use=B.ARRANGEMENT_REUSE)
    assert st.item() == B.STATUS_ARRANGEMENT and not _np(k2).any()
    # the buffer is for the histogram kernel only, and is kept from all weights
    with pytest.raises(B.CmpqError):
        B.kmeans_quantize(_dev(W.astype(np.float32)), db, None, 0, None, 3, c2, k2, ws, arrangement=tables,
                          arrangement_use=B.ARRANGEMENT_KEEP)
    with pytest.raises(B.CmpqError):
        B.kmeans_quantize(dW, db, _dev(np.array([5], np.int32)), 1, None, 3, c2, k2, ws, arrangement=tables,
                          arrangement_use=B.ARRANGEMENT_KEEP)


def test_kmeans_with_stored_format_other_inputs_and_flags(env):
    """The same job on inputs the histogram kernel does not take (fp32 weights, importance
    weights, the brute-force rounds): the general kernels run and the stored format follows in
    its own pass - same outputs as the two calls; a non-finite channel raises the flag, gets a
    row of zero codes and no number for its error while the other channels are untouched."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(3)
    d_in, d_out, bit_set = 12, 640, (2, 3, 4)
    bits = rng.choice(np.array(bit_set, np.uint8), d_in)
    counts = [int((bits == b).sum()) for b in bit_set]

    def run(W, ew=None, algorithm=B.KMEANS_HISTOGRAM, status=None):
        packed = [torch.full((c, (d_out * b + 31) // 32), -1, dtype=torch.int32, device=DEV) if c else None
                  for b, c in zip(bit_set, counts)]
        chan = [torch.full((c,), -1, dtype=torch.int32, device=DEV) if c else None for c in counts]
        lut = [torch.full((c, 1 << b), -1, dtype=torch.float16, device=DEV) if c else None
               for b, c in zip(bit_set, counts)]
        err = torch.full((d_in,), -1.0, dtype=torch.float64, device=DEV)
        tot = torch.full((2,), -1.0, dtype=torch.float64, device=DEV)
        cent = torch.empty((d_in, 16), dtype=torch.float32, device=DEV)
        codes = torch.empty((d_in, d_out), dtype=torch.uint8, device=DEV)
        B.kmeans_quantize_pack(_dev(W), _dev(bits), None, 0, 4, cent, codes, bit_set, counts, packed, chan, lut, None,
                               err, tot, ws, status, algorithm=algorithm, elem_weight=None if ew is None else _dev(ew))
        return _np(cent), _np(codes), packed, lut, _np(err), _np(tot)

    W32 = rng.normal(0, 0.05, (d_in, d_out)).astype(np.float32)
    ew = rng.lognormal(0, 1, (d_in, d_out)).astype(np.float32)
    for W, e, algo in ((W32, None, B.KMEANS_HISTOGRAM), (W32.astype(np.float16), ew, B.KMEANS_HISTOGRAM),
                       (W32.astype(np.float16), None, B.KMEANS_DIRECT)):
        cent, codes, packed, lut, err, tot = run(W, e, algo)
        ocent, ocodes = orc.kmeans(W, bits, elem_weight=e, iters=4)
        assert _rel(cent, ocent) <= 1e-5 and (codes != ocodes).mean() <= 1e-4
        oerr, otot = orc.dequant_error(W, cent, codes, bits)          # the GPU's own levels and codes
        assert _rel(err, oerr) < 1e-12 and _rel(tot, otot) < 1e-12
        for j, b in enumerate(bit_set):
            opk, _, olut = orc.pack(codes, bits, cent, b)
            assert np.array_equal(_np(packed[j]).view(np.uint32), opk) and np.array_equal(_np(lut[j]).view(np.uint16), olut)
    bad = W32.astype(np.float16)
    bad[5, 77] = np.inf
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    cent, codes, packed, lut, err, tot = run(bad, status=st)
    good = run(W32.astype(np.float16))
    assert st.item() & B.STATUS_NONFINITE and np.isnan(err[5]) and not codes[5].any()
    keep = np.arange(d_in) != 5
    assert np.array_equal(err[keep], good[4][keep]) and np.array_equal(codes[keep], good[1][keep])
    j5 = bit_set.index(int(bits[5]))
    row5 = int((bits[:5] == bits[5]).sum())
    assert not _np(packed[j5])[row5].any() and not _np(lut[j5]).view(np.uint16)[row5].any()


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
@pytest.mark.parametrize("d_in,d_out", [(1, 1), (7, 31), (45, 1234), (19, 4096 + 48), (6, 8192 + 32 * 256 + 8)])
def test_pack_with_error_parity(env, dtype, d_in, d_out):
    """Stored format and error in one pass: against the oracle (packed rows, channel lists and
    tables bit for bit, errors to 1e-12), and bit for bit against the two separate calls."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in * 131 + d_out)
    W = rng.normal(0, 0.05, (d_in, d_out)).astype(dtype)
    bit_set = (2, 3, 4)
    bits = rng.choice(np.array(bit_set + (16,), np.uint8), d_in, p=[0.3, 0.3, 0.3, 0.1])
    cent, codes = orc.kmeans(W, bits, iters=3)
    sumsq = rng.lognormal(3, 1, d_in).astype(np.float32)
    n_q = min(d_in * d_out, 1 + d_in * d_out // 50)
    out_idx = np.sort(rng.choice(d_in * d_out, n_q, replace=False)).astype(np.int64)
    counts = [int((bits == b).sum()) for b in bit_set]

    def outputs():
        packed = [torch.full((c, (d_out * b + 31) // 32), -1, dtype=torch.int32, device=DEV) if c else None
                  for b, c in zip(bit_set, counts)]
        chan = [torch.full((c,), -1, dtype=torch.int32, device=DEV) if c else None for c in counts]
        lut = [torch.full((c, 1 << b), -1, dtype=torch.float16, device=DEV) if c else None
               for b, c in zip(bit_set, counts)]
        return packed, chan, lut, torch.empty(d_in, dtype=torch.float64, device=DEV), \
            torch.empty(2, dtype=torch.float64, device=DEV)

    dW, dk, db, dc = _dev(W), _dev(codes), _dev(bits), _dev(cent)
    for oi in (None, out_idx):
        for ss in (None, sumsq):
            d_oi = None if oi is None else _dev(oi.astype(np.int32))
            n_oi = 0 if oi is None else len(oi)
            d_ss = None if ss is None else _dev(ss)
            packed, chan, lut, err, tot = outputs()
            B.pack_with_error(dW, dk, db, dc, bit_set, counts, packed, chan, lut, d_oi, n_oi, d_ss, err, tot, ws)
            p2, c2, l2, e2, t2 = outputs()
            B.pack(dk, db, dc, bit_set, counts, p2, c2, l2, ws)
            B.dequant_error(dW, dc, dk, db, d_oi, n_oi, d_ss, e2, t2, ws)
            oerr, otot = orc.dequant_error(W, cent, codes, bits, oi, ss)
            assert _rel(_np(err), oerr) < 1e-12 and _rel(_np(tot), otot) < 1e-12
            assert _rel(_np(err), _np(e2)) < 1e-12 and _rel(_np(tot), _np(t2)) < 1e-12
            for j, b in enumerate(bit_set):
                if counts[j] == 0:
                    continue
                opk, och, olut = orc.pack(codes, bits, cent, b)
                assert np.array_equal(_np(packed[j]).view(np.uint32), opk)
                assert np.array_equal(_np(chan[j]), och)
                assert np.array_equal(_np(lut[j]).view(np.uint16), olut)
                assert torch.equal(packed[j], p2[j]) and torch.equal(chan[j], c2[j])
                assert torch.equal(lut[j].view(torch.int16), l2[j].view(torch.int16))


# ------------------------------------------------------------------ the whole path, free running

def _compare_layer(env, r, o, bit_set, exact_levels):
    assert r.counts == list(o["counts"])
    assert np.array_equal(_np(r.act_idx), o["act_idx"])
    assert np.array_equal(_np(r.chan_mask), o["chan_mask"])
    assert np.array_equal(_np(r.bits), o["bits"])                                  # bit-exact
    _check_kmeans(_np(r.centroids_prelim), _np(r.codes_prelim), o["cent1"], o["codes1"], exact_levels)
    assert np.array_equal(_np(r.out_idx).astype(np.int64), o["out_idx"])           # bit-exact set
    assert np.array_equal(_np(r.out_val).view(np.uint16), o["out_val"])
    _check_kmeans(_np(r.centroids), _np(r.codes), o["centroids"], o["codes"], exact_levels)
    if np.array_equal(_np(r.codes), o["codes"]):
        for j, b in enumerate(bit_set):
            opk, och, olut = o["packs"][b]
            if r.counts[j]:
                assert np.array_equal(_np(r.packed[j]).view(np.uint32), opk)
                assert np.array_equal(_np(r.chan_idx[j]), och)
                assert np.array_equal(_np(r.lut[j]).view(np.uint16), olut)
    assert _rel(_np(r.err_total), o["totals"]) <= 1e-4                             # bar on the layer error


def test_end_to_end_tiny_config(env):
    """The smallest configuration at its full size: 512x256 fp32, 256 tokens, {2,3} avg 2.5, 10 rounds."""
    P, synth, ws, orc = env["P"], env["synth"], env["ws"], env["orc"]
    wl = synth.workload("tiny")
    wts, xs = synth.materialize(wl, "cpu")
    W, X = wts["linear"], xs["x"]
    _, sumsq = P.activation_stats(X.to(DEV), ws)
    r = P.quantize_layer(W.to(DEV), sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters,
                         ws, with_error=True, keep_prelim=True)
    o = orc.quantize_layer(W.numpy().T.copy(), X.numpy(), wl.bit_set, wl.avg_bits, wl.rho_act_ppm,
                           wl.rho_q_ppm, wl.iters)
    assert np.array_equal(_np(r.sumsq), o["sumsq"])
    _compare_layer(env, r, o, wl.bit_set, exact_levels=False)


def test_shader_clock_probe_reads_a_plausible_clock(env):
    """The measurement helper: both counters advance in every workgroup and their ratio is a
    clock between 0.5 and 3.5 GHz (the part's shader clock is 2.4 GHz at most)."""
    B = env["B"]
    ticks = torch.zeros((64, 2), dtype=torch.int64, device=DEV)
    khz = B.shader_clock_probe(500, ticks)
    torch.cuda.synchronize()
    t = _np(ticks).astype(np.float64)
    assert khz > 0 and (t > 0).all()
    ghz = t[:, 0] / t[:, 1] * khz * 1e3 / 1e9
    assert 0.5 < ghz.min() and ghz.max() < 3.5, (ghz.min(), ghz.max())


@pytest.mark.parametrize("rho_act_ppm,rho_q_ppm", [(0, 0), (5000, 0), (0, 5000), (4500, 500), (2500, 2500),
                                                    (500, 4500), (4500, 10000), (4500, 20000)])
def test_outlier_ratio_sweep(env, rho_act_ppm, rho_q_ppm):
    """The appendix's sweep over the share of outliers and its split between the two kinds (none,
    one kind only, 0.5 % split three ways, 1 % and 2 % of weight outliers): every setting
    against the oracle on one layer with a ragged channel length."""
    P, synth, ws, orc = env["P"], env["synth"], env["ws"], env["orc"]
    d_in, d_out, n = 320, 1336, 512
    W = synth.make_weight(d_out, d_in, "f16", 11, DEV)
    X = synth.make_activations(n, d_in, "f16", 12, DEV, hot_frac=0.02, hot_scale=20.0)
    _, sumsq = P.activation_stats(X, ws)
    bit_set, avg, iters = (2, 3, 4), 3.25, 6
    r = P.quantize_layer(W, sumsq, bit_set, avg, rho_act_ppm, rho_q_ppm, iters, ws, with_error=True,
                         keep_prelim=True)
    o = orc.quantize_layer(_np(W).T.copy(), None, bit_set, avg, rho_act_ppm, rho_q_ppm, iters, sumsq=_np(sumsq))
    assert len(o["act_idx"]) == env["B"].count_ppm(rho_act_ppm, d_in)
    assert len(o["out_idx"]) == env["B"].count_ppm(rho_q_ppm, d_in * d_out)
    _compare_layer(env, r, o, bit_set, exact_levels=True)


@pytest.mark.parametrize("from_prelim", [None, 5])
@pytest.mark.parametrize("name,shrink,tokens", [("q7b", 8, 2048), ("block7b", 16, 1024),
                                                ("block13b", 16, 1024), ("block70b", 32, 512)])
def test_end_to_end_scaled_workloads(env, name, shrink, tokens, from_prelim):
    """Every configuration's structure (layer mix, budget, outlier fractions, rounds) at a size the
    oracle finishes in seconds; dimensions stay multiples of 8, several tiles and ragged tails.
    Also with the final K-means continued from the preliminary levels for 5 rounds (the variant)."""
    P, synth, ws, orc = env["P"], env["synth"], env["ws"], env["orc"]
    wl = synth.scaled(synth.workload(name), tokens=tokens, shrink=shrink)
    wts, xs = synth.materialize(wl, DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    stats = {}
    for layer in wl.layers:
        if layer.x_key not in stats:
            stats[layer.x_key] = P.activation_stats(xs[layer.x_key], ws, status=status)[1]
            _, osum = orc.act_stats(_np(xs[layer.x_key]))
            assert np.array_equal(_np(stats[layer.x_key]), osum)
        W = wts[layer.name]
        r = P.quantize_layer(W, stats[layer.x_key], wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm,
                             wl.iters, ws, with_error=True, keep_prelim=True, status=status,
                             iters_final_from_prelim=from_prelim)
        assert torch.equal(r.W_t, W.t().contiguous())
        o = orc.quantize_layer(_np(W).T.copy(), None, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm,
                               wl.iters, sumsq=_np(stats[layer.x_key]), iters_final_from_prelim=from_prelim)
        _compare_layer(env, r, o, wl.bit_set, exact_levels=True)
    assert status.item() == 0


def test_block_over_several_streams_matches_one_stream(env):
    """Layers of a block shared out over 3 streams: every output bit-identical to the
    single-stream run (which the tests above check against the oracle)."""
    P, B, synth = env["P"], env["B"], env["synth"]
    wl = synth.scaled(synth.workload("block70b"), tokens=512, shrink=8)
    wts, xs = synth.materialize(wl, DEV)
    layers = [(l.name, l.x_key) for l in wl.layers]
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    args = (wts, xs, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters)
    one = P.quantize_block(*args, B.Workspace(DEV), with_error=True, status=status)
    for _ in range(2):                                  # the second run reuses streams and workspaces
        many = P.quantize_block(*args, [B.Workspace(DEV) for _ in range(3)], with_error=True,
                                status=status, streams=3)
        torch.cuda.synchronize()
        assert list(many) == list(one)
        for name in one:
            a, b = one[name], many[name]
            assert a.counts == b.counts
            for f in ("sumsq", "act_idx", "bits", "centroids", "codes", "out_idx", "out_val", "err_ch", "err_total"):
                assert torch.equal(getattr(a, f), getattr(b, f)), (name, f)
            for x, y in zip(a.packed + a.chan_idx + a.lut, b.packed + b.chan_idx + b.lut):
                assert (x is None) == (y is None) and (x is None or torch.equal(x, y)), name
    assert status.item() == 0


def test_blocks_run_on_without_a_join_between_them(env):
    """Three blocks enqueued one after the other without joining the streams in between (earlier
    results dropped while later blocks are still being enqueued, as a model quantized block after
    block would do), one join at the end: the last block equals a joined run bit for bit."""
    P, B, synth = env["P"], env["B"], env["synth"]
    wl = synth.scaled(synth.workload("block70b"), tokens=512, shrink=8)
    wts, xs = synth.materialize(wl, DEV)
    layers = [(l.name, l.x_key) for l in wl.layers]
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    args = (wts, xs, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters)
    wss = [B.Workspace(DEV) for _ in range(3)]
    want = P.quantize_block(*args, wss, with_error=True, status=status, streams=3)
    torch.cuda.synchronize()
    got = None
    for _ in range(3):
        got = P.quantize_block(*args, wss, with_error=True, status=status, streams=3, join=False)
    P.join_streams(DEV, 3)
    torch.cuda.synchronize()
    for name in want:
        a, b = want[name], got[name]
        for f in ("sumsq", "act_idx", "bits", "centroids", "codes", "out_idx", "out_val", "err_ch", "err_total"):
            assert torch.equal(getattr(a, f), getattr(b, f)), (name, f)
        for x, y in zip(a.packed + a.chan_idx + a.lut, b.packed + b.chan_idx + b.lut):
            assert (x is None) == (y is None) and (x is None or torch.equal(x, y)), name
    assert status.item() == 0


@pytest.mark.parametrize("seed", range(int(os.environ.get("CMPQ_RANDOM_CASES", "24"))))
def test_randomized_layers_end_to_end(env, seed):
    """Random shapes (any d_out, including odd ones), dtypes, bit sets, budgets, outlier fractions,
    round counts and value patterns (heavy ties, constant stretches, signed zeros, spikes) through
    the whole path, every output against the oracle."""
    P, ws, orc = env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(1000 + seed)
    d_in = int(rng.integers(1, 90))
    d_out = int(rng.choice([rng.integers(1, 40), rng.integers(40, 700), rng.integers(700, 6000)]))
    dtype = np.float16 if rng.random() < 0.7 else np.float32
    lo = int(rng.integers(1, 4))
    hi = int(rng.integers(lo + 1, 5))
    bit_set = tuple(range(lo, hi + 1))
    avg = float(np.round(rng.uniform(lo, hi), 2)) if rng.random() < 0.8 else float(rng.integers(lo, hi + 1))
    rho_act = int(rng.choice([0, 4500, 30000]))
    rho_q = int(rng.choice([0, 500, 10000, 60000]))
    iters = int(rng.integers(0, 9))
    W = rng.normal(0, 0.02, (d_in, d_out))
    style = int(rng.integers(0, 4))
    if style == 1:
        W = np.round(W * 128) / 128                                 # heavy ties
    elif style == 2:
        W[:, : d_out // 2] = 0.0                                    # constant stretch, zeros
        W[rng.random(W.shape) < 0.05] = -0.0
    elif style == 3:
        W[rng.random(W.shape) < 0.01] *= 30                         # spikes
    W = W.astype(dtype)
    X = (rng.normal(0, 1, (64, d_in)) * np.exp(rng.normal(0, 1, d_in))).astype(dtype)
    _, sumsq = P.activation_stats(_dev(X), ws)
    r = P.quantize_layer(_dev(W), sumsq, bit_set, avg, rho_act, rho_q, iters, ws, with_error=True, keep_prelim=True,
                         transposed=True)
    o = orc.quantize_layer(W, X, bit_set, avg, rho_act, rho_q, iters)
    assert np.array_equal(_np(r.sumsq), o["sumsq"]) or _rel(_np(r.sumsq), o["sumsq"]) <= 1e-5
    if not np.array_equal(_np(r.sumsq), o["sumsq"]):                # rank on identical statistics
        o = orc.quantize_layer(W, None, bit_set, avg, rho_act, rho_q, iters, sumsq=_np(r.sumsq))
    _compare_layer(env, r, o, bit_set, exact_levels=dtype == np.float16)


@pytest.mark.parametrize("seed", range(int(os.environ.get("CMPQ_RANDOM_CASES", "24"))))
def test_randomized_long_channels_kmeans(env, seed):
    """The workgroup shapes of long channels (256 and 512 lanes, table coding, re-fetched weights):
    random lengths up to the limit, widths, removed entries, round counts and value patterns."""
    rng = np.random.default_rng(5000 + seed)
    d_in = int(rng.integers(2, 7))
    d_out = int(rng.choice([4096, 8192, 8192 + 4 * int(rng.integers(1, 500)), 12288, 16384, 20000, 28672, 32768]))
    W = rng.normal(0, float(rng.choice([0.02, 1.0, 30.0])), (d_in, d_out))
    style = int(rng.integers(0, 4))
    if style == 1:
        W = np.round(W * 16) / 16
    elif style == 2:
        W[:, ::3] = 0.0
        W[rng.random(W.shape) < 0.02] = -0.0
    elif style == 3:
        W[rng.random(W.shape) < 0.002] *= 100
    W = np.clip(W, -60000, 60000).astype(np.float16)
    bits = rng.integers(1, 5, d_in).astype(np.uint8)
    if rng.random() < 0.3:
        bits[int(rng.integers(0, d_in))] = 16
    iters = int(rng.integers(0, 21))
    out_idx = None
    if rng.random() < 0.6:
        n = int(rng.integers(1, d_in * d_out // 50))
        out_idx = np.sort(rng.choice(d_in * d_out, n, replace=False)).astype(np.int64)
    cent, codes = _kmeans_gpu(env, W, bits, out_idx=out_idx, iters=iters)
    ocent, ocodes = env["orc"].kmeans(W, bits, out_idx=out_idx, iters=iters)
    _check_kmeans(cent, codes, ocent, ocodes, exact=True)


@pytest.mark.parametrize("seed", range(6))
def test_randomized_large_selection(env, seed):
    """O_q on layers large enough for a sampled first guess: random k, score, tie structure and
    concentration; the selected set and values are exact."""
    B, ws, orc = env["B"], env["ws"], env["orc"]
    rng = np.random.default_rng(9000 + seed)
    d_out = int(rng.choice([4096, 8192 + 8, 11008]))
    d_in = int(13_000_000 // d_out + rng.integers(0, 200))
    W = rng.normal(0, 0.02, (d_in, d_out)).astype(np.float32)
    style = seed % 3
    if style == 1:
        W = np.round(W * 256) / 256                                 # many equal scores
    elif style == 2:
        W[int(rng.integers(0, d_in))] *= 40                         # one channel holds most of the answer
    W = W.astype(np.float16)
    bits = rng.integers(2, 5, d_in).astype(np.uint8)
    bits[rng.choice(d_in, 5, replace=False)] = 16
    ocent, ocodes = orc.kmeans(W, bits, iters=1)
    live = int((bits <= 4).sum()) * d_out
    k = int(live * float(rng.choice([0.0005, 0.005, 0.01, 0.03])))
    score = B.SCORE_RESIDUAL if seed % 2 == 0 else B.SCORE_MAGNITUDE
    idx = torch.full((k,), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros(k, dtype=torch.float16, device=DEV)
    B.extract_weight_outliers(_dev(W), _dev(ocent), _dev(ocodes), _dev(bits), k, idx, val, ws, score)
    oidx, oval = orc.weight_outliers(W, ocent, ocodes, bits, k, score)
    assert np.array_equal(_np(idx).astype(np.int64), oidx)
    assert np.array_equal(_np(val).view(np.uint16), oval)
