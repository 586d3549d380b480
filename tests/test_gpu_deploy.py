"""GPU-vs-oracle parity of the product with the deployed weight (Sec. 6 / Fig. 4), through
the C ABI: cmpq_gather_channels, cmpq_outliers_by_column, cmpq_lut_matvec.

Bars: the regrouped outlier structure is bit-exact (integers; deltas are differences of two
FP16 values formed in fp32 on both sides).  The product is summed in fp32 on the GPU and in
fp64 by the oracle: |Y - Y_ref| <= 2e-6 * sum_i |X[t,i] * W_hat[i,o]| + 1e-30 per output
(the fp32 rounding of d_in products and additions stays far below it; one wrong, missing or
doubled term of typical size exceeds it), and the GPU result is bit-reproducible.
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
    B.lib()
    return dict(B=B, P=P, synth=synth, ws=B.Workspace(DEV), orc=orc)


def _np(t):
    return t.detach().cpu().numpy()


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _what(W, cent, codes, bits, out_idx):
    lut = cent.astype(np.float16).astype(np.float64)
    what = np.take_along_axis(lut, codes.astype(np.int64), axis=1)
    w16 = W.astype(np.float16).astype(np.float64)
    keep = np.zeros(W.shape, bool)
    keep[(bits < 1) | (bits > 4), :] = True
    if out_idx is not None and len(out_idx):
        keep.reshape(-1)[out_idx] = True
    return np.where(keep, w16, what)


def _check_product(Y, Yref, X, What):
    bound = 2e-6 * (np.abs(X.astype(np.float64)) @ np.abs(What)) + 1e-30
    err = np.abs(Y.astype(np.float64) - Yref)
    assert (err <= bound).all(), float((err / bound).max())


def test_gather_channels(env):
    B = env["B"]
    rng = np.random.default_rng(0)
    for dtype in (np.float16, np.float32):
        W = rng.normal(0, 1, (40, 333)).astype(dtype)
        idx = np.array([3, 17, 39, 0], np.int32)
        out = torch.empty((4, 333), dtype=torch.float16, device=DEV)
        B.gather_channels(_dev(W), _dev(idx), out)
        assert np.array_equal(_np(out), W[idx].astype(np.float16))
    B.gather_channels(_dev(W), torch.empty(0, dtype=torch.int32, device=DEV),
                      torch.empty((0, 333), dtype=torch.float16, device=DEV))      # nothing to do


@pytest.mark.parametrize("d_in,d_out,n", [(7, 5, 0), (7, 5, 9), (64, 1000, 3000), (300, 4096, 20000)])
def test_outliers_by_column(env, d_in, d_out, n):
    B, ws = env["B"], env["ws"]
    rng = np.random.default_rng(n)
    cent = rng.normal(0, 0.1, (d_in, 16)).astype(np.float32)
    codes = rng.integers(0, 16, (d_in, d_out)).astype(np.uint8)
    idx = np.sort(rng.choice(d_in * d_out, n, replace=False)).astype(np.int32)
    if n > 20:                                   # one crowded column: a long stretch to order
        crowd = (np.arange(min(d_in, 40)) * d_out + 3).astype(np.int32)
        idx = np.unique(np.concatenate([idx, crowd]))
        n = len(idx)
    val = rng.normal(0, 0.1, n).astype(np.float16)
    colptr = torch.full((d_out + 1,), -1, dtype=torch.int32, device=DEV)
    row = torch.full((max(n, 1),), -1, dtype=torch.int32, device=DEV)
    delta = torch.zeros(max(n, 1), dtype=torch.float32, device=DEV)
    B.outliers_by_column(_dev(idx) if n else None, _dev(val) if n else None, n, d_in, d_out, _dev(cent), _dev(codes),
                         colptr, row, delta, ws)
    i, o = idx // d_out, idx % d_out
    order = np.lexsort((i, o))                   # by column, then channel
    want_ptr = np.concatenate([[0], np.cumsum(np.bincount(o, minlength=d_out))]).astype(np.int32)
    level = cent.astype(np.float16)[i, codes[i, o]].astype(np.float32)
    want_delta = (val.astype(np.float32) - level)[order]
    assert np.array_equal(_np(colptr), want_ptr)
    assert np.array_equal(_np(row)[:n], i[order].astype(np.int32))
    assert np.array_equal(_np(delta)[:n], want_delta)


@pytest.mark.parametrize("bit_set,avg,d_in,d_out", [((1, 2), 1.5, 96, 50), ((2, 3, 4), 3.0, 300, 2048 + 40),
                                                    ((3, 4), 3.5, 520, 4096 + 8), ((1, 2, 3, 4), 2.5, 260, 33),
                                                    ((2, 3, 4), 3.3, 1100, 2000)])
def test_lut_matvec_parity_end_to_end(env, bit_set, avg, d_in, d_out):
    """Quantize with the library (checked against the oracle elsewhere), deploy, multiply;
    the oracle multiplies with the weight rebuilt from W, levels, codes and outlier indices."""
    B, P, ws, orc = env["B"], env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(d_in + d_out)
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = W.astype(np.float16)
    Xcal = (rng.normal(0, 1, (256, d_in)) * np.exp(rng.normal(0, 0.5, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(Xcal), ws)
    r = P.quantize_layer(_dev(W), sumsq, bit_set, avg, rho_act_ppm=20000, rho_q_ppm=10000, iters=5, ws=ws,
                         transposed=True)
    dep = P.prepare_deployment(r, ws)
    bits, cent, codes, out_idx = _np(r.bits), _np(r.centroids), _np(r.codes), _np(r.out_idx).astype(np.int64)
    What = _what(W, cent, codes, bits, out_idx)
    for m in (1, 3, 5, 8):                        # groups of 1, 2 and 4 tokens, with ragged last groups
        X = rng.normal(0, 1, (m, d_in)).astype(np.float16)
        Y = _np(P.lut_matvec(dep, _dev(X), ws))
        Yref = orc.lut_matvec(X, W, cent, codes, bits, out_idx)
        assert np.allclose(Yref, X.astype(np.float64) @ What, rtol=1e-12, atol=1e-12)
        _check_product(Y, Yref, X, What)
        assert np.array_equal(Y, _np(P.lut_matvec(dep, _dev(X), ws)))          # reproducible
    # a strided input and output
    Xw = torch.zeros((2, d_in + 8), dtype=torch.float16, device=DEV)
    Xw[:, :d_in] = _dev(X[:2] if m >= 2 else np.repeat(X, 2, 0))
    Yw = torch.full((2, d_out + 5), 7.0, dtype=torch.float32, device=DEV)
    B.lut_matvec(Xw[:, :d_in], d_out, dep.bit_set, dep.counts, dep.packed, dep.chan_idx, dep.lut, dep.act_idx,
                 dep.W_act, dep.colptr, dep.row_idx, dep.delta, Yw[:, :d_out], ws)
    assert np.array_equal(_np(Yw[:, :d_out]), Y[:2]) and (_np(Yw[:, d_out:]) == 7.0).all()


@pytest.mark.parametrize("bit_set,avg,d_in,d_out,per_channel", [((2, 3, 4), 3.0, 300, 2048 + 40, False),
                                                                ((1, 2, 3, 4), 2.5, 130, 28672, False),
                                                                ((3, 4), 3.5, 520, 4096 + 8, True),
                                                                ((2, 3), 2.5, 96, 50, False)])
def test_shared_tables_route_equals_rebuilt_tables(env, bit_set, avg, d_in, d_out, per_channel):
    """The layer quantized with the preliminary K-means handing its per-channel tables to the
    final one (the default) and with the final one building them again: every output the same
    bit for bit (levels, codes, O_q, stored format, errors).  d_out = 50 is a shape the shared
    route does not take (rows not whole groups of 4): both calls then run the same kernels."""
    P, ws = env["P"], env["ws"]
    rng = np.random.default_rng(3 * d_in + d_out)
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = _dev(W.astype(np.float16))
    Xcal = (rng.normal(0, 1, (128, d_in)) * np.exp(rng.normal(0, 0.5, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(Xcal), ws)
    runs = [P.quantize_layer(W, sumsq, bit_set, avg, rho_act_ppm=20000, rho_q_ppm=10000, iters=4, ws=ws,
                             transposed=True, with_error=True, oq_per_channel=per_channel, share_tables=share)
            for share in (True, False)]
    a, b = runs
    for name in ("bits", "centroids", "codes", "out_idx", "out_val", "err_ch", "err_total"):
        x, y = _np(getattr(a, name)), _np(getattr(b, name))
        assert x.tobytes() == y.tobytes(), name
    assert a.counts == b.counts
    for name in ("packed", "chan_idx", "lut"):
        for x, y in zip(getattr(a, name), getattr(b, name)):
            assert (x is None) == (y is None)
            if x is not None:
                assert _np(x).tobytes() == _np(y).tobytes(), name


def _fp16_run_sums(X, cent, codes, bits, bit_set, run):
    """The packed part of the FP16-sum product as its entry point defines it: products rounded
    to FP16, runs of `run` consecutive rows of a width added in FP16 one after the other; the
    run sums are returned added up exactly, with the sum of their magnitudes."""
    m, d_out = X.shape[0], codes.shape[1]
    lut16 = cent.astype(np.float16)
    total = np.zeros((m, d_out)); mag = np.zeros((m, d_out))
    for b in bit_set:
        chans = np.flatnonzero(bits == b)
        for s in range(0, len(chans), run):
            acc = np.zeros((m, d_out), np.float16)
            for i in chans[s:s + run]:
                lv = lut16[i, codes[i].astype(np.int64)]
                prod = (X[:, i:i + 1].astype(np.float32) * lv[None, :].astype(np.float32)).astype(np.float16)
                acc = (acc.astype(np.float64) + prod.astype(np.float64)).astype(np.float16)   # one rounding
            total += acc.astype(np.float64)
            mag += np.abs(acc.astype(np.float64))
    return total, mag


@pytest.mark.parametrize("bit_set,avg,d_in,d_out", [((2, 3, 4), 3.0, 300, 2048 + 40), ((3, 4), 3.5, 520, 4096 + 8),
                                                    ((1, 2, 3, 4), 2.5, 260, 33), ((2, 3, 4), 3.3, 1100, 2000)])
def test_lut_matvec_fp16_sums(env, bit_set, avg, d_in, d_out):
    """cmpq_lut_matvec_group_fp16acc: equal to the emulation of its three steps (FP16 products,
    FP16 run sums at one of the three run lengths, fp32 after that) up to the fp32 rounding of
    the last step - one wrong, missing or doubled term of typical size exceeds that bar -, within
    its documented bound of the exact product, and reproducible."""
    B, P, ws, orc = env["B"], env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(7 * d_in + d_out)
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = W.astype(np.float16)
    Xcal = (rng.normal(0, 1, (256, d_in)) * np.exp(rng.normal(0, 0.5, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(Xcal), ws)
    r = P.quantize_layer(_dev(W), sumsq, bit_set, avg, rho_act_ppm=20000, rho_q_ppm=10000, iters=5, ws=ws,
                         transposed=True)
    dep = P.prepare_deployment(r, ws)
    bits, cent, codes, out_idx = _np(r.bits), _np(r.centroids), _np(r.codes), _np(r.out_idx).astype(np.int64)
    What = _what(W, cent, codes, bits, out_idx)
    lut16 = cent.astype(np.float16).astype(np.float64)
    level = np.take_along_axis(np.where(np.isfinite(lut16), lut16, 0.0), codes.astype(np.int64), axis=1)
    packed_rows = (bits >= 1) & (bits <= 4)
    # what O_act and O_q add to the packed part: the FP16 rows, and weight minus level per entry
    extra = np.zeros(W.shape)
    extra[~packed_rows] = W[~packed_rows].astype(np.float64)
    if len(out_idx):
        extra.reshape(-1)[out_idx] = (W.astype(np.float64) - level).reshape(-1)[out_idx]
    call = P.group_products([dep], fp16acc=True)
    for m in (1, 3):
        X = rng.normal(0, 1, (m, d_in)).astype(np.float16)
        Y = torch.empty((m, d_out), dtype=torch.float32, device=DEV)
        call([_dev(X)], [Y], ws)
        Yg = _np(Y).astype(np.float64)
        X64 = X.astype(np.float64)
        rest = X64 @ extra
        rest_mag = np.abs(X64) @ np.abs(extra)
        best = None
        for run in (32, 16, 8):
            total, mag = _fp16_run_sums(X, cent, codes, bits, bit_set, run)
            bound = 2e-6 * (mag + rest_mag) + 1e-30
            ratio = float((np.abs(Yg - (total + rest)) / bound).max())
            best = ratio if best is None else min(best, ratio)
            if ratio <= 1.0:
                # the documented bound against the exact product, for this run length
                Yref = orc.lut_matvec(X, W, cent, codes, bits, out_idx)
                packed_mag = np.abs(X64[:, packed_rows]) @ np.abs(level[packed_rows])
                loose = (run + 1) * 2.0 ** -11 * packed_mag + 2e-6 * (np.abs(X64) @ np.abs(What)) + 1e-30
                assert (np.abs(Yg - Yref) <= loose).all()
                break
        assert best is not None and best <= 1.0, best
        Y2 = torch.empty_like(Y)
        call([_dev(X)], [Y2], ws)
        assert np.array_equal(_np(Y), _np(Y2))                                  # reproducible
    # the fp32 product of the same layer is untouched by the variant's existence
    Yf = _np(P.lut_matvec(dep, _dev(X), ws))
    _check_product(Yf, orc.lut_matvec(X, W, cent, codes, bits, out_idx), X, What)


def test_lut_matvec_without_outliers_and_all_protected(env):
    B, P, ws, orc = env["B"], env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(3)
    d_in, d_out = 150, 700
    W = rng.normal(0, 0.05, (d_in, d_out)).astype(np.float16)
    X = rng.normal(0, 1, (2, d_in)).astype(np.float16)
    sumsq = _dev(rng.random(d_in).astype(np.float32) + 0.1)
    # no outliers of either kind
    r = P.quantize_layer(_dev(W), sumsq, (2, 3), 2.5, rho_act_ppm=0, rho_q_ppm=0, iters=3, ws=ws, transposed=True)
    dep = P.prepare_deployment(r, ws)
    assert dep.act_idx.numel() == 0 and dep.row_idx.numel() == 0
    What = _what(W, _np(r.centroids), _np(r.codes), _np(r.bits), None)
    Y = _np(P.lut_matvec(dep, _dev(X), ws))
    _check_product(Y, X.astype(np.float64) @ What, X, What)
    # every channel protected: the plain FP16 product
    idx = torch.arange(d_in, dtype=torch.int32, device=DEV)
    W_act = torch.empty((d_in, d_out), dtype=torch.float16, device=DEV)
    B.gather_channels(_dev(W), idx, W_act)
    Y = torch.empty((2, d_out), dtype=torch.float32, device=DEV)
    B.lut_matvec(_dev(X), d_out, (2, 3), (0, 0), [None, None], [None, None], [None, None], idx, W_act,
                 None, None, None, Y, ws)
    Wd = W.astype(np.float64)
    _check_product(_np(Y), X.astype(np.float64) @ Wd, X, Wd)


def test_lut_matvec_full_size_layer(env):
    """down_proj of the 70B-shaped block at full size, one token: every output against the oracle."""
    P, synth, ws, orc = env["P"], env["synth"], env["ws"], env["orc"]
    wl = synth.workload("block70b")
    layer = next(l for l in wl.layers if l.name == "down_proj")
    W = synth.make_weight(layer.d_out, layer.d_in, "f16", 11, DEV)          # [d_out, d_in] as a framework keeps it
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    sumsq = (torch.rand(layer.d_in, generator=g) + 0.05).to(DEV)
    r = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, 3, ws)
    dep = P.prepare_deployment(r, ws)
    X = torch.randn((1, layer.d_in), generator=g).to(torch.float16).to(DEV)
    Y = _np(P.lut_matvec(dep, X, ws))
    Wt, cent, codes, bits = _np(r.W_t), _np(r.centroids), _np(r.codes), _np(r.bits)
    out_idx = _np(r.out_idx).astype(np.int64)
    Yref = orc.lut_matvec(_np(X), Wt, cent, codes, bits, out_idx)
    What = _what(Wt, cent, codes, bits, out_idx)
    _check_product(Y, Yref, _np(X), What)


def _deploy_random_layer(env, rng, d_in, d_out, bit_set, avg, rho_act=20000, rho_q=10000):
    P, ws = env["P"], env["ws"]
    W = rng.normal(0, 0.02, (d_in, d_out))
    W[rng.random(W.shape) < 0.01] *= 10
    W = W.astype(np.float16)
    sumsq = _dev((rng.random(d_in) ** 3 + 0.01).astype(np.float32))
    r = P.quantize_layer(_dev(W), sumsq, bit_set, avg, rho_act_ppm=rho_act, rho_q_ppm=rho_q, iters=3, ws=ws,
                         transposed=True)
    return W, r, P.prepare_deployment(r, ws)


def test_grouped_products_equal_single_calls_and_oracle(env):
    """Products launched together (three that read one input, as query/key/value do, and two
    with inputs of their own, one without outliers) give bit for bit what one call per layer
    gives, and so match the oracle."""
    P, ws, orc = env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(21)
    shapes = [(520, 2048 + 40, (2, 3, 4), 3.2, 20000, 10000), (520, 300, (3, 4), 3.5, 20000, 10000),
              (520, 33, (1, 2), 1.5, 20000, 10000), (96, 4100, (2, 3), 2.5, 0, 0),
              (1100, 2000, (2, 3, 4), 2.4, 4500, 500)]
    layers = [_deploy_random_layer(env, rng, *s) for s in shapes]
    deps = [d for _, _, d in layers]
    group = P.group_products(deps)
    for m in (1, 3):
        shared = _dev(rng.normal(0, 1, (m, 520)).astype(np.float16))
        Xs = [shared, shared, shared, _dev(rng.normal(0, 1, (m, 96)).astype(np.float16)),
              _dev(rng.normal(0, 1, (m, 1100)).astype(np.float16))]
        Ys = [torch.full((m, d.d_out), 3.0, dtype=torch.float32, device=DEV) for d in deps]
        group(Xs, Ys, ws)
        torch.cuda.synchronize()
        for (W, r, dep), X, Y in zip(layers, Xs, Ys):
            single = P.lut_matvec(dep, X, ws)
            assert torch.equal(single, Y)
            What = _what(W, _np(r.centroids), _np(r.codes), _np(r.bits), _np(r.out_idx).astype(np.int64))
            Yref = orc.lut_matvec(_np(X), W, _np(r.centroids), _np(r.codes), _np(r.bits),
                                  _np(r.out_idx).astype(np.int64))
            _check_product(_np(Y), Yref, _np(X), What)
    # a group of one, and the largest group
    one = P.group_products(deps[:1])
    Y1 = torch.empty((1, deps[0].d_out), dtype=torch.float32, device=DEV)
    one([Xs[0][:1]], [Y1], ws)
    assert torch.equal(Y1, P.lut_matvec(deps[0], Xs[0][:1], ws))
    eight = P.group_products([deps[1]] * 8)
    Y8 = [torch.empty((1, deps[1].d_out), dtype=torch.float32, device=DEV) for _ in range(8)]
    eight([Xs[1][:1]] * 8, Y8, ws)
    want = P.lut_matvec(deps[1], Xs[1][:1], ws)
    assert all(torch.equal(y, want) for y in Y8)
    with pytest.raises(ValueError):
        P.group_products([deps[1]] * 9)


def test_grouped_products_full_size_block(env):
    """The products of the 70B-shaped block that read one input, grouped as the benchmark
    groups them (query/key/value; gate/up), against one call per layer."""
    P, synth, ws = env["P"], env["synth"], env["ws"]
    wl = synth.workload("block70b")
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    for names in (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj")):
        deps = []
        for name in names:
            layer = [l for l in wl.layers if l.name == name][0]
            W = synth.make_weight(layer.d_out, layer.d_in, "f16", 11 + len(deps), DEV)
            sumsq = (torch.rand(layer.d_in, generator=g) + 0.05).to(DEV)
            r = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, 2, ws)
            deps.append(P.prepare_deployment(r, ws))
            del r, W
        X = torch.randn((1, deps[0].d_in), generator=g).to(torch.float16).to(DEV)
        Ys = [torch.empty((1, d.d_out), dtype=torch.float32, device=DEV) for d in deps]
        P.group_products(deps)([X] * len(deps), Ys, ws)
        for d, Y in zip(deps, Ys):
            assert torch.equal(Y, P.lut_matvec(d, X, ws))
        del deps


@pytest.mark.parametrize("seed", range(int(os.environ.get("CMPQ_RANDOM_CASES", "12"))))
def test_randomized_products_and_groups(env, seed):
    """Random shapes (ragged tiles, odd d_out), bit sets down to one bit, budgets, outlier fractions
    and token counts; 1 to 4 layers launched as a group, each product against the oracle and
    against its own single call."""
    P, ws, orc = env["P"], env["ws"], env["orc"]
    rng = np.random.default_rng(7000 + seed)
    n_layers = int(rng.integers(1, 5))
    m = int(rng.integers(1, 4))
    layers, Xs = [], []
    for _ in range(n_layers):
        d_in = int(rng.integers(8, 400))
        d_out = int(rng.choice([rng.integers(1, 64), rng.integers(64, 2100), rng.integers(2100, 6500)]))
        lo = int(rng.integers(1, 4))
        hi = int(rng.integers(lo + 1, 5))
        bit_set = tuple(range(lo, hi + 1))
        avg = float(np.round(rng.uniform(lo, hi), 2))
        layers.append(_deploy_random_layer(env, rng, d_in, d_out, bit_set, avg, int(rng.choice([0, 4500, 50000])),
                                           int(rng.choice([0, 500, 20000]))))
        Xs.append(_dev(rng.normal(0, 1, (m, d_in)).astype(np.float16)))
    deps = [d for _, _, d in layers]
    Ys = [torch.full((m, d.d_out), -5.0, dtype=torch.float32, device=DEV) for d in deps]
    P.group_products(deps)(Xs, Ys, ws)
    torch.cuda.synchronize()
    for (W, r, dep), X, Y in zip(layers, Xs, Ys):
        assert torch.equal(Y, P.lut_matvec(dep, X, ws))
        out_idx = _np(r.out_idx).astype(np.int64)
        What = _what(W, _np(r.centroids), _np(r.codes), _np(r.bits), out_idx)
        Yref = orc.lut_matvec(_np(X), W, _np(r.centroids), _np(r.codes), _np(r.bits), out_idx)
        _check_product(_np(Y), Yref, _np(X), What)


def test_products_replayed_from_a_hip_graph_equal_eager_launches(env):
    """The launches of a token recorded once (two groups, three layers) and replayed four times
    with new inputs, eager work and synchronisations in between: every replay equals the eager
    result of the same inputs bit for bit."""
    P, B = env["P"], env["B"]
    ws = B.Workspace(DEV)
    rng = np.random.default_rng(31)
    deps = [_deploy_random_layer(env, rng, d_in, d_out, (2, 3, 4), 3.0)[2] for d_in, d_out in
            ((96, 512), (96, 160), (160, 96))]
    xa = torch.zeros((1, 96), dtype=torch.float16, device=DEV)
    xb = torch.zeros((1, 160), dtype=torch.float16, device=DEV)
    ys = [torch.zeros((1, d.d_out), dtype=torch.float32, device=DEV) for d in deps]
    steps = [(P.group_products(deps[:2]), [xa, xa], ys[:2]), (P.group_products(deps[2:]), [xb], ys[2:])]
    graph = P.capture_products(steps, ws)
    gen = torch.Generator(device=DEV).manual_seed(11)
    for it in range(4):
        xa.copy_(torch.randn((1, 96), generator=gen, device=DEV).to(torch.float16))
        xb.copy_(torch.randn((1, 160), generator=gen, device=DEV).to(torch.float16))
        graph.replay()
        torch.cuda.synchronize()
        got = [y.clone() for y in ys]
        for y in ys:
            y.fill_(-1.0)
        want = [P.lut_matvec(d, x, B.Workspace(DEV)) for d, x in zip(deps, (xa, xa, xb))]   # eager, own workspace
        torch.cuda.synchronize()
        for g, w in zip(got, want):
            assert torch.equal(g, w), it
