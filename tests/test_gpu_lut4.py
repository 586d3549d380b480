"""GPU-vs-oracle parity of the look-up tables in 4 bits (Sec. 5.1 / Tab. 7), through the C ABI:
cmpq_lut4_quantize, then the unchanged cmpq_pack / cmpq_dequant_error / product with the rebuilt
tables.

Bars: in both modes codes, table (levels, or range of the uniform grid) and rebuilt levels are
bit-exact - the per-layer table comes from exact integer sums over FP16 values and one fp64
division per level on the GPU, fp64 sums of the same values in the oracle (equal as long as a
sum stays below 2^53 units of 2^-24, which every case here does); the uniform grid from single
IEEE fp32 operations.  The FP16 tables written by cmpq_pack are bit-exact; the error follows
the bar of the main parity tests (1e-4 relative on the layer total).
"""
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


def _gpu_lut4(env, cent, bits, uniform=False, iters=20):
    """(codes4, table, centroids_q); for the uniform grid `table` is cut to (minimum, step)."""
    B = env["B"]
    d_in = cent.shape[0]
    codes4 = torch.full((d_in, 16), 0xee, dtype=torch.uint8, device=DEV)
    table = torch.full((16,), -3.0, dtype=torch.float32, device=DEV)
    cq = torch.full((d_in, 16), -3.0, dtype=torch.float32, device=DEV)
    B.lut4_quantize(_dev(cent), _dev(bits), codes4, table, cq, env["ws"],
                    B.LUT4_UNIFORM if uniform else B.LUT4_CODEBOOK, iters)
    torch.cuda.synchronize()
    t = _np(table)
    if uniform:
        assert np.all(t[2:] == -3.0)                                # left alone
        t = t[:2]
    return _np(codes4), t, _np(cq)


def _same(got, want):
    return all(np.array_equal(g, w) for g, w in zip(got, want))


@pytest.mark.parametrize("seed", range(12))
def test_lut4_parity_random_tables(env, seed):
    r = np.random.default_rng(40 + seed)
    d_in = int(r.choice([1, 7, 64, 333, 4096]))
    bits = r.choice(np.array([1, 2, 3, 4, 16], np.uint8), d_in)
    if seed == 3:
        bits[:] = 16                                               # nothing quantized
    cent = np.full((d_in, 16), np.inf, np.float32)
    scale = float(r.choice([1e-3, 0.03, 1.0, 1e20, 1e-30]))
    for i, b in enumerate(bits):
        if b <= 4:
            vals = np.sort(r.normal(0, scale, 1 << b)).astype(np.float32)
            if seed == 5:
                vals[:] = np.float32(0.125)                         # every centre the same: step 0
            cent[i, :1 << b] = vals
    assert _same(_gpu_lut4(env, cent, bits, uniform=True), env["orc"].lut4(cent, bits))
    if scale in (1e20, 1e-30):
        # beyond FP16's range the stored centres would be infinite: finite ones in a narrower band
        # (narrow enough that the oracle's fp64 sums stay exact)
        cent = np.where(np.isfinite(cent), np.clip(cent, -100.0, 100.0), cent).astype(np.float32)
    iters = int(r.choice([0, 1, 5, 20, 60]))
    assert _same(_gpu_lut4(env, cent, bits, iters=iters), env["orc"].lut4_codebook(cent, bits, iters))


def test_lut4_codebook_awkward_tables(env):
    """The per-layer table on inputs that strain the clustering: fewer distinct centres than
    levels, mass ties between levels, -0 and +0, subnormal and largest FP16 values, centres that
    FP16 rounds onto each other, a single channel, and no channel at all."""
    orc = env["orc"]
    r = np.random.default_rng(77)
    cases = []
    few = np.full((50, 16), np.inf, np.float32)
    few[:, :4] = np.array([-0.5, 0.0, 0.25, 1.0], np.float32)
    cases.append((few, np.full(50, 2, np.uint8)))
    grid = np.full((64, 16), np.inf, np.float32)                   # every value midway between its neighbours
    grid[:, :16] = (np.arange(16, dtype=np.float32) - 8) / 8
    cases.append((grid, np.full(64, 4, np.uint8)))
    zeros = np.full((9, 16), np.inf, np.float32)
    zeros[:, :8] = np.array([-1.0, -0.0, 0.0, 6e-8, 1.2e-7, 1e-3, 65504.0, -65504.0], np.float32)
    cases.append((zeros, np.full(9, 3, np.uint8)))
    close = np.full((40, 16), np.inf, np.float32)
    close[:, :8] = (1.0 + r.normal(0, 1e-5, (40, 8))).astype(np.float32)     # FP16 merges most of them
    cases.append((close, np.full(40, 3, np.uint8)))
    one = np.full((1, 16), np.inf, np.float32)
    one[0, :2] = [-0.3, 0.7]
    cases.append((one, np.array([1], np.uint8)))
    cases.append((np.full((5, 16), np.inf, np.float32), np.full(5, 16, np.uint8)))
    for cent, bits in cases:
        for iters in (0, 3, 20):
            assert _same(_gpu_lut4(env, cent, bits, iters=iters), orc.lut4_codebook(cent, bits, iters))


@pytest.mark.parametrize("uniform", [False, True])
def test_lut4_layer_end_to_end(env, uniform):
    """Quantize a layer, put its tables into 4 bits (per-layer table, or the uniform grid), write
    the stored format again and measure the error and the product: everything against the
    oracle fed with the same chain."""
    P, orc, ws, B = env["P"], env["orc"], env["ws"], env["B"]
    r = np.random.default_rng(9)
    d_in, d_out = 300, 1024
    W = (r.standard_t(4, size=(d_in, d_out)) * 0.02).astype(np.float16)
    X = (r.normal(0, 1, (128, d_in)) * np.exp(r.normal(0, 0.7, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(X), ws)
    res = P.quantize_layer(_dev(W), sumsq, (2, 3, 4), 2.8, 4500, 2000, 6, ws, with_error=True, transposed=True)
    codes4, table, q = P.tables_in_4_bits(res, ws, with_error=True, mode=B.LUT4_UNIFORM if uniform else B.LUT4_CODEBOOK)
    torch.cuda.synchronize()
    bits, codes = _np(res.bits), _np(res.codes)
    if uniform:
        o4, otab, ocq = orc.lut4(_np(res.centroids), bits)
        assert np.array_equal(_np(table)[:2], otab)
    else:
        o4, otab, ocq = orc.lut4_codebook(_np(res.centroids), bits)
        assert np.array_equal(_np(table), otab)
    assert np.array_equal(_np(codes4), o4) and np.array_equal(_np(q.centroids), ocq)
    for j, b in enumerate((2, 3, 4)):
        if q.packed[j] is None:
            continue
        opacked, ochan, olut = orc.pack(codes, bits, ocq, b)
        assert np.array_equal(_np(q.packed[j]).view(np.uint32), opacked)
        assert np.array_equal(_np(q.lut[j]).view(np.uint16), olut.view(np.uint16))
        assert np.array_equal(_np(q.chan_idx[j]), ochan)
    out_idx = _np(res.out_idx).astype(np.int64)
    oerr, otot = orc.dequant_error(W, ocq, codes, bits, out_idx, _np(res.sumsq))
    tot = _np(q.err_total)
    assert abs(tot[0] - otot[0]) <= 1e-4 * otot[0] and np.allclose(_np(q.err_ch), oerr, rtol=1e-9, atol=1e-30)
    assert tot[1] >= _np(res.err_total)[1] * (1 - 1e-3)             # coarser tables do not reduce the error
    if not uniform:
        assert tot[1] <= 1.5 * _np(res.err_total)[1]                # Tab. 7: a small loss
    # the product reads the rebuilt tables
    dep = P.prepare_deployment(q, ws)
    Xt = r.normal(0, 1, (2, d_in)).astype(np.float16)
    Y = _np(P.lut_matvec(dep, _dev(Xt), ws)).astype(np.float64)
    Yref = orc.lut_matvec(Xt, W, ocq, codes, bits, out_idx)
    assert np.max(np.abs(Y - Yref)) <= 1e-4 * np.max(np.abs(Yref))


def test_lut4_full_size_layer(env):
    """The tables of down_proj of the 70B-shaped block (28672 channels)."""
    r = np.random.default_rng(2)
    d_in = 28672
    bits = r.choice(np.array([2, 3, 4, 16], np.uint8), d_in, p=[0.2, 0.4, 0.395, 0.005])
    cent = np.full((d_in, 16), np.inf, np.float32)
    for b in (2, 3, 4):
        rows = np.nonzero(bits == b)[0]
        cent[rows[:, None], np.arange(1 << b)[None, :]] = np.sort(
            r.normal(0, 0.02, (len(rows), 1 << b)).astype(np.float32), axis=1)
    assert _same(_gpu_lut4(env, cent, bits, uniform=True), env["orc"].lut4(cent, bits))
    assert _same(_gpu_lut4(env, cent, bits), env["orc"].lut4_codebook(cent, bits))
