"""GPU-vs-oracle parity of the look-up tables in 4 bits (Sec. 5.1 / Tab. 7), through the C ABI:
cmpq_lut4_quantize, then the unchanged cmpq_pack / cmpq_dequant_error / product with the rebuilt
tables.

Bars: codes, range and rebuilt levels come from single IEEE fp32 operations and one exact sum on
both sides - bit-exact; the FP16 tables written by cmpq_pack are bit-exact; the error follows the
bar of the main parity tests (1e-4 relative on the layer total).
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


def _gpu_lut4(env, cent, bits):
    B = env["B"]
    d_in = cent.shape[0]
    codes4 = torch.full((d_in, 16), 0xee, dtype=torch.uint8, device=DEV)
    rng = torch.full((2,), -3.0, dtype=torch.float32, device=DEV)
    cq = torch.full((d_in, 16), -3.0, dtype=torch.float32, device=DEV)
    B.lut4_quantize(_dev(cent), _dev(bits), codes4, rng, cq)
    torch.cuda.synchronize()
    return _np(codes4), _np(rng), _np(cq)


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
    got = _gpu_lut4(env, cent, bits)
    want = env["orc"].lut4(cent, bits)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])


def test_lut4_layer_end_to_end(env):
    """Quantize a layer, put its tables on the 4-bit grid, write the stored format again and
    measure the error and the product: everything against the oracle fed with the same chain."""
    P, orc, ws = env["P"], env["orc"], env["ws"]
    r = np.random.default_rng(9)
    d_in, d_out = 300, 1024
    W = (r.standard_t(4, size=(d_in, d_out)) * 0.02).astype(np.float16)
    X = (r.normal(0, 1, (128, d_in)) * np.exp(r.normal(0, 0.7, d_in))).astype(np.float16)
    _, sumsq = P.activation_stats(_dev(X), ws)
    res = P.quantize_layer(_dev(W), sumsq, (2, 3, 4), 2.8, 4500, 2000, 6, ws, with_error=True, transposed=True)
    codes4, rng, q = P.tables_in_4_bits(res, ws, with_error=True)
    torch.cuda.synchronize()
    bits, codes = _np(res.bits), _np(res.codes)
    o4, orng, ocq = orc.lut4(_np(res.centroids), bits)
    assert np.array_equal(_np(codes4), o4) and np.array_equal(_np(rng), orng) and np.array_equal(_np(q.centroids), ocq)
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
    assert tot[1] >= _np(res.err_total)[1]                          # coarser tables cannot reduce the error
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
    got = _gpu_lut4(env, cent, bits)
    want = env["orc"].lut4(cent, bits)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])
