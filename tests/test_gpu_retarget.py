"""Retargeting a layer to other average widths from runs kept per width (the cost the paper's
closing section names), through the C ABI: cmpq_select_by_width and the unchanged rest of the path.

A channel's preliminary K-means depends on its own weights and width only, so the route
through the kept runs must give the very results of the direct route - and both must match
the oracle, which only knows the direct route (Sec. 3.2.1 / 3.2.2 in order).
Bars: integers, bytes and levels bit-identical between the two GPU routes; against the
oracle the bars of the main parity tests (levels 1e-5 relative, codes 1e-4 mismatches).
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


def _same(a, b):
    assert np.array_equal(_np(a.bits), _np(b.bits)) and a.counts == b.counts
    assert np.array_equal(_np(a.act_idx), _np(b.act_idx))
    assert np.array_equal(_np(a.centroids_prelim), _np(b.centroids_prelim))
    assert np.array_equal(_np(a.codes_prelim), _np(b.codes_prelim))
    assert np.array_equal(_np(a.out_idx), _np(b.out_idx)) and np.array_equal(_np(a.out_val), _np(b.out_val))
    assert np.array_equal(_np(a.centroids), _np(b.centroids)) and np.array_equal(_np(a.codes), _np(b.codes))
    for x, y in zip(a.packed + a.chan_idx + a.lut, b.packed + b.chan_idx + b.lut):
        assert (x is None) == (y is None)
        if x is not None:
            assert np.array_equal(_np(x).view(np.uint8), _np(y).view(np.uint8))
    assert np.array_equal(_np(a.err_ch), _np(b.err_ch)) and np.array_equal(_np(a.err_total), _np(b.err_total))


@pytest.mark.parametrize("dtype,d_in,d_out", [("f16", 300, 1024), ("f32", 257, 520), ("f16", 96, 4104)])
def test_cache_route_equals_direct_route_and_oracle(env, dtype, d_in, d_out):
    P, orc = env["P"], env["orc"]
    rng = np.random.default_rng(d_in + d_out)
    W = (rng.standard_t(4, size=(d_out, d_in)) * 0.02).astype(np.float16 if dtype == "f16" else np.float32)
    X = (rng.normal(0, 1, size=(200, d_in)) * rng.lognormal(0, 1, size=d_in)).astype(W.dtype)
    Wd = torch.from_numpy(W).to(DEV)
    _, sumsq = P.activation_stats(torch.from_numpy(X).to(DEV), env["ws"])
    bit_set, iters = (2, 3, 4), 6
    cache = P.build_width_cache(Wd, bit_set, iters, env["ws"])
    for avg, rho_act, rho_q in [(2.2, 4500, 500), (3.0, 4500, 500), (3.63, 10000, 2000), (4.0, 0, 0), (2.0, 4500, 0)]:
        a = P.quantize_layer_from_cache(cache, sumsq, avg, rho_act, rho_q, env["ws"], with_error=True,
                                        keep_prelim=True)
        b = P.quantize_layer(Wd, sumsq, bit_set, avg, rho_act, rho_q, iters, env["ws"], with_error=True,
                             keep_prelim=True)
        torch.cuda.synchronize()
        _same(a, b)
    # the variant with the final pass continued from the preliminary levels takes both routes alike
    a = P.quantize_layer_from_cache(cache, sumsq, 3.0, 4500, 500, env["ws"], with_error=True, keep_prelim=True,
                                    iters_final_from_prelim=3)
    b = P.quantize_layer(Wd, sumsq, bit_set, 3.0, 4500, 500, iters, env["ws"], with_error=True, keep_prelim=True,
                         iters_final_from_prelim=3)
    torch.cuda.synchronize()
    _same(a, b)
    # the last budgets against the oracle's direct route
    o = orc.quantize_layer(np.ascontiguousarray(W.T), X, bit_set, 3.63, 10000, 2000, iters)
    a = P.quantize_layer_from_cache(cache, sumsq, 3.63, 10000, 2000, env["ws"], with_error=True)
    torch.cuda.synchronize()
    assert np.array_equal(_np(a.bits), o["bits"]) and np.array_equal(_np(a.act_idx), o["act_idx"])
    assert np.array_equal(_np(a.out_idx).astype(np.int64), o["out_idx"])
    c, oc = _np(a.centroids), o["centroids"]
    fin = np.isfinite(oc)
    assert np.array_equal(np.isfinite(c), fin)
    assert np.max(np.abs(c[fin] - oc[fin]) / np.maximum(np.abs(oc[fin]), 1e-30)) <= 1e-5
    assert (_np(a.codes) != o["codes"]).mean() <= 1e-4
    for j, bw in enumerate(bit_set):
        if a.packed[j] is not None:
            assert np.array_equal(_np(a.packed[j]).view(np.uint32), o["packs"][bw][0])
    tot = _np(a.err_total)
    assert abs(tot[0] - o["totals"][0]) <= 1e-4 * o["totals"][0]


def test_select_by_width_rows_and_missing_widths(env):
    """Rows come from the run of their width; channels of O_act and widths without a kept run
    get the +infinity levels and zero codes that cmpq_kmeans_quantize writes for them; an odd
    d_out takes the byte-wise copy."""
    B = env["B"]
    rng = np.random.default_rng(0)
    d_in, d_out = 37, 333
    runs_c = [torch.from_numpy(rng.normal(size=(d_in, 16)).astype(np.float32)).to(DEV) for _ in range(2)]
    runs_k = [torch.from_numpy(rng.integers(0, 16, size=(d_in, d_out), dtype=np.uint8)).to(DEV) for _ in range(2)]
    bits = rng.choice(np.array([2, 3, 4, 16], np.uint8), size=d_in)
    cent = torch.zeros((d_in, 16), device=DEV)
    codes = torch.full((d_in, d_out), 9, dtype=torch.uint8, device=DEV)
    B.select_by_width(torch.from_numpy(bits).to(DEV), (2, 4), runs_c, runs_k, cent, codes)
    torch.cuda.synchronize()
    for i in range(d_in):
        if bits[i] in (2, 4):
            j = 0 if bits[i] == 2 else 1
            assert np.array_equal(_np(cent[i]), _np(runs_c[j][i])) and np.array_equal(_np(codes[i]), _np(runs_k[j][i]))
        else:
            assert np.all(np.isposinf(_np(cent[i]))) and not _np(codes[i]).any()
    with pytest.raises(B.CmpqError):
        B.select_by_width(torch.from_numpy(bits).to(DEV), (2, 2), runs_c, runs_k, cent, codes)
    with pytest.raises(B.CmpqError):
        B.select_by_width(torch.from_numpy(bits).to(DEV), (2, 5), runs_c, runs_k, cent, codes)


def test_retarget_full_size_layer(env):
    """down_proj of the 70B-shaped block: three budgets from one set of kept runs equal the
    direct route bit for bit."""
    P, synth = env["P"], env["synth"]
    wl = synth.workload("block70b")
    layer = [l for l in wl.layers if l.name == "down_proj"][0]
    W = synth.make_weight(layer.d_out, layer.d_in, "f16", 11, DEV)
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    sumsq = (torch.rand(layer.d_in, generator=g) ** 4 + 0.01).to(DEV)
    cache = P.build_width_cache(W, wl.bit_set, 3, env["ws"])
    for avg in (2.4, 3.5):
        a = P.quantize_layer_from_cache(cache, sumsq, avg, wl.rho_act_ppm, wl.rho_q_ppm, env["ws"])
        b = P.quantize_layer(W, sumsq, wl.bit_set, avg, wl.rho_act_ppm, wl.rho_q_ppm, 3, env["ws"])
        torch.cuda.synchronize()
        assert torch.equal(a.bits, b.bits) and torch.equal(a.out_idx, b.out_idx)
        assert torch.equal(a.codes, b.codes) and torch.equal(a.centroids, b.centroids)
        for x, y in zip(a.packed, b.packed):
            assert (x is None) == (y is None) and (x is None or torch.equal(x, y))
        del a, b
