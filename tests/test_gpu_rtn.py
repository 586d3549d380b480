"""GPU-vs-oracle parity of CMPQ with the uniform quantizer (App. A.2 / Tab. 10), through the
C ABI: cmpq_rtn_quantize.

Bars: codes are integers decided by single IEEE fp32 operations on both sides - bit-exact;
scale and zero are one fp32 division and a minimum - bit-exact; the channel errors are fp64
sums of the same terms in another order: relative 1e-11.
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


def _run(env, Wd, bits, group, with_err=True, status=None):
    B = env["B"]
    d_in, d_out = Wd.shape
    ng = -(-d_out // group)
    codes = torch.full((d_in, d_out), 0xee, dtype=torch.uint8, device=DEV)
    scale = torch.full((d_in, ng), -7.0, dtype=torch.float32, device=DEV)
    zero = torch.full((d_in, ng), -7.0, dtype=torch.float32, device=DEV)
    err = torch.full((d_in,), -1.0, dtype=torch.float64, device=DEV) if with_err else None
    B.rtn_quantize(Wd, torch.from_numpy(bits).to(DEV), group, codes, scale, zero, err, status)
    torch.cuda.synchronize()
    return _np(codes), _np(scale), _np(zero), (None if err is None else _np(err))


def _compare(got, want):
    codes, scale, zero, err = got
    ocodes, oscale, ozero, oerr = want
    assert np.array_equal(codes, ocodes)
    assert np.array_equal(scale, oscale) and np.array_equal(zero, ozero)
    if err is not None:
        fin = np.isfinite(oerr)       # a channel kept in FP16 whose weights exceed the FP16 range: infinite on both sides
        assert np.array_equal(np.isfinite(err), fin) and np.array_equal(err[~fin], oerr[~fin])
        assert np.all(np.abs(err[fin] - oerr[fin]) <= 1e-11 * np.maximum(oerr[fin], 1e-300))


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("d_in,d_out,group", [(40, 2048, 128), (33, 4100, 128), (17, 1000, 32),
                                               (9, 6152, 512), (64, 264, 8), (5, 7, 8), (12, 20480, 256), (3, 100, 512)])
def test_rtn_parity(env, dtype, d_in, d_out, group):
    rng = np.random.default_rng(d_in * 131 + d_out)
    W = (rng.standard_t(4, size=(d_in, d_out)) * 0.02).astype(np.float16 if dtype == "f16" else np.float32)
    W[0, : min(d_out, group)] = W[0, 0]                         # a constant first group
    if d_in > 3:
        W[3] = 0.0
        W[3, ::3] = -0.0                                        # zeros of both signs
    bits = rng.choice(np.array([1, 2, 3, 4, 16], np.uint8), size=d_in)
    got = _run(env, torch.from_numpy(W).to(DEV), bits, group)
    _compare(got, env["orc"].rtn_quantize(W, bits, group))


def test_rtn_strided_and_unaligned_rows(env):
    """Rows with a leading dimension that is no multiple of 8 and a base that is not 16-byte
    aligned take the element-wise loads and stores; the result is the same."""
    rng = np.random.default_rng(2)
    big = torch.from_numpy((rng.normal(0, 0.03, size=(50, 3001))).astype(np.float16)).to(DEV)
    view = big[:, 1:2990]                                       # ld 3001, base off by one half
    bits = rng.choice(np.array([2, 3, 4, 16], np.uint8), size=50)
    got = _run(env, view, bits, 128)
    _compare(got, env["orc"].rtn_quantize(_np(view).copy(), bits, 128))


def test_rtn_without_error_and_status_flag(env):
    rng = np.random.default_rng(4)
    W = rng.normal(0, 0.03, size=(20, 1024)).astype(np.float32)
    bits = np.full(20, 3, np.uint8)
    codes, scale, zero, err = _run(env, torch.from_numpy(W).to(DEV), bits, 128, with_err=False)
    o = env["orc"].rtn_quantize(W, bits, 128)
    assert err is None and np.array_equal(codes, o[0]) and np.array_equal(scale, o[1])
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    _run(env, torch.from_numpy(W).to(DEV), bits, 128, status=status)
    assert status.item() == 0
    W[7, 300] = np.inf
    _run(env, torch.from_numpy(W).to(DEV), bits, 128, status=status)
    assert status.item() & env["B"].STATUS_NONFINITE


def test_rtn_rejects_bad_group_and_shapes(env):
    B = env["B"]
    W = torch.zeros((4, 64), dtype=torch.float16, device=DEV)
    bits = torch.full((4,), 3, dtype=torch.uint8, device=DEV)
    for group in (0, 4, 96, 1024):
        ng = max(1, -(-64 // max(group, 1)))
        with pytest.raises((B.CmpqError, ValueError)):
            B.rtn_quantize(W, bits, group, torch.zeros((4, 64), dtype=torch.uint8, device=DEV),
                           torch.zeros((4, ng), device=DEV), torch.zeros((4, ng), device=DEV))
    # empty inputs are fine
    B.rtn_quantize(W[:0], bits[:0], 128, torch.zeros((0, 64), dtype=torch.uint8, device=DEV),
                   torch.zeros((0, 1), device=DEV), torch.zeros((0, 1), device=DEV))


def test_rtn_layer_end_to_end(env):
    """Statistics -> O_act at 0.5 % -> Algorithm 1 -> uniform quantizer, against the same
    chain of oracle calls."""
    P, orc, synth = env["P"], env["orc"], env["synth"]
    rng = np.random.default_rng(8)
    d_in, d_out, n = 600, 1536, 300
    W = (rng.standard_t(4, size=(d_out, d_in)) * 0.02).astype(np.float16)
    X = (rng.normal(0, 1, size=(n, d_in)) * rng.lognormal(0, 1, size=d_in)).astype(np.float16)
    Xd = torch.from_numpy(X).to(DEV)
    _, sumsq = P.activation_stats(Xd, env["ws"])
    r = P.quantize_layer_rtn(torch.from_numpy(W).to(DEV), sumsq, (2, 3, 4), 2.7, 5000, 128, env["ws"],
                             with_error=True)
    torch.cuda.synchronize()
    _, osum = orc.act_stats(X)
    k_act = orc.count_ppm(5000, d_in)
    act_idx, mask = orc.top_channels(osum, k_act)
    obits, ocounts = orc.allocate_bits(osum, mask, (2, 3, 4), 2.7)
    assert np.array_equal(_np(r.act_idx), act_idx) and np.array_equal(_np(r.bits), obits)
    assert r.counts == list(ocounts)
    _compare((_np(r.codes), _np(r.scale), _np(r.zero), _np(r.err_ch)),
             orc.rtn_quantize(np.ascontiguousarray(W.T), obits, 128))


def test_rtn_full_size_layer_on_sampled_channels(env):
    """gate_proj of the 70B-shaped block (8192 x 28672, FP16) in the launch the benchmark
    times; channels are independent, so the oracle checks a sample of them exactly."""
    synth = env["synth"]
    wl = synth.workload("block70b")
    layer = [l for l in wl.layers if l.name == "gate_proj"][0]
    W = synth.make_weight(layer.d_out, layer.d_in, "f16", 11, DEV)     # [d_out, d_in]
    Wt = W.t().contiguous()
    rng = np.random.default_rng(1)
    bits = rng.choice(np.array([2, 3, 4, 16], np.uint8), size=layer.d_in, p=[0.3, 0.4, 0.295, 0.005])
    codes, scale, zero, err = _run(env, Wt, bits, 128)
    pick = np.sort(rng.choice(layer.d_in, size=96, replace=False))
    o = env["orc"].rtn_quantize(_np(Wt[torch.from_numpy(pick).to(DEV)]), bits[pick], 128)
    _compare((codes[pick], scale[pick], zero[pick], err[pick]), o)
    # every channel: codes within range, steps non-negative
    top = np.where(bits <= 4, (1 << np.minimum(bits, 4).astype(np.int64)) - 1, 0)
    assert np.all(codes.max(axis=1) <= top) and np.all(scale >= 0)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_rtn_exact_ties_and_extreme_ranges(env, dtype):
    """Quotients that are exact half-integers (ramps of whole numbers with Delta = 2, scaled by
    powers of two) must round to the even code on both sides; steps far outside the usual
    range of weights (tiny and huge Delta, fp32 only) take the kernel's ordinary division."""
    rng = np.random.default_rng(6)
    rows, bits = [], []
    exps = (-10, -3, 0, 4) if dtype == "f16" else (-100, -70, -59, -30, 0, 40, 61, 90)
    for N in (1, 2, 3, 4):
        top = 2 ** N - 1
        ramp = np.arange(2 * top + 1, dtype=np.float64)          # 0 .. 2 top: Delta = 2
        for e in exps:
            row = np.zeros(256)
            row[:128] = rng.permutation(np.resize(ramp, 128)) * 2.0 ** e
            row[128:] = (rng.permutation(np.resize(ramp, 128)) - top) * 2.0 ** e   # centred on 0
            rows.append(row)
            bits.append(N)
    # wide dynamic range inside a group
    for N in (2, 3, 4):
        mag = np.exp(rng.uniform(-8 if dtype == "f16" else -40, 8 if dtype == "f16" else 40, size=256))
        rows.append(mag * rng.choice([-1.0, 1.0], size=256))
        bits.append(N)
    W = np.array(rows).astype(np.float16 if dtype == "f16" else np.float32)
    bits = np.array(bits, np.uint8)
    got = _run(env, torch.from_numpy(W).to(DEV), bits, 128)
    want = env["orc"].rtn_quantize(W, bits, 128)
    _compare(got, want)
    assert (want[0][:4 * len(exps)] % 2 == 0).mean() > 0.6          # the ties went to even codes


def test_rtn_many_random_groups(env):
    """Two million weights in random groups of every width and both input types: any quotient the
    kernel's division rounded differently from the IEEE one would show as a code mismatch."""
    rng = np.random.default_rng(12)
    for dtype in (np.float16, np.float32):
        W = (rng.standard_t(3, size=(1024, 1024)) * rng.lognormal(-4, 2, size=(1024, 1))).astype(dtype)
        bits = rng.choice(np.array([1, 2, 3, 4], np.uint8), size=1024)
        got = _run(env, torch.from_numpy(W).to(DEV), bits, 64)
        _compare(got, env["orc"].rtn_quantize(W, bits, 64))


@pytest.mark.parametrize("seed", range(int(os.environ.get("CMPQ_RANDOM_CASES", "12"))))
def test_rtn_randomized(env, seed):
    """Random shapes, group sizes, widths, input types, row strides and value patterns (ties on a
    grid, constant stretches, spikes, tiny and huge scales)."""
    rng = np.random.default_rng(9000 + seed)
    d_in = int(rng.integers(1, 70))
    d_out = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 9000)]))
    group = int(2 ** rng.integers(3, 10))
    dtype = np.float16 if rng.random() < 0.6 else np.float32
    W = rng.normal(0, 0.02, (d_in, d_out))
    style = int(rng.integers(0, 4))
    if style == 1:
        W = np.round(W * 64) / 64
    elif style == 2:
        W[:, : d_out // 2] = 0.25
        W[rng.random(W.shape) < 0.05] = -0.0
    elif style == 3:
        W[rng.random(W.shape) < 0.01] *= 50
    if dtype == np.float32 and rng.random() < 0.3:
        W = W * float(2.0 ** rng.integers(-90, 90))
    W = W.astype(dtype)
    bits = rng.choice(np.array([1, 2, 3, 4, 16], np.uint8), size=d_in)
    pad = int(rng.choice([0, 0, 3, 8]))
    big = torch.zeros((d_in, d_out + pad), dtype=torch.from_numpy(W).dtype, device=DEV)
    big[:, :d_out] = torch.from_numpy(W).to(DEV)
    got = _run(env, big[:, :d_out], bits, group)
    _compare(got, env["orc"].rtn_quantize(W, bits, group))
