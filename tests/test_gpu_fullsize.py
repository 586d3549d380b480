"""Parity at the full sizes of the named configurations, in the launch configuration
bench.py times.  Where the oracle can afford the whole layer (the 4096x4096 layer) every
output is compared; for the 70B-shaped layers the oracle recomputes sampled channels one by
one and the global selections are checked through properties that hold at any size."""
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


def _sampled_stats_check(env, X, sumsq, n_cols=48, seed=0):
    cols = np.sort(np.random.default_rng(seed).choice(X.shape[1], n_cols, replace=False))
    sub = _np(X[:, torch.from_numpy(cols).to(DEV)].contiguous())
    _, osum = env["orc"].act_stats(sub)
    assert np.array_equal(_np(sumsq)[cols], osum)


def test_q7b_layer_full_size(env):
    """4096x4096 fp16 layer, 262144 tokens, bits {2,3,4} avg 3.0, 0.5 % weight outliers, 20 rounds."""
    P, synth, ws, orc = env["P"], env["synth"], env["ws"], env["orc"]
    wl = synth.workload("q7b")
    wts, xs = synth.materialize(wl, DEV)
    W, X = wts["q_proj"], xs["x"]
    assert X.shape == (262144, 4096)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    _, sumsq = P.activation_stats(X, ws, status=status)
    _sampled_stats_check(env, X, sumsq)
    del X, xs
    r = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters, ws,
                         with_error=True, keep_prelim=True, status=status)
    o = orc.quantize_layer(_np(W).T.copy(), None, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm,
                           wl.iters, sumsq=_np(sumsq))
    assert status.item() == 0
    assert r.counts == list(o["counts"]) and np.array_equal(_np(r.bits), o["bits"])
    assert np.array_equal(_np(r.act_idx), o["act_idx"])
    assert np.array_equal(_np(r.centroids_prelim), o["cent1"])
    assert np.array_equal(_np(r.codes_prelim), o["codes1"])
    assert len(o["out_idx"]) == 83886
    assert np.array_equal(_np(r.out_idx).astype(np.int64), o["out_idx"])
    assert np.array_equal(_np(r.out_val).view(np.uint16), o["out_val"])
    assert np.array_equal(_np(r.centroids), o["centroids"])      # bar 1e-5 relative; identical in fact
    assert np.array_equal(_np(r.codes), o["codes"])
    for j, b in enumerate(wl.bit_set):
        opk, och, olut = o["packs"][b]
        assert np.array_equal(_np(r.packed[j]).view(np.uint32), opk)
        assert np.array_equal(_np(r.chan_idx[j]), och)
        assert np.array_equal(_np(r.lut[j]).view(np.uint16), olut)
    tot = _np(r.err_total)
    assert abs(tot[0] - o["totals"][0]) <= 1e-4 * o["totals"][0]
    # the call as the pipeline makes it by default: the preliminary run leaves levels and its
    # per-channel tables but no codes, and O_q ranks the distance to the nearest level
    r2 = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters, ws,
                          with_error=True, status=status)
    assert status.item() == 0 and r2.codes_prelim is None
    _same_outputs(r, r2)


def _same_outputs(a, b):
    """Two runs of a layer left the same results, bit for bit (what is checked on one holds for the other)."""
    assert a.counts == b.counts
    for name in ("act_idx", "bits", "out_idx", "out_val", "centroids", "codes", "err_ch", "err_total"):
        x, y = getattr(a, name), getattr(b, name)
        assert (x is None) == (y is None), name
        if x is not None:
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name
    for name in ("packed", "chan_idx", "lut"):
        for x, y in zip(getattr(a, name), getattr(b, name)):
            assert (x is None) == (y is None), name
            if x is not None:
                assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name


def _selection_properties(Wt, cent1, codes1, bits, out_idx, out_val, k):
    """What makes the top-k set unique: size, order, membership, threshold, tie rule."""
    d_in, d_out = Wt.shape
    live = (bits >= 1) & (bits <= 4)
    key = (Wt.float() - torch.gather(cent1, 1, codes1.long())).abs()
    key[~live] = -1.0                                            # O_act channels are no candidates
    key = key.reshape(-1)
    idx = out_idx.long()
    assert idx.numel() == k
    assert bool((idx[1:] > idx[:-1]).all())                      # ascending, no repeats
    assert bool((key[idx] >= 0).all())
    assert torch.equal(out_val, Wt.reshape(-1)[idx].half())
    T = key[idx].min()
    sel = torch.zeros_like(key, dtype=torch.bool)
    sel[idx] = True
    assert bool((key[~sel] <= T).all())                          # nothing larger was left behind
    tie_in = torch.nonzero(sel & (key == T)).flatten()
    tie_out = torch.nonzero(~sel & (key == T)).flatten()
    if tie_in.numel() and tie_out.numel():
        assert int(tie_in.max()) < int(tie_out.min())            # equal scores: smaller index first


@pytest.mark.parametrize("workload,layer", [
    ("block70b", "gate_proj"), ("block70b", "down_proj"), ("block70b", "k_proj"), ("block70b", "q_proj"),
    ("block7b", "gate_proj"), ("block7b", "down_proj"), ("block13b", "gate_proj"), ("block13b", "down_proj"),
    ("block13b", "q_proj")])
def test_block_layers_full_size(env, workload, layer):
    """Layers of the three decoder-block configurations at full size, with each configuration's
    own widths, outlier fractions and round count: 70B-shaped 8192->28672, 28672->8192,
    8192->1024, 8192->8192 (bits {2,3,4} avg 3.5, 1 % weight outliers); 7B-shaped 4096->11008,
    11008->4096 ({2,3} avg 2.2, the paper's 0.45 % / 0.05 %); 13B-shaped 5120->13824,
    13824->5120, 5120->5120 ({2,3,4} avg 2.5, 0.5 %).  Channel lengths 1024 ... 28672 reach every
    launch variant of the K-means kernel."""
    P, synth, ws, orc, B = env["P"], env["synth"], env["ws"], env["orc"], env["B"]
    wl = synth.workload(workload)
    spec = next(l for l in wl.layers if l.name == layer)
    j = wl.layers.index(spec)
    W = synth.make_weight(spec.d_out, spec.d_in, wl.dtype, seed=wl.seed * 1000 + j, device=DEV)
    n_tok = wl.x_shapes[spec.x_key][0]
    X = synth.make_activations(n_tok, spec.d_in, wl.dtype, seed=77, device=DEV, hot_frac=wl.hot_frac,
                               hot_scale=wl.hot_scale, gated=wl.x_gated[spec.x_key])
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    _, sumsq = P.activation_stats(X, ws, status=status)
    _sampled_stats_check(env, X, sumsq, n_cols=24)
    del X
    r = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters, ws,
                         with_error=True, keep_prelim=True, status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    d_in, d_out = spec.d_in, spec.d_out
    assert torch.equal(r.W_t, W.t().contiguous())
    # rankings over d_in keys: the oracle does them whole
    s = _np(sumsq)
    oact, omask = orc.top_channels(s, B.count_ppm(wl.rho_act_ppm, d_in))
    obits, ocounts = orc.allocate_bits(s, omask, wl.bit_set, wl.avg_bits)
    assert np.array_equal(_np(r.act_idx), oact) and np.array_equal(_np(r.bits), obits)
    assert r.counts == list(ocounts)
    # global selection of O_q: properties
    k_q = B.count_ppm(wl.rho_q_ppm, d_in * d_out)
    _selection_properties(r.W_t, r.centroids_prelim, r.codes_prelim, r.bits, r.out_idx, r.out_val, k_q)
    # k-means of both passes, coding, packing, error: sampled channels, recomputed one by one
    rng = np.random.default_rng(5)
    sample = np.sort(np.concatenate([rng.choice(d_in, 40, replace=False), oact[:2]]))
    sample = np.unique(sample)
    st = torch.from_numpy(sample).to(DEV)
    Ws = _np(r.W_t[st])
    bs = obits[sample]
    c1, k1 = orc.kmeans(Ws, bs, iters=wl.iters)
    assert np.array_equal(_np(r.centroids_prelim[st]), c1) and np.array_equal(_np(r.codes_prelim[st]), k1)
    oi = _np(r.out_idx).astype(np.int64)
    local = []
    for t, i in enumerate(sample):
        seg = oi[(oi >= i * d_out) & (oi < (i + 1) * d_out)] - i * d_out
        local.append(seg + t * d_out)
    local = np.concatenate(local)
    c2, k2 = orc.kmeans(Ws, bs, out_idx=local, iters=wl.iters)
    assert np.array_equal(_np(r.centroids[st]), c2) and np.array_equal(_np(r.codes[st]), k2)
    for jw, b in enumerate(wl.bit_set):
        opk, och, olut = orc.pack(k2, bs, c2, b)
        if r.counts[jw] == 0:
            assert len(och) == 0 and not (obits == b).any()
            continue
        chan = _np(r.chan_idx[jw])
        assert np.array_equal(chan, np.flatnonzero(obits == b))
        rows = np.searchsorted(chan, sample[och])
        assert np.array_equal(_np(r.packed[jw][torch.from_numpy(rows).to(DEV)]).view(np.uint32), opk)
        assert np.array_equal(_np(r.lut[jw][torch.from_numpy(rows).to(DEV)]).view(np.uint16), olut)
    oerr, _ = orc.dequant_error(Ws, c2, k2, bs, local, None)
    got = _np(r.err_ch[st])
    assert np.allclose(got, oerr, rtol=1e-12, atol=0)
    tot = _np(r.err_total)
    ref_w = float((r.err_ch * sumsq.double()).sum())
    assert abs(tot[0] - ref_w) <= 1e-9 * ref_w
    # the call as the pipeline makes it by default (no preliminary codes: O_q from the distance to
    # the nearest level), and the route that builds the final run's tables again: the same results
    r2 = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters, ws,
                          with_error=True, status=status)
    assert status.item() == 0 and r2.codes_prelim is None
    _same_outputs(r, r2)
    del r2
    r3 = P.quantize_layer(W, sumsq, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters, ws,
                          with_error=True, status=status, share_tables=False, prelim_codes=True)
    assert status.item() == 0
    _same_outputs(r, r3)


@pytest.mark.parametrize("join", [False, True])
def test_block70b_three_streams_equals_one_stream_full_size(env, join):
    """The whole 70B-shaped block exactly as bench.py runs it by default (layers shared out over
    three streams; steps enqueued one after the other with one join at the end, or joined one by
    one): every output of the last step bit-identical to the one-stream run of the same call
    chain, whose layers the tests above check against the oracle."""
    P, B, synth = env["P"], env["B"], env["synth"]
    wl = synth.workload("block70b")
    wts, xs = synth.materialize(wl, DEV)
    layers = [(l.name, l.x_key) for l in wl.layers]
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    args = (wts, xs, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters)
    one = P.quantize_block(*args, env["ws"], with_error=True, status=status)
    wss = [B.Workspace(DEV) for _ in range(3)]
    many = None
    for _ in range(2):
        many = P.quantize_block(*args, wss, with_error=True, status=status, streams=3, join=join)
    if not join:
        P.join_streams(DEV, 3)
    torch.cuda.synchronize()
    assert status.item() == 0
    for name in one:
        a, b = one[name], many[name]
        assert a.counts == b.counts
        for f in ("sumsq", "act_idx", "bits", "centroids", "codes", "out_idx", "out_val", "err_ch", "err_total"):
            assert torch.equal(getattr(a, f), getattr(b, f)), (name, f)
        for x, y in zip(a.packed + a.chan_idx + a.lut, b.packed + b.chan_idx + b.lut):
            assert (x is None) == (y is None) and (x is None or torch.equal(x, y)), name
