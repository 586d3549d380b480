"""Host-side logic that needs no GPU: the benchmark's one-GPU contract, the seeded input
recipe, and the sharing of layers over streams."""
import os
import subprocess
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip()


def test_workloads_have_the_named_shapes():
    from paper_2410_13056_amd import synth
    wl = synth.workload("block70b")
    shapes = {l.name: (l.d_in, l.d_out) for l in wl.layers}
    assert shapes == {"q_proj": (8192, 8192), "k_proj": (8192, 1024), "v_proj": (8192, 1024),
                      "o_proj": (8192, 8192), "gate_proj": (8192, 28672), "up_proj": (8192, 28672),
                      "down_proj": (28672, 8192)}
    assert wl.params == sum(a * b for a, b in shapes.values()) == 855638016
    assert min(wl.bit_set) <= wl.avg_bits <= max(wl.bit_set)
    tiny = synth.workload("tiny")
    assert tiny.params < 1 << 20


def test_inputs_are_seeded_and_heavy_tailed():
    from paper_2410_13056_amd import synth
    a = synth.make_weight(256, 512, "f32", 3, "cpu")
    b = synth.make_weight(256, 512, "f32", 3, "cpu")
    c = synth.make_weight(256, 512, "f32", 4, "cpu")
    assert torch.equal(a, b) and not torch.equal(a, c) and tuple(a.shape) == (256, 512)
    x = a.numpy().ravel().astype(np.float64)
    kurt = np.mean((x - x.mean()) ** 4) / np.var(x) ** 2
    assert kurt > 3.5                                     # heavier tails than a Gaussian
    X = synth.make_activations(512, 256, "f32", 1, "cpu").numpy().astype(np.float64)
    energy = np.sort((X ** 2).sum(axis=0))[::-1]
    assert energy[:3].sum() > 0.2 * energy.sum()          # a few channels carry much of the energy
    assert torch.equal(synth.make_activations(64, 32, "f16", 9, "cpu"), synth.make_activations(64, 32, "f16", 9, "cpu"))


def test_layers_are_shared_out_largest_first():
    from paper_2410_13056_amd.pipeline import assign_layers
    sizes = {"q": 64, "k": 8, "v": 8, "o": 64, "gate": 224, "up": 224, "down": 224}
    plan = assign_layers(sizes, 3)
    assert [n for n, _ in plan] == ["gate", "up", "down", "q", "o", "k", "v"]
    assert sorted(n for n, _ in plan) == sorted(sizes)
    load = [0, 0, 0]
    for n, j in plan:
        load[j] += sizes[n]
    assert max(load) - min(load) <= max(sizes.values())
    assert [j for _, j in plan[:3]] == [0, 1, 2]
    assert assign_layers(sizes, 1) == [(n, 0) for n, _ in plan]
    assert assign_layers({}, 2) == []


def _arrangement_bounds(d_out, keys, kept, shape):
    """Every index the histogram K-means kernel forms for one channel, recomputed on the host from
    the launch shape the library reports: bucket counts, padded stretches of the place array, the
    16-bit prefix tables, the removed-entry bitmap, the scatter cursors / coding table, and the
    per-lane ownership of weight groups.  Raises AssertionError on any index out of its array."""
    T, G, LB, arr_bytes, dyn, static = shape
    buckets = 1 << (16 - LB)
    n_groups = d_out // 4
    assert G * T >= n_groups                                    # every group of 4 weights has a lane
    assert T in (64, 128, 256, 512) and (T // 16) * 16 == T     # T/16 lanes share a boundary: 15 boundaries fit
    assert max(1, buckets // T) * T >= buckets                  # the prefix pass covers every bucket
    # dynamic LDS = place array | removed bitmap (whole 16-byte pieces) | one word per bucket
    n_words = (d_out + 31) >> 5
    assert dyn == arr_bytes + ((n_words + 3) & ~3) * 4 + buckets * 4
    assert arr_bytes % 16 == 0
    assert ((n_groups - 1) >> 3) < n_words                       # bitmap word of the last group
    b = keys[kept] >> LB
    assert b.max(initial=0) < buckets
    n = np.bincount(b, minlength=buckets).astype(np.int64)
    padded = (n + 3) & ~3
    start = np.concatenate([[0], np.cumsum(padded)])
    ncum = np.concatenate([[0], np.cumsum(n)])
    assert start[-1] <= arr_bytes                               # scatter and scans stay inside the array
    assert start[-1] < 65536 and ncum[-1] < 65536               # the tables are 16 bits wide
    per = max(1, buckets // T)
    packed = (n | (padded << 16)).reshape(-1, per).sum(1)       # a lane's share of the (count, stretch) scan
    assert int(packed.sum()) < 1 << 32 and int((n.reshape(-1, per).sum(1)).max()) < 65536
    # scans read whole words of a stretch: [start >> 2, end >> 2), 4 * L at a time, guarded by the end
    assert np.all(start % 4 == 0) and start[-1] // 4 <= arr_bytes // 4
    # three workgroups of the longest configured channels (28 672 weights) share a compute unit's 160 KiB
    total = static + 512 + dyn                                  # + what the compiler adds to the static part
    if d_out <= 28672:
        assert 3 * total <= 160 * 1024
    return int(start[-1]), total


def test_kmeans_kernel_indices_stay_in_bounds_on_adversarial_channels():
    """The two builds of the K-means kernel that faulted on the GPU differed from the shipped one
    only in register allocation; a cause in the shared index arithmetic would show here.  Every
    launch shape, its extreme channel lengths, and key layouts that push each table to its
    limit: all keys in one bucket, every bucket occupied, counts of 1 mod 4 everywhere (most
    padding), everything removed, the largest channel."""
    from paper_2410_13056_amd import binding as B
    B.lib()
    rng = np.random.default_rng(0)
    lengths = sorted({4, 8, 252, 256, 260, 512, 1024, 2044, 2048, 2052, 4096, 4100, 5120, 8192, 8196, 11008,
                      13824, 16384, 16388, 28672, 32764, 32768})
    worst = 0
    for d_out in lengths:
        shape = B.kmeans_launch_shape(d_out)
        LB = shape[2]
        buckets = 1 << (16 - LB)
        layouts = {
            "one bucket": np.full(d_out, 0x8000 + 5, np.uint16),
            "every bucket": (np.arange(d_out) % buckets).astype(np.uint16) << LB,
            "most padding": np.repeat(np.arange(buckets, dtype=np.uint16) << LB, 5)[:d_out]
            if d_out >= 5 else np.zeros(d_out, np.uint16),
            "random": rng.integers(0, 65536, d_out).astype(np.uint16),
            "gaussian": (0x8000 + np.clip(rng.normal(0, 900, d_out), -30000, 30000)).astype(np.uint16),
        }
        for name, keys in layouts.items():
            keys = np.resize(keys, d_out).astype(np.int64)
            for kept in (np.ones(d_out, bool), np.zeros(d_out, bool), rng.random(d_out) < 0.99):
                used, total = _arrangement_bounds(d_out, keys, kept, shape)
                worst = max(worst, total)
    assert worst <= 64 * 1024                                   # the largest workgroup's LDS
    with np.testing.assert_raises(Exception):
        B.kmeans_launch_shape(32772)
    with np.testing.assert_raises(Exception):
        B.kmeans_launch_shape(6)
