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
