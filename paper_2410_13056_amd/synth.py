"""Seeded synthetic inputs for the CMPQ quantization path.

This module only draws random tensors.  It holds none of the method's
arithmetic and is the one piece of code that the CPU oracle's tests and the
HIP path's tests both use, so that the two sides see identical inputs.

The paper calibrates on C4 segments and quantizes OPT / LLaMA weights (Sec. 4.1);
neither is available, so the tensors below stand in for them.  They keep the
structure the method reacts to:

* weights: a narrow Gaussian bulk with a small fraction of heavy-tailed
  entries (Sec. 3.2.2 describes a few weights much larger than the rest);
* activations: outliers that persist along a channel over all tokens
  (Sec. 3.2.2, Fig. 2), plus a log-normal spread of per-channel scales;
* the down-projection input of a gated MLP: silu(g) * u, heavy tailed.

Everything is drawn from a ``torch.Generator`` seeded by the caller, on the
device the caller names, in fp32, and rounded once to the requested dtype.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import torch

_DTYPES = {"f16": torch.float16, "f32": torch.float32}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_weight(d_out: int, d_in: int, dtype: str = "f16", seed: int = 0,
                device="cpu", sigma: float = 0.02, tail_frac: float = 0.005,
                tail_scale: float = 0.1, row_chunk: int = 4096) -> torch.Tensor:
    """Weight of a linear layer in the framework layout ``[d_out, d_in]``.

    Entries are N(0, sigma^2); each entry is independently replaced, with
    probability ``tail_frac``, by ``tail_scale`` times a Student-t draw with
    three degrees of freedom (a normal over the root of a chi-square / 3).
    """
    g = _gen(seed, device)
    out = torch.empty((d_out, d_in), dtype=_DTYPES[dtype], device=device)
    for r0 in range(0, d_out, row_chunk):
        r1 = min(d_out, r0 + row_chunk)
        shape = (r1 - r0, d_in)
        w = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * sigma
        pick = torch.rand(shape, generator=g, device=device) < tail_frac
        z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        chi = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(3):
            chi += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
        t3 = z / torch.sqrt(chi / 3.0)
        w = torch.where(pick, tail_scale * t3, w)
        out[r0:r1] = w.to(_DTYPES[dtype])
    return out


def make_activations(n: int, d_in: int, dtype: str = "f16", seed: int = 0,
                     device="cpu", hot_frac: float = 0.01, hot_scale: float = 30.0,
                     lognormal_sigma: float = 0.5, gated: bool = False,
                     row_chunk: int = 8192) -> torch.Tensor:
    """Calibration activations ``[n, d_in]`` (tokens by input channels).

    Every channel has its own scale ``exp(N(0, lognormal_sigma^2))``;
    ``round(hot_frac * d_in)`` channels picked at random carry an extra factor
    ``hot_scale`` on every token.  With ``gated`` the base draw is
    ``silu(g) * u`` for two independent standard normals, the shape of a
    down-projection input; otherwise it is a standard normal.
    """
    g = _gen(seed, device)
    scale = torch.exp(torch.randn((d_in,), generator=g, device=device) * lognormal_sigma) \
        if lognormal_sigma > 0 else torch.ones((d_in,), device=device)
    n_hot = int(round(hot_frac * d_in))
    if n_hot > 0:
        hot = torch.randperm(d_in, generator=g, device=device)[:n_hot]
        scale[hot] *= hot_scale
    out = torch.empty((n, d_in), dtype=_DTYPES[dtype], device=device)
    for r0 in range(0, n, row_chunk):
        r1 = min(n, r0 + row_chunk)
        shape = (r1 - r0, d_in)
        x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        if gated:
            u = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
            x = torch.nn.functional.silu(x) * u
        out[r0:r1] = (x * scale).to(_DTYPES[dtype])
    return out


@dataclasses.dataclass
class LayerSpec:
    """One linear layer of a workload: its shape and which activation feeds it."""
    name: str
    d_out: int
    d_in: int
    x_key: str


@dataclasses.dataclass
class Workload:
    """A named quantization job: layers, activations, budget and knobs."""
    name: str
    layers: List[LayerSpec]
    x_shapes: Dict[str, Tuple[int, int]]      # x_key -> (n tokens, d_in)
    x_gated: Dict[str, bool]
    dtype: str
    bit_set: Tuple[int, ...]
    avg_bits: float
    rho_act_ppm: int                          # activation-outlier channels, parts per million
    rho_q_ppm: int                            # residual-outlier weights, parts per million
    iters: int
    hot_frac: float
    hot_scale: float
    lognormal_sigma: float
    seed: int

    @property
    def params(self) -> int:
        return sum(l.d_out * l.d_in for l in self.layers)


def _block(name, hidden, ffn, kv, n_tok, dtype, bit_set, avg_bits, rho_q_ppm, iters,
           hot_frac, hot_scale, seed) -> Workload:
    layers = [
        LayerSpec("q_proj", hidden, hidden, "attn_in"),
        LayerSpec("k_proj", kv, hidden, "attn_in"),
        LayerSpec("v_proj", kv, hidden, "attn_in"),
        LayerSpec("o_proj", hidden, hidden, "o_in"),
        LayerSpec("gate_proj", ffn, hidden, "mlp_in"),
        LayerSpec("up_proj", ffn, hidden, "mlp_in"),
        LayerSpec("down_proj", hidden, ffn, "down_in"),
    ]
    xs = {"attn_in": (n_tok, hidden), "o_in": (n_tok, hidden),
          "mlp_in": (n_tok, hidden), "down_in": (n_tok, ffn)}
    gated = {"attn_in": False, "o_in": False, "mlp_in": False, "down_in": True}
    return Workload(name, layers, xs, gated, dtype, bit_set, avg_bits, 4500, rho_q_ppm,
                    iters, hot_frac, hot_scale, 0.5, seed)


def workload(name: str) -> Workload:
    """The five configurations the build is measured and tested on.

    ``tiny``      one 512x256 fp32 layer, 256 tokens, bits {2,3} avg 2.5, 10 rounds.
    ``q7b``       one 4096x4096 fp16 layer, 262144 tokens, bits {2,3,4} avg 3.0.
    ``block7b``   LLaMA-7B-shaped decoder block, 65536 tokens, bits {2,3} avg 2.2.
    ``block13b``  LLaMA-13B-shaped decoder block, 65536 tokens, bits {2,3,4} avg 2.5.
    ``block70b``  LLaMA-70B-shaped GQA decoder block, 32768 tokens, {2,3,4} avg 3.5.
    """
    if name == "tiny":
        return Workload("tiny", [LayerSpec("linear", 512, 256, "x")], {"x": (256, 256)},
                        {"x": False}, "f32", (2, 3), 2.5, 4500, 5000, 10,
                        0.02, 20.0, 0.0, 0)
    if name == "q7b":
        return Workload("q7b", [LayerSpec("q_proj", 4096, 4096, "x")], {"x": (262144, 4096)},
                        {"x": False}, "f16", (2, 3, 4), 3.0, 4500, 5000, 20,
                        0.01, 30.0, 0.5, 1)
    if name == "block7b":
        return _block("block7b", 4096, 11008, 4096, 65536, "f16", (2, 3), 2.2, 500, 20,
                      0.01, 30.0, 2)
    if name == "block13b":
        return _block("block13b", 5120, 13824, 5120, 65536, "f16", (2, 3, 4), 2.5, 5000, 20,
                      0.01, 30.0, 3)
    if name == "block70b":
        return _block("block70b", 8192, 28672, 1024, 32768, "f16", (2, 3, 4), 3.5, 10000, 20,
                      0.005, 50.0, 4)
    raise KeyError(name)


def scaled(wl: Workload, tokens: Optional[int] = None, shrink: int = 1) -> Workload:
    """A copy of ``wl`` with fewer tokens and / or every dimension divided by
    ``shrink`` (kept a multiple of 8) - same structure, test-sized."""
    def s(v):
        return max(8, (v // shrink) // 8 * 8)
    layers = [LayerSpec(l.name, s(l.d_out), s(l.d_in), l.x_key) for l in wl.layers]
    xs = {k: (tokens if tokens is not None else n, s(d)) for k, (n, d) in wl.x_shapes.items()}
    return dataclasses.replace(wl, name=f"{wl.name}/s{shrink}", layers=layers, x_shapes=xs)


def materialize(wl: Workload, device="cpu"):
    """Draw every tensor of a workload.  Returns ``(weights, activations)``:
    ``weights[layer.name]`` is ``[d_out, d_in]``, ``activations[x_key]`` is ``[n, d_in]``."""
    xs = {}
    for j, (key, (n, d)) in enumerate(sorted(wl.x_shapes.items())):
        xs[key] = make_activations(n, d, wl.dtype, seed=wl.seed * 1000 + 100 + j, device=device,
                                   hot_frac=wl.hot_frac, hot_scale=wl.hot_scale,
                                   lognormal_sigma=wl.lognormal_sigma, gated=wl.x_gated[key])
    ws = {}
    for j, l in enumerate(wl.layers):
        ws[l.name] = make_weight(l.d_out, l.d_in, wl.dtype, seed=wl.seed * 1000 + j, device=device)
    return ws, xs
