"""ctypes front end of the CPU oracle (``cmpq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

All arrays are NumPy, host resident, in the paper's orientation
(Sec. 3.2.1): ``W[d_in, d_out]``, row ``i`` = input channel ``i``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cmpq_oracle.c")
_LIB = os.path.join(_HERE, "libcmpq_oracle.so")

KMAX = 16
PROTECTED = 16
SCORE_RESIDUAL = 0
SCORE_MAGNITUDE = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math and no FMA contraction, so
    every operation rounds the way the source reads."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_count_ppm.restype = ctypes.c_int64
        _lib.orc_count_ppm.argtypes = [ctypes.c_int64, ctypes.c_int64]
        _lib.orc_pack.restype = ctypes.c_int64
        _lib.orc_weight_outliers_per_channel.restype = ctypes.c_int64
        _lib.orc_f32_to_f16.restype = ctypes.c_uint16
        _lib.orc_f32_to_f16.argtypes = [ctypes.c_float]
        _lib.orc_f16_to_f64.restype = ctypes.c_double
        _lib.orc_f16_to_f64.argtypes = [ctypes.c_uint16]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError(f"oracle takes float16 or float32, got {a.dtype}")


def _c(a, dtype=None) -> np.ndarray:
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def count_ppm(ppm: int, n: int) -> int:
    return int(lib().orc_count_ppm(int(ppm), int(n)))


def num_threads() -> int:
    return int(lib().orc_num_threads())


def f32_to_f16_bits(x: float) -> int:
    return int(lib().orc_f32_to_f16(ctypes.c_float(x)))


def f16_bits_to_f64(h: int) -> float:
    return float(lib().orc_f16_to_f64(ctypes.c_uint16(h)))


def act_stats(X: np.ndarray, acc: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Returns ``(acc float64[d_in], sumsq float32[d_in])``; pass ``acc`` back in to add tokens."""
    X = _c(X)
    n, d_in = X.shape
    acc = np.zeros(d_in, np.float64) if acc is None else _c(acc, np.float64).copy()
    sumsq = np.zeros(d_in, np.float32)
    rc = lib().orc_act_stats(_p(X), _dtype_code(X), ctypes.c_int64(n), ctypes.c_int64(d_in),
                             ctypes.c_int64(d_in), _p(acc), _p(sumsq))
    assert rc == 0, rc
    return acc, sumsq


def act_stats_norm(X: np.ndarray, norm: int, acc: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Tab. 13: ``(acc float64[d_in], stat float32[d_in])`` for norm 0 (l2, squared), 1 (l1), 2 (l-infinity)."""
    X = _c(X)
    n, d_in = X.shape
    acc = np.zeros(d_in, np.float64) if acc is None else _c(acc, np.float64).copy()
    stat = np.zeros(d_in, np.float32)
    rc = lib().orc_act_stats_norm(_p(X), _dtype_code(X), ctypes.c_int64(n), ctypes.c_int64(d_in),
                                  ctypes.c_int64(d_in), int(norm), _p(acc), _p(stat))
    assert rc == 0, rc
    return acc, stat


def top_channels(sumsq: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    sumsq = _c(sumsq, np.float32)
    d_in = sumsq.shape[0]
    idx = np.zeros(max(k, 1), np.int32)
    mask = np.zeros(d_in, np.uint8)
    rc = lib().orc_top_channels(_p(sumsq), ctypes.c_int64(d_in), ctypes.c_int64(k), _p(idx), _p(mask))
    assert rc == 0, rc
    return idx[:k], mask


def allocate_bits(sumsq: np.ndarray, chan_mask: Optional[np.ndarray], bit_set: Sequence[int],
                  avg_bits: float) -> Tuple[np.ndarray, np.ndarray]:
    sumsq = _c(sumsq, np.float32)
    d_in = sumsq.shape[0]
    bs = np.asarray(bit_set, np.int32)
    bits = np.zeros(d_in, np.uint8)
    counts = np.zeros(len(bs), np.int64)
    cm = None if chan_mask is None else _c(chan_mask, np.uint8)
    rc = lib().orc_allocate_bits(_p(sumsq), ctypes.c_int64(d_in), _p(cm), _p(bs), len(bs),
                                 ctypes.c_double(avg_bits), _p(bits), _p(counts))
    if rc != 0:
        raise ValueError(f"orc_allocate_bits rc={rc}")
    return bits, counts


def kmeans(W: np.ndarray, bits: np.ndarray, out_idx: Optional[np.ndarray] = None,
           elem_weight: Optional[np.ndarray] = None, iters: int = 20, trace: bool = False,
           start: Optional[np.ndarray] = None):
    """Returns ``(centroids float32[d_in,16], codes uint8[d_in,d_out][, sse float64[d_in,iters+1]])``.
    `start` [d_in,16] float32 replaces the quantile start of every channel by the given levels."""
    W = _c(W)
    d_in, d_out = W.shape
    bits = _c(bits, np.uint8)
    oi = None if out_idx is None else _c(out_idx, np.int64)
    ew = None if elem_weight is None else _c(elem_weight, np.float32)
    cent = np.zeros((d_in, KMAX), np.float32)
    codes = np.zeros((d_in, d_out), np.uint8)
    sse = np.zeros((d_in, iters + 1), np.float64) if trace else None
    st = None if start is None else _c(start, np.float32)
    if st is not None and st.shape != (d_in, KMAX):
        raise ValueError("start must be [d_in, 16]")
    rc = lib().orc_kmeans(_p(W), _dtype_code(W), ctypes.c_int64(d_in), ctypes.c_int64(d_out),
                          ctypes.c_int64(d_out), _p(bits), _p(oi),
                          ctypes.c_int64(0 if oi is None else oi.shape[0]), _p(ew),
                          int(iters), _p(st), _p(cent), _p(codes), _p(sse))
    assert rc == 0, rc
    return (cent, codes, sse) if trace else (cent, codes)


def weight_outliers(W: np.ndarray, centroids: Optional[np.ndarray], codes: Optional[np.ndarray],
                    bits: np.ndarray, k: int, score: int = SCORE_RESIDUAL):
    """Returns ``(idx int64[k] ascending, val uint16[k] = FP16 bit patterns)``."""
    W = _c(W)
    d_in, d_out = W.shape
    bits = _c(bits, np.uint8)
    cent = None if centroids is None else _c(centroids, np.float32)
    cd = None if codes is None else _c(codes, np.uint8)
    idx = np.zeros(max(k, 1), np.int64)
    val = np.zeros(max(k, 1), np.uint16)
    rc = lib().orc_weight_outliers(_p(W), _dtype_code(W), ctypes.c_int64(d_in), ctypes.c_int64(d_out),
                                   ctypes.c_int64(d_out), _p(cent), _p(cd), _p(bits), int(score),
                                   ctypes.c_int64(k), _p(idx), _p(val))
    if rc != 0:
        raise ValueError(f"orc_weight_outliers rc={rc}")
    return idx[:k], val[:k]


def weight_outliers_per_channel(W: np.ndarray, centroids: Optional[np.ndarray], codes: Optional[np.ndarray],
                                bits: np.ndarray, k: int, score: int = SCORE_RESIDUAL):
    """The variant of O_q with `k` entries in every channel whose width is in 1..4.  Returns
    ``(idx int64[k * n_live] ascending, val uint16[k * n_live] = FP16 bit patterns)``."""
    W = _c(W)
    d_in, d_out = W.shape
    bits = _c(bits, np.uint8)
    cent = None if centroids is None else _c(centroids, np.float32)
    cd = None if codes is None else _c(codes, np.uint8)
    n_live = int(((bits >= 1) & (bits <= 4)).sum())
    idx = np.zeros(max(k * n_live, 1), np.int64)
    val = np.zeros(max(k * n_live, 1), np.uint16)
    n = lib().orc_weight_outliers_per_channel(_p(W), _dtype_code(W), ctypes.c_int64(d_in), ctypes.c_int64(d_out),
                                              ctypes.c_int64(d_out), _p(cent), _p(cd), _p(bits), int(score),
                                              ctypes.c_int64(k), _p(idx), _p(val))
    if n < 0:
        raise ValueError(f"orc_weight_outliers_per_channel rc={n}")
    assert n == k * n_live, (n, k, n_live)
    return idx[:n], val[:n]


def pack(codes: np.ndarray, bits: np.ndarray, centroids: np.ndarray, b: int):
    """Returns ``(packed uint32[rows, ceil(d_out*b/32)], chan_idx int32[rows], lut uint16[rows, 2^b])``."""
    codes = _c(codes, np.uint8)
    d_in, d_out = codes.shape
    bits = _c(bits, np.uint8)
    cent = _c(centroids, np.float32)
    rows = int((bits == b).sum())
    wpr = (d_out * b + 31) // 32
    packed = np.zeros((max(rows, 1), max(wpr, 1)), np.uint32)
    chan = np.zeros(max(rows, 1), np.int32)
    lut = np.zeros((max(rows, 1), 1 << b), np.uint16)
    r = lib().orc_pack(_p(codes), ctypes.c_int64(d_in), ctypes.c_int64(d_out), _p(bits), _p(cent),
                       int(b), _p(packed), _p(chan), _p(lut))
    assert r == rows, (r, rows)
    return packed[:rows, :wpr], chan[:rows], lut[:rows]


def dequant_error(W: np.ndarray, centroids: np.ndarray, codes: np.ndarray, bits: np.ndarray,
                  out_idx: Optional[np.ndarray] = None, sumsq: Optional[np.ndarray] = None):
    """Returns ``(err_ch float64[d_in], totals float64[2] = [activation weighted, plain])``."""
    W = _c(W)
    d_in, d_out = W.shape
    oi = None if out_idx is None else _c(out_idx, np.int64)
    ss = None if sumsq is None else _c(sumsq, np.float32)
    err = np.zeros(d_in, np.float64)
    tot = np.zeros(2, np.float64)
    rc = lib().orc_dequant_error(_p(W), _dtype_code(W), ctypes.c_int64(d_in), ctypes.c_int64(d_out),
                                 ctypes.c_int64(d_out), _p(_c(centroids, np.float32)),
                                 _p(_c(codes, np.uint8)), _p(_c(bits, np.uint8)), _p(oi),
                                 ctypes.c_int64(0 if oi is None else oi.shape[0]), _p(ss),
                                 _p(err), _p(tot))
    assert rc == 0, rc
    return err, tot


def lut_matvec(X: np.ndarray, W: np.ndarray, centroids: np.ndarray, codes: np.ndarray, bits: np.ndarray,
               out_idx: Optional[np.ndarray] = None) -> np.ndarray:
    """Fig. 4: ``Y float64[m, d_out] = X [m, d_in] @ W_hat`` with the deployed W_hat (FP16 LUT
    levels, outliers as FP16 weights)."""
    X = _c(X)
    W = _c(W)
    m, d_in = X.shape
    d_in2, d_out = W.shape
    assert d_in == d_in2
    oi = None if out_idx is None else _c(out_idx, np.int64)
    Y = np.zeros((m, d_out), np.float64)
    rc = lib().orc_lut_matvec(_p(X), _dtype_code(X), ctypes.c_int64(m), ctypes.c_int64(d_in),
                              ctypes.c_int64(d_in), _p(W), _dtype_code(W), ctypes.c_int64(d_out),
                              ctypes.c_int64(d_out), _p(_c(centroids, np.float32)), _p(_c(codes, np.uint8)),
                              _p(_c(bits, np.uint8)), _p(oi), ctypes.c_int64(0 if oi is None else oi.shape[0]),
                              _p(Y))
    assert rc == 0, rc
    return Y


def rtn_quantize(W: np.ndarray, bits: np.ndarray, group: int = 128):
    """App. A.2: round-to-nearest with the uniform quantizer of Sec. 3, groups of `group`
    consecutive outputs per input channel.  Returns ``(codes uint8[d_in, d_out],
    scale float32[d_in, n_groups], zero float32[d_in, n_groups], err_ch float64[d_in])``."""
    W = _c(W)
    d_in, d_out = W.shape
    ng = (d_out + group - 1) // group
    codes = np.zeros((d_in, d_out), np.uint8)
    scale = np.zeros((d_in, ng), np.float32)
    zero = np.zeros((d_in, ng), np.float32)
    err = np.zeros(d_in, np.float64)
    rc = lib().orc_rtn_quantize(_p(W), _dtype_code(W), ctypes.c_int64(d_in), ctypes.c_int64(d_out),
                                ctypes.c_int64(d_out), _p(_c(bits, np.uint8)), ctypes.c_int64(int(group)),
                                _p(codes), _p(scale), _p(zero), _p(err))
    assert rc == 0, rc
    return codes, scale, zero, err


def lut4(centroids: np.ndarray, bits: np.ndarray):
    """Sec. 5.1 / Tab. 7: the look-up tables in 4 bits, one uniform grid per layer.  Returns
    ``(codes4 uint8[d_in,16], range float32[2] = [min, step], centroids_q float32[d_in,16])``."""
    cent = _c(centroids, np.float32)
    d_in = cent.shape[0]
    codes4 = np.zeros((d_in, KMAX), np.uint8)
    rng = np.zeros(2, np.float32)
    cq = np.zeros((d_in, KMAX), np.float32)
    rc = lib().orc_lut4(_p(cent), _p(_c(bits, np.uint8)), ctypes.c_int64(d_in), _p(codes4), _p(rng), _p(cq))
    assert rc == 0, rc
    return codes4, rng, cq


def lut4_codebook(centroids: np.ndarray, bits: np.ndarray, iters: int = 20):
    """Sec. 5.1 / Tab. 7: the look-up tables in 4 bits, as codes into one 16-entry table per layer
    found by K-means over all the layer's FP16 centres.  Returns ``(codes4 uint8[d_in,16],
    table float32[16], centroids_q float32[d_in,16])``."""
    cent = _c(centroids, np.float32)
    d_in = cent.shape[0]
    codes4 = np.zeros((d_in, KMAX), np.uint8)
    table = np.zeros(KMAX, np.float32)
    cq = np.zeros((d_in, KMAX), np.float32)
    rc = lib().orc_lut4_codebook(_p(cent), _p(_c(bits, np.uint8)), ctypes.c_int64(d_in), int(iters), _p(codes4),
                                 _p(table), _p(cq))
    assert rc == 0, rc
    return codes4, table, cq


def quantize_layer(W: np.ndarray, X: np.ndarray, bit_set: Sequence[int], avg_bits: float,
                   rho_act_ppm: int = 4500, rho_q_ppm: int = 500, iters: int = 20,
                   sumsq: Optional[np.ndarray] = None, score: int = SCORE_RESIDUAL,
                   iters_final_from_prelim: Optional[int] = None, per_channel: bool = False) -> dict:
    """The whole path of Sec. 3.2, step by step, on one layer.

    ``W`` is ``[d_in, d_out]`` (paper orientation), ``X`` is ``[n, d_in]``.
    ``iters_final_from_prelim`` (variant): the final K-means starts from the levels of the
    preliminary one and runs that many rounds, instead of `iters` rounds from the quantile start.
    ``per_channel`` (variant): O_q takes ``round_half_up(rho_q * d_out)`` entries in every channel
    outside O_act instead of ``round_half_up(rho_q * d_in * d_out)`` over the layer.
    """
    d_in, d_out = W.shape
    if sumsq is None:
        _, sumsq = act_stats(X)
    k_act = count_ppm(rho_act_ppm, d_in)
    act_idx, chan_mask = top_channels(sumsq, k_act)                      # O_act
    bits, counts = allocate_bits(sumsq, chan_mask, bit_set, avg_bits)     # Algorithm 1 on W'
    cent1, codes1 = kmeans(W, bits, iters=iters)                          # W'_q
    if per_channel:
        out_idx, out_val = weight_outliers_per_channel(W, cent1, codes1, bits, count_ppm(rho_q_ppm, d_out), score)
    else:
        k_q = count_ppm(rho_q_ppm, d_in * d_out)
        out_idx, out_val = weight_outliers(W, cent1, codes1, bits, k_q, score)  # O_q
    if iters_final_from_prelim is None:
        cent, codes = kmeans(W, bits, out_idx=out_idx, iters=iters)       # W_q
    else:
        cent, codes = kmeans(W, bits, out_idx=out_idx, iters=iters_final_from_prelim, start=cent1)
    packs = {b: pack(codes, bits, cent, b) for b in bit_set}
    err_ch, totals = dequant_error(W, cent, codes, bits, out_idx, sumsq)
    return dict(sumsq=sumsq, act_idx=act_idx, chan_mask=chan_mask, bits=bits, counts=counts,
                cent1=cent1, codes1=codes1, out_idx=out_idx, out_val=out_val, centroids=cent,
                codes=codes, packs=packs, err_ch=err_ch, totals=totals)
