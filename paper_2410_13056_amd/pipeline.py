"""Host driver of the CMPQ quantization path: the order of Sec. 3.2 of
arXiv 2410.13056, one C-ABI call per step.  Nothing is computed here; the code
allocates outputs, derives integer counts from shapes and chains the calls on the
current stream without synchronising.
"""
from __future__ import annotations

import contextlib
import dataclasses
from typing import Dict, List, Optional, Sequence

import torch

from . import binding as B


# the kernel that dominates each stage: `StageTimer(kernels=True)` times it by itself
_KERNEL_OF_STAGE = {"act_stats": B.KERNEL_ACT_STATS, "transpose": B.KERNEL_TRANSPOSE,
                    "kmeans_prelim": B.KERNEL_KMEANS, "kmeans_final": B.KERNEL_KMEANS,
                    "outlier_weights": B.KERNEL_OUTLIER_STAGE, "pack_with_error": B.KERNEL_PACK_ERROR}


class StageTimer:
    """Brackets each C-ABI call with a pair of events on the stream the call is
    enqueued on; `totals()` returns {stage: (calls, milliseconds)} once they ran.

    With ``kernels=True`` the library's measurement hook also brackets the one kernel that
    dominates the stage (`cmpq_time_kernel`: events recorded right before and after that launch,
    on its stream); `kernel_totals()` returns the same shape for those."""

    def __init__(self, kernels: bool = False):
        self.pairs: Dict[str, list] = {}
        self.kpairs: Dict[str, list] = {}
        self.kernels = kernels

    @contextlib.contextmanager
    def stage(self, name: str):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        kid = _KERNEL_OF_STAGE.get(name) if self.kernels else None
        if kid is not None:
            k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            k0.record(), k1.record()          # creates the handles; the library records them again
            B.time_kernel(kid, k0.cuda_event, k1.cuda_event)
        a.record()
        yield
        b.record()
        self.pairs.setdefault(name, []).append((a, b))
        if kid is not None:
            B.time_kernel(kid, None, None)    # in case the call took a path without that kernel
            self.kpairs.setdefault(name, []).append((k0, k1))

    def totals(self) -> Dict[str, tuple]:
        torch.cuda.synchronize()
        return {k: (len(v), sum(a.elapsed_time(b) for a, b in v)) for k, v in self.pairs.items()}

    def kernel_totals(self) -> Dict[str, tuple]:
        torch.cuda.synchronize()
        return {k: (len(v), sum(a.elapsed_time(b) for a, b in v)) for k, v in self.kpairs.items()}


def _stage(timer: Optional[StageTimer], name: str):
    return timer.stage(name) if timer is not None else contextlib.nullcontext()


@dataclasses.dataclass
class LayerResult:
    """Everything the path produces for one linear layer (device tensors)."""
    d_in: int
    d_out: int
    bit_set: Sequence[int]
    counts: List[int]                 # channels per width
    sumsq: torch.Tensor               # [d_in] fp32 activation statistic
    act_idx: torch.Tensor             # [k_act] int32: channels of O_act
    chan_mask: torch.Tensor           # [d_in] uint8
    bits: torch.Tensor                # [d_in] uint8 (16 = O_act channel)
    centroids: torch.Tensor           # [d_in,16] fp32 levels of the final quantizer
    codes: torch.Tensor               # [d_in,d_out] uint8
    out_idx: torch.Tensor             # [k_q] int32 linear indices i*d_out+o of O_q
    out_val: torch.Tensor             # [k_q] fp16 values of O_q
    packed: List[Optional[torch.Tensor]]    # per width: [rows, ceil(d_out*b/32)] int32 words
    chan_idx: List[Optional[torch.Tensor]]  # per width: [rows] int32
    lut: List[Optional[torch.Tensor]]       # per width: [rows, 2^b] fp16
    centroids_prelim: Optional[torch.Tensor] = None
    codes_prelim: Optional[torch.Tensor] = None
    err_ch: Optional[torch.Tensor] = None
    err_total: Optional[torch.Tensor] = None
    W_t: Optional[torch.Tensor] = None      # the d_in x d_out copy the steps ran on


def activation_stats(X: torch.Tensor, ws: B.Workspace, acc: Optional[torch.Tensor] = None,
                     status: Optional[torch.Tensor] = None, timer: Optional[StageTimer] = None):
    """Sec. 3.2.1: per-channel sum of squares of X [n, d_in]; pass `acc` to add more tokens."""
    d_in = X.shape[1]
    first = acc is None
    if first:
        acc = torch.empty(d_in, dtype=torch.float64, device=X.device)
    sumsq = torch.empty(d_in, dtype=torch.float32, device=X.device)
    with _stage(timer, "act_stats"):
        B.act_stats(X, acc, sumsq, not first, ws, status)
    return acc, sumsq


def _oriented(W: torch.Tensor, transposed: bool, timer):
    """The d_in x d_out copy the steps run on."""
    if transposed:
        return W
    d_out, d_in = W.shape
    Wt = torch.empty((d_in, d_out), dtype=W.dtype, device=W.device)
    with _stage(timer, "transpose"):
        B.transpose(W, Wt)
    return Wt


def _channels_and_widths(sumsq, d_in, bit_set, avg_bits, rho_act_ppm, ws, timer):
    """O_act (Sec. 3.2.2), then Algorithm 1 on W' = W - O_act.  Both depend on the statistic of
    the layer's input only, not on its weights."""
    dev = sumsq.device
    k_act = B.count_ppm(rho_act_ppm, d_in)
    act_idx = torch.empty(k_act, dtype=torch.int32, device=dev)
    chan_mask = torch.empty(d_in, dtype=torch.uint8, device=dev)
    with _stage(timer, "outlier_channels"):
        B.extract_channel_outliers(sumsq, k_act, act_idx, chan_mask, ws)
    bits = torch.empty(d_in, dtype=torch.uint8, device=dev)
    with _stage(timer, "allocate_bits"):
        counts = B.allocate_bits(sumsq, chan_mask, k_act, bit_set, avg_bits, bits, ws)
    return act_idx, chan_mask, bits, counts


def _histogram_kernel_takes(Wt: torch.Tensor) -> bool:
    """Whether the histogram K-means kernel runs on this input (fp16, rows of whole groups of 4
    entries, 8-byte aligned, a length it has a launch shape for): only it keeps per-channel
    tables and leaves the coding pass out when no codes are asked for."""
    d_in, d_out = Wt.shape
    if Wt.dtype != torch.float16 or d_out % 4 or Wt.data_ptr() % 8 or (d_in > 1 and Wt.stride(0) % 4):
        return False
    return B.arrangement_bytes(d_in, d_out) > 0


def _shared_tables(Wt: torch.Tensor) -> Optional[torch.Tensor]:
    """The buffer through which the preliminary K-means of a layer hands its per-channel tables
    to the final one (`cmpq_kmeans_job.arrangement`), or None where the histogram kernel would
    not take the input."""
    if not _histogram_kernel_takes(Wt):
        return None
    return torch.empty(B.arrangement_bytes(*Wt.shape), dtype=torch.uint8, device=Wt.device)


def _after_first_pass(Wt, sumsq, bit_set, counts, act_idx, chan_mask, bits, cent1, codes1, rho_q_ppm, iters,
                      ws, score, with_error, keep_prelim, status, timer,
                      iters_final_from_prelim: Optional[int] = None, oq_per_channel: bool = False,
                      fused: bool = True, tables: Optional[torch.Tensor] = None) -> LayerResult:
    """O_q from the preliminary quantization, the final quantization, the stored format."""
    dev = Wt.device
    d_in, d_out = Wt.shape
    # O_q: largest |W' - W'_q|, over the layer (Sec. 3.2.2) or, as a variant, per channel
    if oq_per_channel:
        k_each = B.count_ppm(rho_q_ppm, d_out)
        k_q = k_each * sum(counts)
    else:
        k_each = k_q = B.count_ppm(rho_q_ppm, d_in * d_out)
    out_idx = torch.empty(k_q, dtype=torch.int32, device=dev)
    out_val = torch.empty(k_q, dtype=torch.float16, device=dev)
    with _stage(timer, "outlier_weights"):
        B.extract_weight_outliers(Wt, cent1, codes1, bits, k_each, out_idx, out_val, ws, score,
                                  B.SCOPE_CHANNEL if oq_per_channel else B.SCOPE_LAYER)
    # stored format: one block of packed rows, channel list and FP16 tables per width
    packed, chan_idx, lut = [], [], []
    for b, c in zip(bit_set, counts):
        if c == 0:
            packed.append(None), chan_idx.append(None), lut.append(None)
            continue
        packed.append(torch.empty((c, (d_out * b + 31) // 32), dtype=torch.int32, device=dev))
        chan_idx.append(torch.empty(c, dtype=torch.int32, device=dev))
        lut.append(torch.empty((c, 1 << b), dtype=torch.float16, device=dev))
    # final quantization of W - O
    codes = torch.empty((d_in, d_out), dtype=torch.uint8, device=dev)
    given = iters_final_from_prelim is not None
    # variant: continue from the preliminary levels (a copy; the call updates it in place)
    cent = cent1.clone() if given else torch.empty((d_in, B.KMAX), dtype=torch.float32, device=dev)
    rounds, init = (iters_final_from_prelim, B.INIT_GIVEN) if given else (iters, B.INIT_QUANTILE)
    reuse = B.ARRANGEMENT_REUSE if tables is not None else B.ARRANGEMENT_NONE
    res = LayerResult(d_in, d_out, tuple(bit_set), counts, sumsq, act_idx, chan_mask, bits, cent, codes,
                      out_idx, out_val, packed, chan_idx, lut, W_t=Wt)
    if keep_prelim:
        res.centroids_prelim, res.codes_prelim = cent1, codes1
    if with_error:
        res.err_ch = torch.empty(d_in, dtype=torch.float64, device=dev)
        res.err_total = torch.empty(2, dtype=torch.float64, device=dev)
    if with_error and fused:
        # one call: the coding pass of the final K-means writes the stored format and the error
        with _stage(timer, "kmeans_final"):
            B.kmeans_quantize_pack(Wt, bits, out_idx, k_q, rounds, cent, codes, bit_set, counts, packed, chan_idx,
                                   lut, sumsq, res.err_ch, res.err_total, ws, status, init=init,
                                   arrangement=tables, arrangement_use=reuse)
        return res
    with _stage(timer, "kmeans_final"):
        B.kmeans_quantize(Wt, bits, out_idx, k_q, None, rounds, cent, codes, ws, status, init=init,
                          arrangement=tables, arrangement_use=reuse)
    if with_error:      # stored format and error in one pass over the codes
        with _stage(timer, "pack_with_error"):
            B.pack_with_error(Wt, codes, bits, cent, bit_set, counts, packed, chan_idx, lut, out_idx, k_q, sumsq,
                              res.err_ch, res.err_total, ws)
    else:
        with _stage(timer, "pack"):
            B.pack(codes, bits, cent, bit_set, counts, packed, chan_idx, lut, ws)
    return res


def quantize_layer(W: torch.Tensor, sumsq: torch.Tensor, bit_set: Sequence[int], avg_bits: float,
                   rho_act_ppm: int = 4500, rho_q_ppm: int = 500, iters: int = 20,
                   ws: Optional[B.Workspace] = None, score: int = B.SCORE_RESIDUAL,
                   with_error: bool = False, keep_prelim: bool = False,
                   status: Optional[torch.Tensor] = None, transposed: bool = False,
                   timer: Optional[StageTimer] = None,
                   iters_final_from_prelim: Optional[int] = None, oq_per_channel: bool = False,
                   fused: bool = True, share_tables: bool = True, prelim_codes: bool = False,
                   widths=None) -> LayerResult:
    """Quantizes one layer.  `W` is the framework's [d_out, d_in] weight (or already
    d_in x d_out with ``transposed=True``); `sumsq` comes from `activation_stats`.

    ``oq_per_channel`` (a variant; Sec. 3.2.2 selects over the layer): O_q takes
    ``round_half_up(rho_q * d_out)`` entries in every channel outside O_act.

    ``fused`` (with ``with_error``): the final K-means writes the stored format and the error
    from its coding pass (`cmpq_kmeans_quantize_job`); ``fused=False`` runs `cmpq_kmeans_quantize`
    and `cmpq_pack_with_error` one after the other.  Same results.

    ``prelim_codes`` (off by default): the preliminary K-means also writes its codes and O_q reads
    them, as the calls were first laid out.  Same results; off, the preliminary run leaves only
    its levels and O_q ranks the distance to the nearest level (one byte per weight less written
    and read again), where the histogram kernel runs.

    ``widths``: what `channels_and_widths` returned for this statistic, channel count, bit set,
    average width and share of O_act - layers that read the same input have the same O_act and
    the same widths, so a block ranks and allocates once per input.

    ``share_tables`` (on by default): the preliminary K-means leaves its per-channel tables for
    the final one (`cmpq_kmeans_job.arrangement`), which then does not build them again.  Same
    results, one buffer of about `d_in * (d_out + 8 KiB)` bytes more while the layer is in work;
    measured, the final pass is 10 % shorter and the whole step 2 %.

    ``iters_final_from_prelim`` (a variant; the paper names no start for either K-means of
    Sec. 3.2.2): the final quantization starts from the levels of the preliminary one and runs
    that many rounds, instead of `iters` rounds from the quantile start."""
    ws = ws or B.Workspace(W.device)
    dev = W.device
    Wt = _oriented(W, transposed, timer)
    d_in, d_out = Wt.shape
    if widths is None:
        widths = _channels_and_widths(sumsq, d_in, bit_set, avg_bits, rho_act_ppm, ws, timer)
    act_idx, chan_mask, bits, counts = widths
    # preliminary quantization W'_q.  Only its levels are needed further on: O_q ranks
    # |w - nearest level|, which is |W' - W'_q| (Sec. 3 eq. Q(x)), so where the kernel can leave
    # the codes out they are neither written nor read.
    cent1 = torch.empty((d_in, B.KMAX), dtype=torch.float32, device=dev)
    codes1 = None
    if keep_prelim or prelim_codes or not _histogram_kernel_takes(Wt):
        codes1 = torch.empty((d_in, d_out), dtype=torch.uint8, device=dev)
    tables = _shared_tables(Wt) if share_tables else None
    with _stage(timer, "kmeans_prelim"):
        B.kmeans_quantize(Wt, bits, None, 0, None, iters, cent1, codes1, ws, status, arrangement=tables,
                          arrangement_use=B.ARRANGEMENT_KEEP if tables is not None else B.ARRANGEMENT_NONE)
    return _after_first_pass(Wt, sumsq, bit_set, counts, act_idx, chan_mask, bits, cent1, codes1, rho_q_ppm,
                             iters, ws, score, with_error, keep_prelim, status, timer, iters_final_from_prelim,
                             oq_per_channel, fused, tables)


@dataclasses.dataclass
class WidthCache:
    """One preliminary K-means run per width over all channels of a layer (device tensors):
    what `quantize_layer_from_cache` needs to retarget the layer to any average width."""
    bit_set: Sequence[int]
    iters: int
    W_t: torch.Tensor                 # [d_in, d_out]
    centroids: List[torch.Tensor]     # per width: [d_in, 16] fp32
    codes: List[torch.Tensor]         # per width: [d_in, d_out] uint8


def build_width_cache(W: torch.Tensor, bit_set: Sequence[int], iters: int = 20,
                      ws: Optional[B.Workspace] = None, status: Optional[torch.Tensor] = None,
                      transposed: bool = False, timer: Optional[StageTimer] = None) -> WidthCache:
    """Runs the preliminary K-means of Sec. 3.2.2 once per width of `bit_set` over every
    channel.  A channel's levels and codes do not depend on the other channels' widths, so
    these runs hold the first pass of every possible allocation."""
    ws = ws or B.Workspace(W.device)
    dev = W.device
    Wt = _oriented(W, transposed, timer)
    d_in, d_out = Wt.shape
    cents, codes = [], []
    for b in bit_set:
        bits_b = torch.full((d_in,), int(b), dtype=torch.uint8, device=dev)
        c = torch.empty((d_in, B.KMAX), dtype=torch.float32, device=dev)
        k = torch.empty((d_in, d_out), dtype=torch.uint8, device=dev)
        with _stage(timer, "kmeans_prelim"):
            B.kmeans_quantize(Wt, bits_b, None, 0, None, iters, c, k, ws, status)
        cents.append(c), codes.append(k)
    return WidthCache(tuple(bit_set), iters, Wt, cents, codes)


def quantize_layer_from_cache(cache: WidthCache, sumsq: torch.Tensor, avg_bits: float,
                              rho_act_ppm: int = 4500, rho_q_ppm: int = 500,
                              ws: Optional[B.Workspace] = None, score: int = B.SCORE_RESIDUAL,
                              with_error: bool = False, keep_prelim: bool = False,
                              status: Optional[torch.Tensor] = None,
                              timer: Optional[StageTimer] = None,
                              iters_final_from_prelim: Optional[int] = None, fused: bool = True) -> LayerResult:
    """`quantize_layer` for another average width (or other outlier fractions) of a layer
    whose per-width runs are kept: the first K-means pass is a row-wise choice among them,
    everything after it runs as usual.  Same results as `quantize_layer`, bit for bit."""
    ws = ws or B.Workspace(cache.W_t.device)
    dev = cache.W_t.device
    d_in, d_out = cache.W_t.shape
    act_idx, chan_mask, bits, counts = _channels_and_widths(sumsq, d_in, cache.bit_set, avg_bits, rho_act_ppm,
                                                            ws, timer)
    cent1 = torch.empty((d_in, B.KMAX), dtype=torch.float32, device=dev)
    codes1 = torch.empty((d_in, d_out), dtype=torch.uint8, device=dev)
    with _stage(timer, "select_by_width"):
        B.select_by_width(bits, cache.bit_set, cache.centroids, cache.codes, cent1, codes1)
    return _after_first_pass(cache.W_t, sumsq, cache.bit_set, counts, act_idx, chan_mask, bits, cent1, codes1,
                             rho_q_ppm, cache.iters, ws, score, with_error, keep_prelim, status, timer,
                             iters_final_from_prelim, False, fused)


def tables_in_4_bits(r: LayerResult, ws: Optional[B.Workspace] = None, with_error: bool = False,
                     timer: Optional[StageTimer] = None, mode: int = B.LUT4_CODEBOOK, iters: int = 20):
    """Sec. 5.1 / Tab. 7: re-expresses the look-up tables of a quantized layer in 4 bits per entry -
    codes into one 16-level table per layer (default) or on one uniform grid (``mode =
    B.LUT4_UNIFORM``) - and writes the stored format again with them.  Returns ``(codes4 [d_in,16]
    uint8, table [16] fp32 (the levels; minimum and step in the first two entries for the uniform
    grid), LayerResult with the rebuilt tables)``."""
    ws = ws or B.Workspace(r.codes.device)
    dev = r.codes.device
    codes4 = torch.empty((r.d_in, B.KMAX), dtype=torch.uint8, device=dev)
    rng = torch.zeros(B.KMAX, dtype=torch.float32, device=dev)
    cent_q = torch.empty((r.d_in, B.KMAX), dtype=torch.float32, device=dev)
    with _stage(timer, "lut4"):
        B.lut4_quantize(r.centroids, r.bits, codes4, rng, cent_q, ws, mode, iters)
    packed, chan_idx, lut = [], [], []
    for b, c in zip(r.bit_set, r.counts):
        if c == 0:
            packed.append(None), chan_idx.append(None), lut.append(None)
            continue
        packed.append(torch.empty((c, (r.d_out * b + 31) // 32), dtype=torch.int32, device=dev))
        chan_idx.append(torch.empty(c, dtype=torch.int32, device=dev))
        lut.append(torch.empty((c, 1 << b), dtype=torch.float16, device=dev))
    with _stage(timer, "pack"):
        B.pack(r.codes, r.bits, cent_q, r.bit_set, r.counts, packed, chan_idx, lut, ws)
    q = dataclasses.replace(r, centroids=cent_q, packed=packed, chan_idx=chan_idx, lut=lut, err_ch=None,
                            err_total=None)
    if with_error:
        q.err_ch = torch.empty(r.d_in, dtype=torch.float64, device=dev)
        q.err_total = torch.empty(2, dtype=torch.float64, device=dev)
        with _stage(timer, "dequant_error"):
            B.dequant_error(r.W_t, cent_q, r.codes, r.bits, r.out_idx, int(r.out_idx.numel()), r.sumsq, q.err_ch,
                            q.err_total, ws)
    return codes4, rng, q


@dataclasses.dataclass
class RtnResult:
    """A layer quantized with the uniform quantizer (App. A.2; device tensors)."""
    d_in: int
    d_out: int
    group: int
    bit_set: Sequence[int]
    counts: List[int]
    sumsq: torch.Tensor
    act_idx: torch.Tensor             # [k_act] int32: channels of O_act
    chan_mask: torch.Tensor
    bits: torch.Tensor                # [d_in] uint8 (16 = O_act channel)
    codes: torch.Tensor               # [d_in, d_out] uint8
    scale: torch.Tensor               # [d_in, ceil(d_out/group)] fp32 step of each group
    zero: torch.Tensor                # [d_in, ceil(d_out/group)] fp32 minimum of each group
    err_ch: Optional[torch.Tensor] = None
    W_t: Optional[torch.Tensor] = None


def quantize_layer_rtn(W: torch.Tensor, sumsq: torch.Tensor, bit_set: Sequence[int], avg_bits: float,
                       rho_act_ppm: int = 5000, group: int = 128, ws: Optional[B.Workspace] = None,
                       with_error: bool = False, status: Optional[torch.Tensor] = None,
                       transposed: bool = False, timer: Optional[StageTimer] = None) -> RtnResult:
    """App. A.2 (Tab. 10): the channel-wise widths of Algorithm 1 with round-to-nearest on a
    uniform grid per group of `group` outputs instead of K-means; 0.5 % of the channels stay
    FP16 by default and no single weights are taken out."""
    ws = ws or B.Workspace(W.device)
    dev = W.device
    Wt = _oriented(W, transposed, timer)
    d_in, d_out = Wt.shape
    act_idx, chan_mask, bits, counts = _channels_and_widths(sumsq, d_in, bit_set, avg_bits, rho_act_ppm, ws, timer)
    n_groups = -(-d_out // group)
    codes = torch.empty((d_in, d_out), dtype=torch.uint8, device=dev)
    scale = torch.empty((d_in, n_groups), dtype=torch.float32, device=dev)
    zero = torch.empty((d_in, n_groups), dtype=torch.float32, device=dev)
    err_ch = torch.empty(d_in, dtype=torch.float64, device=dev) if with_error else None
    with _stage(timer, "rtn"):
        B.rtn_quantize(Wt, bits, group, codes, scale, zero, err_ch, status)
    return RtnResult(d_in, d_out, group, tuple(bit_set), counts, sumsq, act_idx, chan_mask, bits, codes,
                     scale, zero, err_ch, Wt)


@dataclasses.dataclass
class Deployed:
    """A layer as the product kernel of Fig. 4 reads it (device tensors)."""
    d_in: int
    d_out: int
    bit_set: Sequence[int]
    counts: List[int]
    packed: List[Optional[torch.Tensor]]
    chan_idx: List[Optional[torch.Tensor]]
    lut: List[Optional[torch.Tensor]]
    act_idx: torch.Tensor             # [k_act] int32
    W_act: torch.Tensor               # [k_act, d_out] fp16 rows of O_act
    colptr: torch.Tensor              # [d_out+1] int32: O_q grouped by output column
    row_idx: torch.Tensor             # [k_q] int32
    delta: torch.Tensor               # [k_q] fp32: outlier value minus the table level it overrides
    _call: Optional[B.LutMatvecCall] = None

    def call(self) -> B.LutMatvecCall:
        """The layer's fixed call arguments, marshalled at the first use."""
        if self._call is None:
            self._call = B.LutMatvecCall(self.d_in, self.d_out, self.bit_set, self.counts, self.packed,
                                         self.chan_idx, self.lut, self.act_idx, self.W_act, self.colptr,
                                         self.row_idx, self.delta)
        return self._call

    def matvec_into(self, X: torch.Tensor, Y: torch.Tensor, ws: B.Workspace) -> None:
        """Y [m, d_out] fp32 = X [m, d_in] fp16 times this weight."""
        self.call()(X, Y, ws)


def prepare_deployment(r: LayerResult, ws: Optional[B.Workspace] = None,
                       timer: Optional[StageTimer] = None) -> Deployed:
    """Sec. 6: what deployment keeps of a quantized layer - the packed streams of
    `quantize_layer`, the FP16 rows of O_act and O_q regrouped by output column."""
    ws = ws or B.Workspace(r.codes.device)
    dev = r.codes.device
    k_act, k_q = int(r.act_idx.numel()), int(r.out_idx.numel())
    W_act = torch.empty((k_act, r.d_out), dtype=torch.float16, device=dev)
    colptr = torch.empty(r.d_out + 1, dtype=torch.int32, device=dev)
    row_idx = torch.empty(k_q, dtype=torch.int32, device=dev)
    delta = torch.empty(k_q, dtype=torch.float32, device=dev)
    with _stage(timer, "prepare_deployment"):
        B.gather_channels(r.W_t, r.act_idx, W_act)
        B.outliers_by_column(r.out_idx, r.out_val.view(torch.int16), k_q, r.d_in, r.d_out, r.centroids, r.codes,
                             colptr, row_idx, delta, ws)
    return Deployed(r.d_in, r.d_out, tuple(r.bit_set), list(r.counts), r.packed, r.chan_idx, r.lut,
                    r.act_idx, W_act, colptr, row_idx, delta)


def lut_matvec(dep: Deployed, X: torch.Tensor, ws: Optional[B.Workspace] = None,
               timer: Optional[StageTimer] = None) -> torch.Tensor:
    """Fig. 4: Y [m, d_out] fp32 = X [m, d_in] fp16 times the deployed weight."""
    ws = ws or B.Workspace(X.device)
    Y = torch.empty((X.shape[0], dep.d_out), dtype=torch.float32, device=X.device)
    with _stage(timer, "lut_matvec"):
        dep.matvec_into(X, Y, ws)
    return Y


def group_products(deps: Sequence[Deployed], fp16acc: bool = False) -> B.LutMatvecGroupCall:
    """Sec. 6: several deployed layers whose products may run side by side (the projections that
    read the same input, or any independent ones) as one pair of launches:
    ``group_products(deps)(Xs, Ys, ws)``.  Same results as one `lut_matvec` per layer.
    `fp16acc`: the packed rows are added up in FP16 (``cmpq_lut_matvec_group_fp16acc``)."""
    return B.LutMatvecGroupCall([d.call() for d in deps], fp16acc=fp16acc)


def capture_products(steps: Sequence[tuple], ws: B.Workspace):
    """Sec. 6: the product launches of one token recorded as a HIP graph.  `steps` is a sequence
    of ``(call, Xs, Ys)`` with `call` from `group_products`; the launches go into the graph in
    that order and ``graph.replay()`` submits them at once, which removes the host's share of a
    chain of short launches.  The graph reads and writes the tensors given here: the caller
    puts the next token into `Xs` and takes the result from `Ys` after the replay.  The steps
    run once before recording, so that the workspace has its final size."""
    for call, xs, ys in steps:
        call(xs, ys, ws)
    dev = steps[0][1][0].device
    torch.cuda.synchronize(dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=_streams_for(dev, 1)[0]):
        for call, xs, ys in steps:
            call(xs, ys, ws)
    return graph


_side_streams: Dict[tuple, list] = {}


def _streams_for(device: torch.device, n: int):
    """`n` streams of default priority on `device`, created once and reused."""
    key = (device.type, device.index)
    have = _side_streams.setdefault(key, [])
    while len(have) < n:
        have.append(torch.cuda.Stream(device=device))
    return have[:n]


def assign_layers(sizes: Dict[str, int], streams: int) -> List[tuple]:
    """Shares independent layers out over `streams` queues: largest first (equal sizes in the
    order given), each to the queue with the least work so far, the lowest-numbered of equals.
    Returns (name, queue) pairs in launch order."""
    order = sorted(sizes, key=lambda n: -sizes[n])
    load = [0] * streams
    plan = []
    for name in order:
        j = min(range(streams), key=lambda t: load[t])
        load[j] += sizes[name]
        plan.append((name, j))
    return plan


def quantize_block(weights: Dict[str, torch.Tensor], acts: Dict[str, torch.Tensor], layers, bit_set,
                   avg_bits: float, rho_act_ppm: int, rho_q_ppm: int, iters: int,
                   ws=None, with_error: bool = False, status: Optional[torch.Tensor] = None,
                   timer: Optional[StageTimer] = None, streams: int = 1,
                   join: bool = True, iters_final_from_prelim: Optional[int] = None,
                   fused: bool = True, share_tables: bool = True,
                   prelim_codes: bool = False) -> Dict[str, LayerResult]:
    """One pass of the whole path over a decoder block: statistics once per distinct
    input, then every linear layer.  `layers` lists (name, x_key) pairs.

    Layers do not depend on each other.  With ``streams > 1`` they are shared out over that
    many streams (largest first, to the stream with the least work so far) so that the
    compute-bound k-means of one layer runs beside the memory-bound steps of another; `ws`
    is then a list with one workspace per stream.  The call returns with everything
    enqueued and the current stream waiting for the others.

    ``iters_final_from_prelim``: see `quantize_layer` (a variant, off by default).

    With ``join=False`` the current stream does not wait: the streams run on into the next
    call (a model is quantized block after block, and the queues of one block need not drain
    before those of the next fill), and the caller joins once at the end with `join_streams`."""
    some = next(iter(weights.values()))
    dev = some.device
    if streams <= 1:
        ws = ws or B.Workspace(dev)
        stats = {}
        out = {}
        for name, x_key in layers:
            if x_key not in stats:
                sumsq = activation_stats(acts[x_key], ws, status=status, timer=timer)[1]
                stats[x_key] = (sumsq, _channels_and_widths(sumsq, sumsq.numel(), bit_set, avg_bits, rho_act_ppm,
                                                            ws, timer))
            sumsq, widths = stats[x_key]
            out[name] = quantize_layer(weights[name], sumsq, bit_set, avg_bits, rho_act_ppm,
                                       rho_q_ppm, iters, ws, with_error=with_error, status=status,
                                       timer=timer, iters_final_from_prelim=iters_final_from_prelim, fused=fused,
                                       share_tables=share_tables, prelim_codes=prelim_codes, widths=widths)
        return out
    if ws is None:
        ws = [B.Workspace(dev) for _ in range(streams)]
    if len(ws) != streams:
        raise ValueError("one workspace per stream")
    main = torch.cuda.current_stream(dev)
    side = _streams_for(dev, streams)
    for st in side:
        st.wait_stream(main)
    x_of = dict(layers)
    stats: Dict[str, tuple] = {}          # x_key -> (sumsq, O_act and widths, event, stream index)
    results: Dict[str, LayerResult] = {}
    for name, j in assign_layers({n: weights[n].numel() for n, _ in layers}, streams):
        x_key = x_of[name]
        with torch.cuda.stream(side[j]):
            if x_key not in stats:
                sumsq = activation_stats(acts[x_key], ws[j], status=status, timer=timer)[1]
                # O_act and the widths follow from the statistic alone: once per input, not per layer
                widths = _channels_and_widths(sumsq, sumsq.numel(), bit_set, avg_bits, rho_act_ppm, ws[j], timer)
                ev = torch.cuda.Event()
                ev.record()
                stats[x_key] = (sumsq, widths, ev, j)
            sumsq, widths, ev, owner = stats[x_key]
            if owner != j:
                side[j].wait_event(ev)
                for t in (sumsq,) + tuple(widths[:3]):
                    t.record_stream(side[j])      # its memory is not reused before this stream is done with it
            results[name] = quantize_layer(weights[name], sumsq, bit_set, avg_bits, rho_act_ppm,
                                           rho_q_ppm, iters, ws[j], with_error=with_error,
                                           status=status, timer=timer,
                                           iters_final_from_prelim=iters_final_from_prelim, fused=fused,
                                           share_tables=share_tables, prelim_codes=prelim_codes, widths=widths)
    if join:
        for st in side:
            main.wait_stream(st)
    return {name: results[name] for name, _ in layers}


def join_streams(device, streams: int) -> None:
    """Makes the current stream wait for the streams `quantize_block(..., join=False)` used."""
    main = torch.cuda.current_stream(device)
    for st in _streams_for(torch.device(device), streams):
        main.wait_stream(st)
