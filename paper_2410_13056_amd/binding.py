"""Thin Python binding of libcmpq.so: same names as include/cmpq.h, argument
marshalling only.  Torch tensors supply device memory and the current stream;
every step of the path runs in the library's HIP kernels.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcmpq.so")

OK = 0
F16, F32 = 0, 1
KMAX = 16
PROTECTED = 16
STATUS_NONFINITE = 1
OP_OUTLIERS_BY_COLUMN, OP_LUT_MATVEC, OP_PACK_WITH_ERROR, OP_LUT4, OP_KMEANS_ARRANGEMENT = 7, 8, 9, 10, 11
ARRANGEMENT_NONE, ARRANGEMENT_KEEP, ARRANGEMENT_REUSE = 0, 1, 2
STATUS_ARRANGEMENT = 2
OP_ACT_STATS, OP_ALLOCATE_BITS, OP_OUTLIER_CHANNELS, OP_OUTLIER_WEIGHTS, OP_KMEANS, OP_PACK, \
    OP_DEQUANT_ERROR = range(7)
OUTLIER_CHANNELS, OUTLIER_WEIGHTS = 0, 1
SCORE_RESIDUAL, SCORE_MAGNITUDE = 0, 1
SCOPE_LAYER, SCOPE_CHANNEL = 0, 1
LUT4_CODEBOOK, LUT4_UNIFORM = 0, 1
KERNEL_ACT_STATS, KERNEL_TRANSPOSE, KERNEL_KMEANS, KERNEL_OUTLIER_STAGE, KERNEL_PACK_ERROR = range(5)
INIT_QUANTILE = 0
INIT_GIVEN = 1
KMEANS_HISTOGRAM, KMEANS_DIRECT = 0, 1
NORM_L2, NORM_L1, NORM_LINF = 0, 1, 2

EXPORTS = ("cmpq_workspace_bytes", "cmpq_strerror", "cmpq_count_ppm", "cmpq_act_stats",
           "cmpq_transpose", "cmpq_allocate_bits", "cmpq_extract_outliers",
           "cmpq_kmeans_quantize", "cmpq_pack", "cmpq_dequant_error", "cmpq_kmeans_quantize_job",
           "cmpq_gather_channels", "cmpq_outliers_by_column", "cmpq_lut_matvec", "cmpq_act_stats_norm",
           "cmpq_rtn_quantize", "cmpq_select_by_width", "cmpq_lut_matvec_group", "cmpq_lut4_quantize",
           "cmpq_pack_with_error", "cmpq_time_kernel", "cmpq_act_stats_static", "cmpq_kmeans_launch_shape",
           "cmpq_shader_clock_probe", "cmpq_lut_matvec_group_fp16acc")

_i64, _i32, _int, _vp, _dbl, _sz = (ctypes.c_int64, ctypes.c_int32, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_double, ctypes.c_size_t)
_lib = None


MAX_GROUP = 8


class DeployedLayer(ctypes.Structure):
    """`cmpq_deployed_layer` of the header, field for field."""
    _fields_ = [("X", _vp), ("d_in", _i64), ("ldx", _i64), ("d_out", _i64), ("bit_set", _vp), ("n_set", _int),
                ("counts_host", _vp), ("packed", _vp), ("chan_idx", _vp), ("lut", _vp), ("act_idx", _vp),
                ("W_act", _vp), ("k_act", _i64), ("ld_act", _i64), ("colptr", _vp), ("row_idx", _vp),
                ("delta", _vp), ("Y", _vp), ("ldy", _i64)]


class KmeansJob(ctypes.Structure):
    """`cmpq_kmeans_job` of the header, field for field."""
    _fields_ = [("W", _vp), ("dtype", _int), ("d_in", _i64), ("d_out", _i64), ("ldw", _i64), ("bits", _vp),
                ("out_idx", _vp), ("n_out", _i64), ("elem_weight", _vp), ("iters", _int), ("init", _int),
                ("centroids", _vp), ("codes", _vp), ("status", _vp), ("algorithm", _int),
                ("bit_set", _vp), ("n_set", _int), ("counts_host", _vp), ("packed", _vp), ("chan_idx", _vp),
                ("lut", _vp), ("sumsq", _vp), ("err_ch", _vp), ("err_total", _vp),
                ("arrangement", _vp), ("arrangement_use", _int)]


class CmpqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_13056_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.cmpq_workspace_bytes.restype = _sz
        L.cmpq_workspace_bytes.argtypes = [_int, _i64, _i64, _i64]
        L.cmpq_strerror.restype = ctypes.c_char_p
        L.cmpq_strerror.argtypes = [_int]
        L.cmpq_count_ppm.restype = _i64
        L.cmpq_count_ppm.argtypes = [_i64, _i64]
        L.cmpq_act_stats.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _vp, _int, _vp, _sz, _vp, _vp]
        L.cmpq_transpose.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _i64, _vp]
        L.cmpq_allocate_bits.argtypes = [_vp, _i64, _vp, _i64, _vp, _int, _dbl, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_extract_outliers.argtypes = [_int, _int, _int, _vp, _vp, _int, _i64, _i64, _i64, _vp, _vp,
                                            _vp, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_kmeans_quantize.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _vp, _i64, _vp, _int,
                                           _int, _vp, _vp, _vp, _sz, _vp, _vp]
        L.cmpq_pack.argtypes = [_vp, _i64, _i64, _vp, _vp, _vp, _int, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_dequant_error.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i64, _vp,
                                         _vp, _vp, _vp, _sz, _vp]
        L.cmpq_pack_with_error.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _int, _vp, _vp, _vp, _vp,
                                           _vp, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_kmeans_quantize_job.argtypes = [ctypes.POINTER(KmeansJob), _vp, _sz, _vp]
        L.cmpq_time_kernel.argtypes = [_int, _vp, _vp]
        L.cmpq_kmeans_launch_shape.argtypes = [_i64, _vp]
        L.cmpq_shader_clock_probe.argtypes = [_int, _int, _vp, _vp, _vp]
        L.cmpq_act_stats_static.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _vp, _int, _vp, _vp]
        L.cmpq_act_stats_norm.argtypes = [_vp, _int, _i64, _i64, _i64, _int, _vp, _vp, _int, _vp, _sz, _vp, _vp]
        L.cmpq_gather_channels.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp]
        L.cmpq_outliers_by_column.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_lut_matvec.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _int, _vp, _vp, _vp, _vp, _vp, _vp,
                                      _i64, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]
        L.cmpq_rtn_quantize.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp]
        L.cmpq_lut4_quantize.argtypes = [_int, _vp, _vp, _i64, _int, _vp, _vp, _vp, _vp, _sz, _vp]
        L.cmpq_lut_matvec_group.argtypes = [_vp, _int, _i64, _vp, _sz, _vp]
        L.cmpq_lut_matvec_group_fp16acc.argtypes = [_vp, _int, _i64, _vp, _sz, _vp]
        L.cmpq_select_by_width.argtypes = [_vp, _i64, _i64, _vp, _int, _vp, _vp, _vp, _vp, _vp]
        for name in EXPORTS[3:]:
            getattr(L, name).restype = _int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().cmpq_strerror(int(code)).decode()


def count_ppm(ppm: int, n: int) -> int:
    return int(lib().cmpq_count_ppm(int(ppm), int(n)))


def kmeans_launch_shape(d_out: int):
    """(lanes, groups of 4 per lane, place bits, place-array bytes, dynamic LDS, static LDS) of the
    histogram K-means kernel for channels of `d_out` fp16 weights."""
    shape = (_i64 * 6)()
    _check(lib().cmpq_kmeans_launch_shape(int(d_out), shape), "cmpq_kmeans_launch_shape")
    return tuple(int(v) for v in shape)


def time_kernel(kernel: int, event_begin: Optional[int], event_end: Optional[int]) -> None:
    """Arms the calling thread: the next launch of `kernel` is bracketed by the two events
    (raw hipEvent_t handles as integers); None disarms."""
    _check(lib().cmpq_time_kernel(int(kernel), event_begin, event_end), "cmpq_time_kernel")


def shader_clock_probe(iters: int, ticks: torch.Tensor) -> int:
    """Enqueues the clock probe with one workgroup per row of `ticks` ([n, 2] int64, device);
    returns the wall counter's rate in kHz.  Read `ticks` after synchronising."""
    assert ticks.dtype == torch.int64 and ticks.dim() == 2 and ticks.shape[1] == 2 and ticks.is_contiguous()
    khz = ctypes.c_int(0)
    _check(lib().cmpq_shader_clock_probe(int(iters), int(ticks.shape[0]), _ptr(ticks), ctypes.byref(khz),
                                         _stream()), "cmpq_shader_clock_probe")
    return int(khz.value)


def workspace_bytes(op: int, d_in: int, d_out: int = 0, n: int = 0) -> int:
    return int(lib().cmpq_workspace_bytes(int(op), int(d_in), int(d_out), int(n)))


def _dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"cmpq takes float16 or float32 tensors, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("cmpq entry points take device tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _rows(t: torch.Tensor):
    """(rows, cols, leading dimension) of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D tensor with unit stride along its rows")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    return t.shape[0], t.shape[1], ld


class Workspace:
    """A growable device buffer handed to the library as its scratch space."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = torch.empty(0, dtype=torch.uint8, device=device)

    def get(self, nbytes: int) -> torch.Tensor:
        if self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
        return self.buf


def _check(rc: int, where: str):
    if rc != OK:
        raise CmpqError(rc, where)


def act_stats(X: torch.Tensor, acc: torch.Tensor, sumsq: Optional[torch.Tensor], accumulate: bool,
              ws: Workspace, status: Optional[torch.Tensor] = None) -> None:
    n, d_in, ldx = _rows(X)
    buf = ws.get(workspace_bytes(OP_ACT_STATS, d_in, 0, n))
    _check(lib().cmpq_act_stats(_ptr(X), _dtype(X), n, d_in, ldx, _ptr(acc), _ptr(sumsq),
                                int(bool(accumulate)), _ptr(buf), buf.numel(), _ptr(status), _stream()),
           "cmpq_act_stats")


def act_stats_static(X: torch.Tensor, acc: torch.Tensor, sumsq: Optional[torch.Tensor], accumulate: bool,
                     status: Optional[torch.Tensor] = None) -> None:
    """`act_stats` without a workspace: the library's own fixed scratch array (no allocation)."""
    n, d_in, ldx = _rows(X)
    _check(lib().cmpq_act_stats_static(_ptr(X), _dtype(X), n, d_in, ldx, _ptr(acc), _ptr(sumsq),
                                       int(bool(accumulate)), _ptr(status), _stream()),
           "cmpq_act_stats_static")


def transpose(src: torch.Tensor, dst: torch.Tensor) -> None:
    rows, cols, ld_src = _rows(src)
    r2, c2, ld_dst = _rows(dst)
    if (r2, c2) != (cols, rows) or src.dtype != dst.dtype:
        raise ValueError("dst must be the transposed shape and the same dtype")
    _check(lib().cmpq_transpose(_ptr(src), _dtype(src), rows, cols, ld_src, _ptr(dst), ld_dst, _stream()),
           "cmpq_transpose")


def allocate_bits(sumsq: torch.Tensor, chan_mask: Optional[torch.Tensor], n_protected: int,
                  bit_set: Sequence[int], avg_bits: float, bits: torch.Tensor, ws: Workspace):
    d_in = sumsq.numel()
    bs = (_i32 * len(bit_set))(*bit_set)
    counts = (_i64 * len(bit_set))()
    buf = ws.get(workspace_bytes(OP_ALLOCATE_BITS, d_in))
    _check(lib().cmpq_allocate_bits(_ptr(sumsq), d_in, _ptr(chan_mask), int(n_protected), bs, len(bit_set),
                                    float(avg_bits), _ptr(bits), counts, _ptr(buf), buf.numel(), _stream()),
           "cmpq_allocate_bits")
    return [int(c) for c in counts]


def extract_channel_outliers(sumsq: torch.Tensor, k: int, idx_out: torch.Tensor,
                             chan_mask_out: Optional[torch.Tensor], ws: Workspace) -> None:
    d_in = sumsq.numel()
    buf = ws.get(workspace_bytes(OP_OUTLIER_CHANNELS, d_in, 0, k))
    _check(lib().cmpq_extract_outliers(OUTLIER_CHANNELS, SCORE_RESIDUAL, SCOPE_LAYER, _ptr(sumsq), None, F16, d_in, 0, 0,
                                       None, None, None, int(k), _ptr(idx_out), None, _ptr(chan_mask_out),
                                       _ptr(buf), buf.numel(), _stream()),
           "cmpq_extract_outliers(channels)")


def extract_weight_outliers(W: torch.Tensor, centroids: Optional[torch.Tensor], codes: Optional[torch.Tensor],
                            bits: torch.Tensor, k: int, idx_out: torch.Tensor, val_out: Optional[torch.Tensor],
                            ws: Workspace, score: int = SCORE_RESIDUAL, scope: int = SCOPE_LAYER) -> None:
    """O_q: the `k` largest scores of the layer (SCOPE_LAYER, Sec. 3.2.2) or of every channel
    (SCOPE_CHANNEL: `idx_out` / `val_out` then hold k entries per quantized channel)."""
    d_in, d_out, ldw = _rows(W)
    buf = ws.get(workspace_bytes(OP_OUTLIER_WEIGHTS, d_in, d_out, k))
    _check(lib().cmpq_extract_outliers(OUTLIER_WEIGHTS, int(score), int(scope), None, _ptr(W), _dtype(W), d_in,
                                       d_out, ldw,
                                       _ptr(centroids), _ptr(codes), _ptr(bits), int(k), _ptr(idx_out),
                                       _ptr(val_out), None, _ptr(buf), buf.numel(), _stream()),
           "cmpq_extract_outliers(weights)")


def kmeans_quantize(W: torch.Tensor, bits: torch.Tensor, out_idx: Optional[torch.Tensor], n_out: int,
                    elem_weight: Optional[torch.Tensor], iters: int, centroids: torch.Tensor,
                    codes: torch.Tensor, ws: Workspace, status: Optional[torch.Tensor] = None,
                    init: int = INIT_QUANTILE, algorithm: Optional[int] = None,
                    arrangement: Optional[torch.Tensor] = None, arrangement_use: int = ARRANGEMENT_NONE) -> None:
    """`cmpq_kmeans_quantize`; with `algorithm` or `arrangement` given, `cmpq_kmeans_quantize_job`."""
    d_in, d_out, ldw = _rows(W)
    buf = ws.get(workspace_bytes(OP_KMEANS, d_in, d_out))
    if algorithm is None and arrangement is None:
        _check(lib().cmpq_kmeans_quantize(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(bits), _ptr(out_idx),
                                          int(n_out), _ptr(elem_weight), int(iters), int(init), _ptr(centroids),
                                          _ptr(codes), _ptr(buf), buf.numel(), _ptr(status), _stream()),
               "cmpq_kmeans_quantize")
        return
    job = KmeansJob(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(bits), _ptr(out_idx), int(n_out),
                    _ptr(elem_weight), int(iters), int(init), _ptr(centroids), _ptr(codes), _ptr(status),
                    int(KMEANS_HISTOGRAM if algorithm is None else algorithm))
    job.arrangement, job.arrangement_use = _ptr(arrangement), int(arrangement_use)
    _check(lib().cmpq_kmeans_quantize_job(ctypes.byref(job), _ptr(buf), buf.numel(), _stream()),
           "cmpq_kmeans_quantize_job")


def arrangement_bytes(d_in: int, d_out: int) -> int:
    """Size of the buffer the two K-means runs of a layer can share (0: not available for this shape)."""
    return workspace_bytes(OP_KMEANS_ARRANGEMENT, d_in, d_out)


def kmeans_quantize_pack(W: torch.Tensor, bits: torch.Tensor, out_idx: Optional[torch.Tensor], n_out: int,
                         iters: int, centroids: torch.Tensor, codes: Optional[torch.Tensor],
                         bit_set: Sequence[int], counts: Sequence[int], packed: Sequence[Optional[torch.Tensor]],
                         chan_idx: Sequence[Optional[torch.Tensor]], lut: Sequence[Optional[torch.Tensor]],
                         sumsq: Optional[torch.Tensor], err_ch: torch.Tensor, err_total: torch.Tensor,
                         ws: Workspace, status: Optional[torch.Tensor] = None, init: int = INIT_QUANTILE,
                         algorithm: int = KMEANS_HISTOGRAM, elem_weight: Optional[torch.Tensor] = None,
                         arrangement: Optional[torch.Tensor] = None, arrangement_use: int = ARRANGEMENT_NONE) -> None:
    """`cmpq_kmeans_quantize_job` with the stored format and the error asked for: the K-means
    call followed by what `pack_with_error` leaves, written from the coding pass where the
    histogram kernel runs.  `codes` may be None there (the dense codes are then not written)."""
    d_in, d_out, ldw = _rows(W)
    n = len(bit_set)
    bs = (_i32 * n)(*bit_set)
    cn = (_i64 * n)(*counts)
    pk = (_vp * n)(*[_ptr(t) for t in packed])
    ci = (_vp * n)(*[_ptr(t) for t in chan_idx])
    lt = (_vp * n)(*[_ptr(t) for t in lut])
    buf = ws.get(workspace_bytes(OP_KMEANS, d_in, d_out))
    c = ctypes.cast
    job = KmeansJob(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(bits), _ptr(out_idx), int(n_out),
                    _ptr(elem_weight), int(iters), int(init), _ptr(centroids), _ptr(codes), _ptr(status),
                    int(algorithm), c(bs, _vp), n, c(cn, _vp), c(pk, _vp), c(ci, _vp), c(lt, _vp), _ptr(sumsq),
                    _ptr(err_ch), _ptr(err_total), _ptr(arrangement), int(arrangement_use))
    _check(lib().cmpq_kmeans_quantize_job(ctypes.byref(job), _ptr(buf), buf.numel(), _stream()),
           "cmpq_kmeans_quantize_job")


def pack(codes: torch.Tensor, bits: torch.Tensor, centroids: torch.Tensor, bit_set: Sequence[int],
         counts: Sequence[int], packed: Sequence[Optional[torch.Tensor]],
         chan_idx: Sequence[Optional[torch.Tensor]], lut: Sequence[Optional[torch.Tensor]], ws: Workspace) -> None:
    d_in, d_out = codes.shape
    n = len(bit_set)
    bs = (_i32 * n)(*bit_set)
    cn = (_i64 * n)(*counts)
    pk = (_vp * n)(*[_ptr(t) for t in packed])
    ci = (_vp * n)(*[_ptr(t) for t in chan_idx])
    lt = (_vp * n)(*[_ptr(t) for t in lut])
    buf = ws.get(workspace_bytes(OP_PACK, d_in, d_out))
    _check(lib().cmpq_pack(_ptr(codes), d_in, d_out, _ptr(bits), _ptr(centroids), bs, n, cn, pk, ci, lt,
                           _ptr(buf), buf.numel(), _stream()),
           "cmpq_pack")


def dequant_error(W: torch.Tensor, centroids: torch.Tensor, codes: torch.Tensor, bits: torch.Tensor,
                  out_idx: Optional[torch.Tensor], n_out: int, sumsq: Optional[torch.Tensor],
                  err_ch: torch.Tensor, err_total: torch.Tensor, ws: Workspace) -> None:
    d_in, d_out, ldw = _rows(W)
    buf = ws.get(workspace_bytes(OP_DEQUANT_ERROR, d_in, d_out))
    _check(lib().cmpq_dequant_error(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(centroids), _ptr(codes),
                                    _ptr(bits), _ptr(out_idx), int(n_out), _ptr(sumsq), _ptr(err_ch),
                                    _ptr(err_total), _ptr(buf), buf.numel(), _stream()),
           "cmpq_dequant_error")


def pack_with_error(W: torch.Tensor, codes: torch.Tensor, bits: torch.Tensor, centroids: torch.Tensor,
                    bit_set: Sequence[int], counts: Sequence[int], packed: Sequence[Optional[torch.Tensor]],
                    chan_idx: Sequence[Optional[torch.Tensor]], lut: Sequence[Optional[torch.Tensor]],
                    out_idx: Optional[torch.Tensor], n_out: int, sumsq: Optional[torch.Tensor],
                    err_ch: torch.Tensor, err_total: torch.Tensor, ws: Workspace) -> None:
    """`pack` and `dequant_error` in one pass over the codes."""
    d_in, d_out, ldw = _rows(W)
    if tuple(codes.shape) != (d_in, d_out):
        raise ValueError("codes must have the shape of W")
    n = len(bit_set)
    bs = (_i32 * n)(*bit_set)
    cn = (_i64 * n)(*counts)
    pk = (_vp * n)(*[_ptr(t) for t in packed])
    ci = (_vp * n)(*[_ptr(t) for t in chan_idx])
    lt = (_vp * n)(*[_ptr(t) for t in lut])
    buf = ws.get(workspace_bytes(OP_PACK_WITH_ERROR, d_in, d_out))
    _check(lib().cmpq_pack_with_error(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(codes), _ptr(bits),
                                      _ptr(centroids), bs, n, cn, pk, ci, lt, _ptr(out_idx), int(n_out),
                                      _ptr(sumsq), _ptr(err_ch), _ptr(err_total), _ptr(buf), buf.numel(),
                                      _stream()),
           "cmpq_pack_with_error")


def gather_channels(W: torch.Tensor, act_idx: torch.Tensor, W_act: torch.Tensor) -> None:
    """Fig. 4: the rows of O_act as deployed, ``W_act[j] = fp16(W[act_idx[j]])``."""
    d_in, d_out, ldw = _rows(W)
    k_act = int(act_idx.numel())
    if k_act:
        ka, do, ld_act = _rows(W_act)
        if (ka, do) != (k_act, d_out) or W_act.dtype != torch.float16:
            raise ValueError("W_act must be fp16 [k_act, d_out]")
    else:
        ld_act = d_out
    _check(lib().cmpq_gather_channels(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(act_idx), k_act,
                                      _ptr(W_act), ld_act, _stream()),
           "cmpq_gather_channels")


def outliers_by_column(out_idx: Optional[torch.Tensor], out_val: Optional[torch.Tensor], n_out: int,
                       d_in: int, d_out: int, centroids: torch.Tensor, codes: torch.Tensor,
                       colptr: torch.Tensor, row_idx: torch.Tensor, delta: torch.Tensor, ws: Workspace) -> None:
    buf = ws.get(workspace_bytes(OP_OUTLIERS_BY_COLUMN, d_in, d_out, n_out))
    _check(lib().cmpq_outliers_by_column(_ptr(out_idx), _ptr(out_val), int(n_out), d_in, d_out, _ptr(centroids),
                                         _ptr(codes), _ptr(colptr), _ptr(row_idx), _ptr(delta), _ptr(buf),
                                         buf.numel(), _stream()),
           "cmpq_outliers_by_column")


class LutMatvecCall:
    """``cmpq_lut_matvec`` for one deployed layer: everything that stays the same from token to
    token (pointer tables, counts, sizes) is marshalled once, so a call costs little more than
    the launch itself.  Holds the tensors it points into."""

    def __init__(self, d_in: int, d_out: int, bit_set: Sequence[int], counts: Sequence[int],
                 packed: Sequence[Optional[torch.Tensor]], chan_idx: Sequence[Optional[torch.Tensor]],
                 lut: Sequence[Optional[torch.Tensor]], act_idx: Optional[torch.Tensor],
                 W_act: Optional[torch.Tensor], colptr: Optional[torch.Tensor],
                 row_idx: Optional[torch.Tensor], delta: Optional[torch.Tensor]):
        n = len(bit_set)
        if row_idx is None or row_idx.numel() == 0:      # no entries of O_q: the library takes a null colptr
            colptr = row_idx = delta = None
        k_act = 0 if act_idx is None else int(act_idx.numel())
        ld_act = d_out if W_act is None or k_act == 0 else _rows(W_act)[2]
        self._keep = (list(packed), list(chan_idx), list(lut), act_idx, W_act, colptr, row_idx, delta)
        self.d_in, self.d_out = int(d_in), int(d_out)
        self._head = (self.d_out, (_i32 * n)(*bit_set), n, (_i64 * n)(*counts),
                      (_vp * n)(*[_ptr(t) for t in packed]), (_vp * n)(*[_ptr(t) for t in chan_idx]),
                      (_vp * n)(*[_ptr(t) for t in lut]), _ptr(act_idx), _ptr(W_act), k_act, ld_act,
                      _ptr(colptr), _ptr(row_idx), _ptr(delta))
        self._ws_bytes = {}
        self._fn = lib().cmpq_lut_matvec

    def __call__(self, X: torch.Tensor, Y: torch.Tensor, ws: Workspace) -> None:
        if X.dtype != torch.float16 or Y.dtype != torch.float32:
            raise ValueError("X must be fp16 and Y fp32")
        m, d_in, ldx = _rows(X)
        m2, do, ldy = _rows(Y)
        if (m2, do) != (m, self.d_out) or d_in != self.d_in:
            raise ValueError("X must be [m, d_in] and Y [m, d_out]")
        need = self._ws_bytes.get(m)
        if need is None:
            need = self._ws_bytes[m] = workspace_bytes(OP_LUT_MATVEC, d_in, do, m)
        buf = ws.get(need)
        rc = self._fn(_ptr(X), m, d_in, ldx, *self._head, _ptr(Y), ldy, buf.data_ptr(), buf.numel(), _stream())
        if rc:
            _check(rc, "cmpq_lut_matvec")


class LutMatvecGroupCall:
    """``cmpq_lut_matvec_group`` (``cmpq_lut_matvec_group_fp16acc`` with `fp16acc`) for a fixed set
    of deployed layers (`LutMatvecCall` objects): the array of layer descriptions is built once; a
    call fills in inputs and outputs."""

    def __init__(self, calls: Sequence[LutMatvecCall], fp16acc: bool = False):
        if not 1 <= len(calls) <= MAX_GROUP:
            raise ValueError(f"a group holds 1..{MAX_GROUP} layers")
        self._calls = list(calls)
        self._arr = (DeployedLayer * len(calls))()
        for L, c in zip(self._arr, calls):
            d_out, bs, n, cn, pk, ci, lt, act_idx, W_act, k_act, ld_act, colptr, row_idx, delta = c._head
            L.d_in, L.d_out, L.n_set, L.k_act, L.ld_act = c.d_in, d_out, n, k_act, ld_act
            L.bit_set, L.counts_host = ctypes.addressof(bs), ctypes.addressof(cn)
            L.packed, L.chan_idx, L.lut = ctypes.addressof(pk), ctypes.addressof(ci), ctypes.addressof(lt)
            L.act_idx, L.W_act, L.colptr, L.row_idx, L.delta = act_idx, W_act, colptr, row_idx, delta
        self._ws_bytes = {}
        self._fn = lib().cmpq_lut_matvec_group_fp16acc if fp16acc else lib().cmpq_lut_matvec_group

    def __call__(self, Xs: Sequence[torch.Tensor], Ys: Sequence[torch.Tensor], ws: Workspace) -> None:
        if len(Xs) != len(self._calls) or len(Ys) != len(self._calls):
            raise ValueError("one input and one output per layer")
        m = Xs[0].shape[0]
        for L, c, X, Y in zip(self._arr, self._calls, Xs, Ys):
            if X.dtype != torch.float16 or Y.dtype != torch.float32:
                raise ValueError("X must be fp16 and Y fp32")
            mx, d_in, ldx = _rows(X)
            my, do, ldy = _rows(Y)
            if (mx, d_in) != (m, c.d_in) or (my, do) != (m, c.d_out):
                raise ValueError("X must be [m, d_in] and Y [m, d_out], the same m for every layer")
            L.X, L.ldx, L.Y, L.ldy = _ptr(X), ldx, _ptr(Y), ldy
        need = self._ws_bytes.get(m)
        if need is None:
            need = self._ws_bytes[m] = sum(workspace_bytes(OP_LUT_MATVEC, c.d_in, c.d_out, m) for c in self._calls)
        buf = ws.get(need)
        rc = self._fn(self._arr, len(self._calls), m, buf.data_ptr(), buf.numel(), _stream())
        if rc:
            _check(rc, "cmpq_lut_matvec_group")


def lut_matvec(X: torch.Tensor, d_out: int, bit_set: Sequence[int], counts: Sequence[int],
               packed: Sequence[Optional[torch.Tensor]], chan_idx: Sequence[Optional[torch.Tensor]],
               lut: Sequence[Optional[torch.Tensor]], act_idx: Optional[torch.Tensor],
               W_act: Optional[torch.Tensor], colptr: Optional[torch.Tensor], row_idx: Optional[torch.Tensor],
               delta: Optional[torch.Tensor], Y: torch.Tensor, ws: Workspace) -> None:
    """Fig. 4: ``Y [m, d_out] fp32 = X [m, d_in] fp16 @ W_hat`` from the stored format."""
    LutMatvecCall(_rows(X)[1], d_out, bit_set, counts, packed, chan_idx, lut, act_idx, W_act, colptr,
                  row_idx, delta)(X, Y, ws)


def act_stats_norm(X: torch.Tensor, norm: int, acc: torch.Tensor, stat: Optional[torch.Tensor], accumulate: bool,
                   ws: Workspace, status: Optional[torch.Tensor] = None) -> None:
    """Tab. 13: the activation statistic under the l2 (squared), l1 or l-infinity norm."""
    n, d_in, ldx = _rows(X)
    buf = ws.get(workspace_bytes(OP_ACT_STATS, d_in, 0, n))
    _check(lib().cmpq_act_stats_norm(_ptr(X), _dtype(X), n, d_in, ldx, int(norm), _ptr(acc), _ptr(stat),
                                     int(bool(accumulate)), _ptr(buf), buf.numel(), _ptr(status), _stream()),
           "cmpq_act_stats_norm")


def rtn_quantize(W: torch.Tensor, bits: torch.Tensor, group: int, codes: torch.Tensor, scale: torch.Tensor,
                 zero: torch.Tensor, err_ch: Optional[torch.Tensor] = None,
                 status: Optional[torch.Tensor] = None) -> None:
    """App. A.2: round-to-nearest with the uniform quantizer, groups of `group` outputs per channel."""
    d_in, d_out, ldw = _rows(W)
    n_groups = -(-d_out // int(group)) if group > 0 else 0
    if tuple(codes.shape) != (d_in, d_out) or not codes.is_contiguous() or codes.dtype != torch.uint8:
        raise ValueError("codes must be a contiguous uint8 [d_in, d_out]")
    for t in (scale, zero):
        if tuple(t.shape) != (d_in, n_groups) or not t.is_contiguous() or t.dtype != torch.float32:
            raise ValueError("scale and zero must be contiguous float32 [d_in, ceil(d_out / group)]")
    if err_ch is not None and (err_ch.numel() != d_in or err_ch.dtype != torch.float64):
        raise ValueError("err_ch must be float64 [d_in]")
    _check(lib().cmpq_rtn_quantize(_ptr(W), _dtype(W), d_in, d_out, ldw, _ptr(bits), int(group), _ptr(codes),
                                   _ptr(scale), _ptr(zero), _ptr(err_ch), _ptr(status), _stream()),
           "cmpq_rtn_quantize")


def select_by_width(bits: torch.Tensor, bit_set: Sequence[int], centroids_by_width: Sequence[torch.Tensor],
                    codes_by_width: Sequence[torch.Tensor], centroids: torch.Tensor, codes: torch.Tensor) -> None:
    """The first K-means pass for the allocation `bits`, chosen row by row from one kept run per width."""
    d_in, d_out = codes.shape
    n = len(bit_set)
    for c, k in zip(centroids_by_width, codes_by_width):
        if tuple(c.shape) != (d_in, KMAX) or tuple(k.shape) != (d_in, d_out) or not c.is_contiguous() \
                or not k.is_contiguous() or c.dtype != torch.float32 or k.dtype != torch.uint8:
            raise ValueError("kept runs must be contiguous [d_in,16] fp32 levels and [d_in,d_out] uint8 codes")
    if not codes.is_contiguous() or not centroids.is_contiguous() or tuple(centroids.shape) != (d_in, KMAX):
        raise ValueError("outputs must be contiguous [d_in,16] and [d_in,d_out]")
    _check(lib().cmpq_select_by_width(_ptr(bits), d_in, d_out, (_i32 * n)(*bit_set), n,
                                      (_vp * n)(*[_ptr(t) for t in centroids_by_width]),
                                      (_vp * n)(*[_ptr(t) for t in codes_by_width]), _ptr(centroids), _ptr(codes),
                                      _stream()),
           "cmpq_select_by_width")


def lut4_quantize(centroids: torch.Tensor, bits: torch.Tensor, codes4: torch.Tensor, table: torch.Tensor,
                  centroids_q: torch.Tensor, ws: Workspace, mode: int = LUT4_CODEBOOK, iters: int = 20) -> None:
    """Sec. 5.1 / Tab. 7: the tables of a layer in 4 bits - codes into one 16-level table per layer
    (LUT4_CODEBOOK; `table` receives the levels) or on one uniform grid (LUT4_UNIFORM; `table[0:2]`
    receives minimum and step)."""
    d_in = centroids.shape[0]
    for t, dt in ((centroids, torch.float32), (centroids_q, torch.float32), (codes4, torch.uint8)):
        if tuple(t.shape) != (d_in, KMAX) or not t.is_contiguous() or t.dtype != dt:
            raise ValueError("tables are contiguous [d_in, 16]: fp32 levels, uint8 codes")
    if table.numel() != KMAX or table.dtype != torch.float32 or not table.is_contiguous():
        raise ValueError("table is fp32 [16]")
    buf = ws.get(workspace_bytes(OP_LUT4, d_in))
    _check(lib().cmpq_lut4_quantize(int(mode), _ptr(centroids), _ptr(bits), d_in, int(iters), _ptr(codes4),
                                    _ptr(table), _ptr(centroids_q), _ptr(buf), buf.numel(), _stream()),
           "cmpq_lut4_quantize")
