"""The C-ABI library loads, exports every symbol include/cmpq.h declares, and rejects bad
arguments on the host before anything is launched (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cmpq.h")


@pytest.fixture(scope="module")
def L():
    from paper_2410_13056_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2410_13056_amd import build
        build.build()
    return binding.lib()


def _declared():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(cmpq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared()
    assert {"cmpq_act_stats", "cmpq_allocate_bits", "cmpq_extract_outliers", "cmpq_kmeans_quantize",
            "cmpq_pack", "cmpq_dequant_error"} <= set(names)
    for n in names:
        assert getattr(L, n) is not None
    from paper_2410_13056_amd import binding
    assert set(binding.EXPORTS) == set(names)


def test_header_is_plain_c():
    src = os.path.join(ROOT, "tests", "_hdr_check.c")
    with open(src, "w") as f:
        f.write('#include "cmpq.h"\nint main(void){return CMPQ_OK;}\n')
    try:
        assert os.system(f"gcc -std=c99 -pedantic -Wall -Werror -I{ROOT}/include -fsyntax-only {src}") == 0
    finally:
        os.remove(src)


def test_counts_and_messages(L):
    from paper_2410_13056_amd import binding as B
    assert B.count_ppm(4500, 4096) == 18 and B.count_ppm(500, 4096 * 4096) == 8389
    assert B.count_ppm(10000, 28672 * 8192) == 2348810
    assert B.count_ppm(4500, 111) == 0 and B.count_ppm(4500, 112) == 1      # half rounds up
    for code in range(0, -7, -1):
        assert B.strerror(code) and "unknown cmpq" not in B.strerror(code)
    assert "unknown cmpq" in B.strerror(-99)
    for op in range(11):
        assert B.workspace_bytes(op, 4096, 4096, 1000) % 256 == 0
        assert B.workspace_bytes(op, 4096, 4096, 1000) >= 256
    assert B.workspace_bytes(99, 1, 1, 1) == 0


def test_host_side_argument_errors(L):
    from paper_2410_13056_amd import binding as B
    i32, i64 = ctypes.c_int32, ctypes.c_int64
    fake = ctypes.c_void_p(256)          # never dereferenced: every call below fails on the host
    bs = (i32 * 3)(2, 3, 4)
    # null pointers / bad enums
    assert L.cmpq_act_stats(fake, 0, 4, 8, 8, None, None, 0, fake, 1 << 20, None, None) == -1
    assert L.cmpq_act_stats(fake, 7, 4, 8, 8, fake, None, 0, fake, 1 << 20, None, None) == -1
    assert L.cmpq_act_stats(fake, 0, 4, 8, 4, fake, None, 0, fake, 1 << 20, None, None) == -2   # ldx < d_in
    assert L.cmpq_act_stats(fake, 0, 4, 8, 8, fake, None, 0, None, 0, None, None) == -5          # no workspace
    assert L.cmpq_act_stats(fake, 0, 4, 8, 8, fake, None, 0, ctypes.c_void_p(257), 1 << 20, None, None) == -5
    assert L.cmpq_transpose(None, 0, 4, 4, 4, fake, 4, None) == -1
    assert L.cmpq_transpose(fake, 0, 4, 4, 3, fake, 4, None) == -2
    # budget errors
    cnt = (i64 * 3)()
    assert L.cmpq_allocate_bits(fake, 16, None, 0, bs, 3, ctypes.c_double(4.5), fake, cnt, fake, 256, None) == -3
    assert L.cmpq_allocate_bits(fake, 16, None, 0, bs, 3, ctypes.c_double(1.5), fake, cnt, fake, 256, None) == -3
    assert L.cmpq_allocate_bits(fake, 16, None, 0, (i32 * 2)(2, 4), 2, ctypes.c_double(3.0), fake, cnt, fake, 256, None) == -3
    assert L.cmpq_allocate_bits(fake, 16, None, 0, (i32 * 2)(4, 5), 2, ctypes.c_double(4.0), fake, cnt, fake, 256, None) == -3
    assert L.cmpq_allocate_bits(fake, 16, None, 3, bs, 3, ctypes.c_double(3.0), fake, cnt, fake, 256, None) == -1
    # outliers
    assert L.cmpq_extract_outliers(0, 0, 0, fake, None, 0, 16, 0, 0, None, None, None, 17, fake, None, None, fake, 256, None) == -4
    assert L.cmpq_extract_outliers(1, 0, 0, None, fake, 0, 4, 4, 4, fake, fake, fake, 17, fake, None, None, fake, 1 << 20, None) == -4
    assert L.cmpq_extract_outliers(1, 0, 0, None, fake, 0, 4, 4, 4, None, fake, fake, 1, fake, None, None, fake, 1 << 20, None) == -1
    assert L.cmpq_extract_outliers(1, 0, 0, None, fake, 0, 4, 4, 4, fake, fake, fake, 1, fake, None, None, fake, 16, None) == -5
    assert L.cmpq_extract_outliers(5, 0, 0, None, fake, 0, 4, 4, 4, fake, fake, fake, 1, fake, None, None, fake, 1 << 20, None) == -1
    assert L.cmpq_extract_outliers(1, 0, 0, None, fake, 0, 1 << 20, 1 << 20, 1 << 20, fake, fake, fake, 1, fake, None, None, fake, 1 << 20, None) == -2
    assert L.cmpq_extract_outliers(1, 0, 2, None, fake, 0, 4, 4, 4, fake, fake, fake, 1, fake, None, None, fake, 1 << 20, None) == -1   # scope
    assert L.cmpq_extract_outliers(1, 0, 1, None, fake, 0, 4, 4, 4, fake, fake, fake, 5, fake, None, None, fake, 1 << 20, None) == -4   # per channel: k > d_out
    assert L.cmpq_extract_outliers(1, 0, 1, None, fake, 0, 4, 4, 4, fake, fake, fake, 0, None, None, None, None, 0, None) == 0          # nothing asked
    # k-means
    assert L.cmpq_kmeans_quantize(fake, 0, 4, 40000, 40000, fake, None, 0, None, 5, 0, fake, fake, fake, 256, None, None) == -2
    assert L.cmpq_kmeans_quantize(fake, 1, 4, 20000, 20000, fake, None, 0, None, 5, 0, fake, fake, fake, 256, None, None) == -2
    assert L.cmpq_kmeans_quantize(fake, 0, 4, 64, 64, fake, None, 0, None, -1, 0, fake, fake, fake, 256, None, None) == -1
    assert L.cmpq_kmeans_quantize(fake, 0, 4, 64, 64, fake, None, 0, None, 5, 3, fake, fake, fake, 256, None, None) == -1
    assert L.cmpq_kmeans_quantize(fake, 0, 4, 64, 64, fake, None, 2, None, 5, 0, fake, fake, fake, 256, None, None) == -1
    assert L.cmpq_kmeans_quantize(fake, 0, 4, 64, 32, fake, None, 0, None, 5, 0, fake, fake, fake, 256, None, None) == -2
    # pack / error
    ptrs = (ctypes.c_void_p * 3)(256, 256, 256)
    assert L.cmpq_pack(fake, 4, 64, fake, fake, bs, 3, None, ptrs, ptrs, ptrs, fake, 256, None) == -1
    assert L.cmpq_pack(fake, 4, 64, fake, fake, (i32 * 2)(3, 2), 2, cnt, ptrs, ptrs, ptrs, fake, 256, None) == -3
    cnt2 = (i64 * 3)(1, 1, 2)
    assert L.cmpq_pack(fake, 4, 64, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None) == -5
    assert L.cmpq_dequant_error(fake, 0, 4, 64, 64, fake, fake, fake, None, 0, None, None, fake, fake, 256, None) == -1
    assert L.cmpq_dequant_error(fake, 0, 4, 64, 8, fake, fake, fake, None, 0, None, fake, fake, fake, 256, None) == -2
    # both in one pass: the errors of either call
    pe = L.cmpq_pack_with_error
    assert pe(fake, 0, 4, 64, 64, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None, None, fake, fake, 4096, None) == -1
    assert pe(fake, 2, 4, 64, 64, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None, fake, fake, fake, 4096, None) == -1
    assert pe(fake, 0, 4, 64, 8, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None, fake, fake, fake, 4096, None) == -2
    assert pe(fake, 0, 4, 64, 64, fake, fake, fake, (i32 * 2)(3, 2), 2, cnt, ptrs, ptrs, ptrs, None, 0, None, fake, fake, fake, 4096, None) == -3
    assert pe(fake, 0, 4, 64, 64, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 3, None, fake, fake, fake, 4096, None) == -1
    assert pe(fake, 0, 4, 64, 64, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None, fake, fake, None, 0, None) == -5
    assert pe(fake, 0, 4, 64, 64, fake, fake, fake, bs, 3, cnt2, ptrs, ptrs, ptrs, None, 0, None, fake, fake, fake, 256, None) == -5
    # the deployed product
    assert L.cmpq_gather_channels(fake, 0, 8, 64, 64, None, 2, fake, 64, None) == -1
    assert L.cmpq_gather_channels(fake, 0, 8, 64, 64, fake, 9, fake, 64, None) == -1            # more rows than channels
    assert L.cmpq_gather_channels(fake, 0, 8, 64, 32, fake, 2, fake, 64, None) == -2
    assert L.cmpq_outliers_by_column(fake, fake, 4, 8, 64, fake, fake, None, fake, fake, fake, 1 << 20, None) == -1
    assert L.cmpq_outliers_by_column(fake, fake, 4, 8, 64, fake, fake, fake, fake, fake, None, 0, None) == -5
    assert L.cmpq_outliers_by_column(fake, fake, 4, 8, 1 << 20, fake, fake, fake, fake, fake, fake, 1 << 30, None) == -2
    assert L.cmpq_outliers_by_column(fake, fake, 600, 8, 64, fake, fake, fake, fake, fake, fake, 1 << 20, None) == -4
    one = (i64 * 3)(1, 1, 2)
    assert L.cmpq_lut_matvec(fake, 1, 8, 8, 64, bs, 3, one, ptrs, ptrs, ptrs, None, None, 0, 64, None, None, None,
                             None, 64, fake, 1 << 20, None) == -1                              # no output
    assert L.cmpq_lut_matvec(fake, 1, 8, 4, 64, bs, 3, one, ptrs, ptrs, ptrs, None, None, 0, 64, None, None, None,
                             fake, 64, fake, 1 << 20, None) == -2                              # ldx < d_in
    assert L.cmpq_lut_matvec(fake, 1, 8, 8, 64, bs, 3, (i64 * 3)(4, 4, 4), ptrs, ptrs, ptrs, None, None, 0, 64, None,
                             None, None, fake, 64, fake, 1 << 20, None) == -1                  # more rows than channels
    assert L.cmpq_lut_matvec(fake, 1, 8, 8, 64, (i32 * 1)(5), 1, (i64 * 1)(1), ptrs, ptrs, ptrs, None, None, 0, 64, None,
                             None, None, fake, 64, fake, 1 << 20, None) == -1                  # width outside 1..4
    assert L.cmpq_lut_matvec(fake, 1, 8, 8, 64, bs, 3, one, ptrs, ptrs, ptrs, None, None, 0, 64, fake, None, None,
                             fake, 64, fake, 1 << 20, None) == -1                              # colptr without entries
    assert L.cmpq_lut_matvec(fake, 1, 8, 8, 64, bs, 3, one, ptrs, ptrs, ptrs, None, None, 0, 64, None, None, None,
                             fake, 64, None, 0, None) == -5
    assert L.cmpq_lut_matvec(fake, 70000, 8, 8, 64, bs, 3, one, ptrs, ptrs, ptrs, None, None, 0, 64, None, None, None,
                             fake, 64, fake, 1 << 40, None) == -2                              # too many tokens
    assert L.cmpq_lut_matvec_group(None, 0, 1, None, 0, None) == 0                             # an empty group
    assert L.cmpq_lut_matvec_group(None, 2, 1, None, 0, None) == -1                            # layers missing
    assert L.cmpq_lut_matvec_group(fake, 9, 1, None, 0, None) == -1                            # more than CMPQ_MAX_GROUP
    # tables in 4 bits
    for mode in (0, 1):
        assert L.cmpq_lut4_quantize(mode, fake, fake, 4, 20, fake, None, fake, fake, 1 << 21, None) == -1   # no table
        assert L.cmpq_lut4_quantize(mode, None, fake, 4, 20, fake, fake, fake, fake, 1 << 21, None) == -1   # no centres
        assert L.cmpq_lut4_quantize(mode, fake, fake, -1, 20, fake, fake, fake, fake, 1 << 21, None) == -1
        assert L.cmpq_lut4_quantize(mode, fake, fake, 4, -1, fake, fake, fake, fake, 1 << 21, None) == -1   # rounds
    assert L.cmpq_lut4_quantize(2, fake, fake, 4, 20, fake, fake, fake, fake, 1 << 21, None) == -1          # mode
    assert L.cmpq_lut4_quantize(0, fake, fake, 4, 20, fake, fake, fake, fake, 4096, None) == -5             # workspace
    assert L.cmpq_lut4_quantize(0, fake, fake, 4, 20, fake, fake, fake, None, 0, None) == -5
    # the job form of the K-means call
    from paper_2410_13056_amd.binding import KmeansJob
    def job(**kw):
        j = KmeansJob(256, 0, 4, 64, 64, 256, None, 0, None, 5, 0, 256, 256, None, 0)   # no stored format asked for
        for k, v in kw.items():
            setattr(j, k, v)
        return ctypes.byref(j)
    assert L.cmpq_kmeans_quantize_job(None, fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(algorithm=2), fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(algorithm=1, iters=-1), fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(d_out=40000, ldw=40000), fake, 1 << 20, None) == -2
    assert L.cmpq_kmeans_quantize_job(job(), fake, 16, None) == -5
    assert L.cmpq_kmeans_quantize_job(job(d_in=0), None, 0, None) == 0
    # no codes: only where the histogram kernel runs (fp16, unit importance, rows of whole groups of 4)
    assert L.cmpq_kmeans_quantize_job(job(codes=None, dtype=1), fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(codes=None, d_out=66, ldw=66), fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(codes=None, elem_weight=256), fake, 1 << 20, None) == -1
    assert L.cmpq_kmeans_quantize_job(job(err_ch=256), fake, 1 << 20, None) == -1               # the stored format asked for in part
    bs3, one3 = (i32 * 3)(2, 3, 4), (i64 * 3)(1, 1, 1)
    nul3 = (ctypes.c_void_p * 3)(None, None, None)
    addr = lambda x: ctypes.cast(x, ctypes.c_void_p)
    assert L.cmpq_kmeans_quantize_job(job(bit_set=addr(bs3), n_set=3, counts_host=addr(one3), packed=addr(nul3),
                                          chan_idx=addr(nul3), lut=addr(nul3), err_ch=256, err_total=256),
                                      fake, 1 << 20, None) == -1                                # counts without arrays
    # measurement hook: unknown kernel; arming and disarming touch no GPU state
    assert L.cmpq_time_kernel(-1, fake, fake) == -1 and L.cmpq_time_kernel(5, fake, fake) == -1
    assert L.cmpq_time_kernel(2, fake, fake) == 0 and L.cmpq_time_kernel(2, None, None) == 0
    # the call without a workspace
    assert L.cmpq_act_stats_static(fake, 0, 8, 8, 8, None, None, 0, None, None) == -1            # no accumulator
    assert L.cmpq_act_stats_static(fake, 3, 8, 8, 8, fake, None, 0, None, None) == -1            # dtype
    assert L.cmpq_act_stats_static(fake, 0, 8, 8, 4, fake, None, 0, None, None) == -2            # ldx < d_in
    assert L.cmpq_act_stats_static(fake, 0, 8, 262145, 262145, fake, None, 0, None, None) == -2  # beyond the fixed array
    assert L.cmpq_act_stats_static(None, 0, 0, 0, 0, fake, None, 0, None, None) == 0             # nothing to do
    # the uniform quantizer
    assert L.cmpq_rtn_quantize(fake, 0, 4, 64, 64, fake, 96, fake, fake, fake, None, None, None) == -1    # group no power of two
    assert L.cmpq_rtn_quantize(fake, 0, 4, 64, 64, fake, 4, fake, fake, fake, None, None, None) == -1     # group below 8
    assert L.cmpq_rtn_quantize(fake, 0, 4, 64, 64, fake, 1024, fake, fake, fake, None, None, None) == -1  # group above 512
    assert L.cmpq_rtn_quantize(fake, 2, 4, 64, 64, fake, 128, fake, fake, fake, None, None, None) == -1   # dtype
    assert L.cmpq_rtn_quantize(fake, 0, 4, 64, 64, fake, 128, None, fake, fake, None, None, None) == -1   # no codes
    assert L.cmpq_rtn_quantize(fake, 0, 4, 64, 32, fake, 128, fake, fake, fake, None, None, None) == -2   # ldw < d_out
    assert L.cmpq_rtn_quantize(None, 0, 0, 64, 64, None, 128, None, None, None, None, None, None) == 0    # nothing to do
    # retargeting
    two = (ctypes.c_void_p * 2)(256, 256)
    assert L.cmpq_select_by_width(fake, 4, 64, (i32 * 2)(2, 2), 2, two, two, fake, fake, None) == -1      # width twice
    assert L.cmpq_select_by_width(fake, 4, 64, (i32 * 2)(2, 7), 2, two, two, fake, fake, None) == -1      # width outside 1..4
    assert L.cmpq_select_by_width(fake, 4, 64, (i32 * 2)(2, 3), 2, two, (ctypes.c_void_p * 2)(256, None), fake, fake,
                                  None) == -1                                                             # a run missing
    assert L.cmpq_select_by_width(fake, 4, 64, (i32 * 2)(2, 3), 2, two, two, None, fake, None) == -1      # no output
    assert L.cmpq_select_by_width(None, 0, 64, (i32 * 2)(2, 3), 2, two, two, None, None, None) == 0       # nothing to do
    # the clock probe
    khz = ctypes.c_int(0)
    L.cmpq_shader_clock_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert L.cmpq_shader_clock_probe(100, 4, None, ctypes.byref(khz), None) == -1                         # no output
    assert L.cmpq_shader_clock_probe(0, 4, fake, ctypes.byref(khz), None) == -1                           # no rounds
    assert L.cmpq_shader_clock_probe(100, 0, fake, ctypes.byref(khz), None) == -1                         # no workgroups
    assert L.cmpq_shader_clock_probe(100, 70000, fake, ctypes.byref(khz), None) == -1                     # too many


def test_product_package_does_not_reach_the_oracle():
    """The HIP path must stand alone: no file of the package mentions the oracle."""
    pkg = os.path.join(ROOT, "paper_2410_13056_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "orc_" not in text, f
    src = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "cmpq_oracle.c")).read()
    assert "paper_2410_13056_amd" not in src and "cmpq.h" not in src
