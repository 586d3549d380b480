// Where each channel's slice of an ascending list of linear indices i*d_out+o begins:
// shared by the kernels that take the entries of O_q (Sec. 3.2.2 of arXiv 2410.13056) as
// a sorted list.  One binary search per channel, done once, instead of one per workgroup.
#include "common.h"

namespace {

__global__ __launch_bounds__(256) void segment_offsets_kernel(const int32_t *__restrict__ idx, int64_t n,
                                                              int64_t d_in, int64_t d_out,
                                                              int32_t *__restrict__ seg) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > d_in) return;
    const int64_t first = i * d_out;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)idx[mid] < first) lo = mid + 1; else hi = mid;
    }
    seg[i] = (int32_t)lo;
}

}  // namespace

int launch_segment_offsets(const int32_t *idx, int64_t n, int64_t d_in, int64_t d_out, int32_t *seg,
                           hipStream_t s) {
    segment_offsets_kernel<<<(unsigned)cdiv(d_in + 1, 256), 256, 0, s>>>(idx, n, d_in, d_out, seg);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
