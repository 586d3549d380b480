// cmpq_select_by_width: the first K-means pass of a layer for a new bit budget, taken from
// results kept per width.
//
// The preliminary quantization W'_q of Sec. 3.2.2 of arXiv 2410.13056 treats every input
// channel on its own: levels and codes of channel i depend on W[i,:] and on its width only,
// not on the widths Algorithm 1 gives the other channels.  So after one K-means run per
// width of the bit set over all channels, the pass for any budget is a row-wise choice
// among those runs - the paper's "limitation" paragraph names repeated retargeting to many
// budgets as the cost this removes.
//
// HBM bound: one byte read and one written per weight.  One workgroup per channel.
#include "common.h"

namespace {

constexpr int kT = 256;
constexpr int kMaxSet = 4;

struct SelArgs {
    const float *cent[kMaxSet];
    const uint8_t *codes[kMaxSet];
    int32_t width[kMaxSet];
    int n_set;
};

__global__ __launch_bounds__(kT) void select_by_width_kernel(const uint8_t *__restrict__ bits, int64_t d_out,
                                                              SelArgs a, float *__restrict__ centroids,
                                                              uint8_t *__restrict__ codes, int vec_ok) {
    const int64_t i = blockIdx.x;
    const int b = bits[i];
    int j = -1;
    for (int t = 0; t < a.n_set; ++t)
        if (a.width[t] == b) j = t;
    if (threadIdx.x < CMPQ_KMAX)
        centroids[i * CMPQ_KMAX + threadIdx.x] = j >= 0 ? a.cent[j][i * CMPQ_KMAX + threadIdx.x] : INFINITY;
    uint8_t *dst = codes + i * d_out;
    if (j < 0) {  // a channel of O_act, or a width no run was kept for: no codes
        if (vec_ok)
            for (int64_t o = (int64_t)threadIdx.x * 16; o < d_out; o += kT * 16)
                *reinterpret_cast<uint4 *>(dst + o) = make_uint4(0u, 0u, 0u, 0u);
        else
            for (int64_t o = threadIdx.x; o < d_out; o += kT) dst[o] = 0;
        return;
    }
    const uint8_t *src = a.codes[j] + i * d_out;
    if (vec_ok)
        for (int64_t o = (int64_t)threadIdx.x * 16; o < d_out; o += kT * 16)
            *reinterpret_cast<uint4 *>(dst + o) = *reinterpret_cast<const uint4 *>(src + o);
    else
        for (int64_t o = threadIdx.x; o < d_out; o += kT) dst[o] = src[o];
}

}  // namespace

extern "C" int cmpq_select_by_width(const uint8_t *bits, int64_t d_in, int64_t d_out, const int32_t *bit_set,
                                    int n_set, const float *const *centroids_by_width,
                                    const uint8_t *const *codes_by_width, float *centroids, uint8_t *codes,
                                    void *stream) {
    if (d_in < 0 || d_out < 0 || n_set < 1 || n_set > kMaxSet) return CMPQ_EINVAL;
    if (!bit_set || !centroids_by_width || !codes_by_width) return CMPQ_EINVAL;
    SelArgs a;
    a.n_set = n_set;
    bool aligned = reinterpret_cast<uintptr_t>(codes) % 16 == 0 && d_out % 16 == 0;
    for (int j = 0; j < kMaxSet; ++j) {
        a.cent[j] = nullptr;
        a.codes[j] = nullptr;
        a.width[j] = -1;
    }
    for (int j = 0; j < n_set; ++j) {
        if (bit_set[j] < 1 || bit_set[j] > 4) return CMPQ_EINVAL;
        for (int t = 0; t < j; ++t)
            if (bit_set[t] == bit_set[j]) return CMPQ_EINVAL;
        if (!centroids_by_width[j] || !codes_by_width[j]) return CMPQ_EINVAL;
        a.cent[j] = centroids_by_width[j];
        a.codes[j] = codes_by_width[j];
        a.width[j] = bit_set[j];
        aligned = aligned && reinterpret_cast<uintptr_t>(codes_by_width[j]) % 16 == 0;
    }
    if (d_in == 0) return CMPQ_OK;
    if (!bits || !centroids || (d_out > 0 && !codes)) return CMPQ_EINVAL;
    if (d_in > 0x7fffffff) return CMPQ_ESHAPE;
    select_by_width_kernel<<<(unsigned)d_in, kT, 0, static_cast<hipStream_t>(stream)>>>(bits, d_out, a, centroids,
                                                                                       codes, aligned ? 1 : 0);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
