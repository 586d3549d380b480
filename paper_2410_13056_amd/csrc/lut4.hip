// cmpq_lut4_quantize: the look-up tables of a layer held in 4 bits (Sec. 5.1 / Tab. 7 of
// arXiv 2410.13056: the variant whose overhead is (1*4 + 8*4)/4096 bits per weight).
//
// The paper does not say how the centres are quantized and its figure leaves no room for a
// scale per channel.  Reading: one uniform 16-level grid per layer - the quantizer of Sec. 3
// with N = 4 over all centres at once.  Two small kernels: the range of all centres (one
// workgroup; minimum and maximum do not depend on the order), then code and rebuilt level
// of every table entry.  The code is decided in fp32 with one IEEE division, the rebuilt
// level is min + code * Delta formed exactly (fp64) and rounded once to fp32.
#include "common.h"

namespace {

constexpr int kT = 1024;

// range[0] = min, range[1] = (max - min) / 15 over the first 2^bits levels of every channel
// with bits in 1..4; 0, 0 when there is none.
__global__ __launch_bounds__(kT) void lut4_range_kernel(const float *__restrict__ centroids,
                                                        const uint8_t *__restrict__ bits, int64_t d_in,
                                                        float *__restrict__ range) {
    __shared__ float red_lo[kT / CMPQ_WAVE], red_hi[kT / CMPQ_WAVE];
    float lo = INFINITY, hi = -INFINITY;
    for (int64_t e = threadIdx.x; e < d_in * CMPQ_KMAX; e += kT) {
        const int64_t i = e / CMPQ_KMAX;
        const int j = (int)(e % CMPQ_KMAX), b = bits[i];
        if (b >= 1 && b <= 4 && j < (1 << b)) {
            const float c = centroids[e];
            lo = fminf(lo, c);
            hi = fmaxf(hi, c);
        }
    }
    for (int off = 1; off < CMPQ_WAVE; off <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    if ((threadIdx.x & (CMPQ_WAVE - 1)) == 0) {
        red_lo[threadIdx.x / CMPQ_WAVE] = lo;
        red_hi[threadIdx.x / CMPQ_WAVE] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kT / CMPQ_WAVE; ++w) {
            lo = fminf(lo, red_lo[w]);
            hi = fmaxf(hi, red_hi[w]);
        }
        const bool any = lo <= hi;
        range[0] = any ? lo : 0.f;
        range[1] = any ? (hi - lo) / 15.f : 0.f;
    }
}

__global__ __launch_bounds__(256) void lut4_code_kernel(const float *__restrict__ centroids,
                                                        const uint8_t *__restrict__ bits, int64_t d_in,
                                                        const float *__restrict__ range,
                                                        uint8_t *__restrict__ codes4,
                                                        float *__restrict__ centroids_q) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d_in * CMPQ_KMAX) return;
    const int64_t i = e / CMPQ_KMAX;
    const int j = (int)(e % CMPQ_KMAX), b = bits[i];
    uint8_t code = 0;
    float cq = INFINITY;
    if (b >= 1 && b <= 4 && j < (1 << b)) {
        const float lo = range[0], delta = range[1];
        float q = 0.f;
        if (delta != 0.f) q = fminf(fmaxf(rintf((centroids[e] - lo) / delta), 0.f), 15.f);
        code = (uint8_t)q;
        cq = (float)fma((double)q, (double)delta, (double)lo);
    }
    codes4[e] = code;
    centroids_q[e] = cq;
}

}  // namespace

extern "C" int cmpq_lut4_quantize(const float *centroids, const uint8_t *bits, int64_t d_in, uint8_t *codes4,
                                  float *range, float *centroids_q, void *stream) {
    if (d_in < 0 || !range) return CMPQ_EINVAL;
    if (d_in > 0 && (!centroids || !bits || !codes4 || !centroids_q)) return CMPQ_EINVAL;
    if (d_in > ((int64_t)1 << 27)) return CMPQ_ESHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    lut4_range_kernel<<<1, kT, 0, s>>>(centroids, bits, d_in, range);
    if (d_in > 0)
        lut4_code_kernel<<<(unsigned)cdiv(d_in * CMPQ_KMAX, 256), 256, 0, s>>>(centroids, bits, d_in, range, codes4,
                                                                                centroids_q);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
