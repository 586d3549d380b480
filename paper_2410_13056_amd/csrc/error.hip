// cmpq_dequant_error: rebuilds W_hat = W_q + O (Sec. 3.2.2 of arXiv 2410.13056) on the
// fly and measures the output error of App. B.3, Delta Y = X (W - W_hat), channel by
// channel: err_ch[i] = sum_o (W[i,o] - W_hat[i,o])^2, weighted by the activation
// statistic for the layer total.
//
// HBM bound: 2 (or 4) bytes of W and 1 byte of code per weight.  One workgroup per
// channel; the slice of the outlier list that falls in the channel is expanded into
// an LDS bitmap first, so the main loop is a plain streaming pass.  Sums are fp64
// per lane, reduced in a fixed order.
#include "common.h"

namespace {

constexpr int kT = 256;

// Eight consecutive weights of one channel and their codes, by vector loads when the
// addresses allow it.  Returns the mask of entries that exist (o0 + j < d_out).
template <typename TW>
__device__ __forceinline__ uint32_t load8(const TW *__restrict__ wrow, const uint8_t *__restrict__ crow,
                                          int64_t o0, int64_t d_out, bool vec_ok, float (&w)[8],
                                          uint32_t (&c)[8]) {
    if (vec_ok && o0 + 8 <= d_out) {
        if constexpr (sizeof(TW) == 2) {
            const uint4 raw = load16_stream(wrow + o0);
            const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 t = __half22float2(h[j]);
                w[2 * j] = t.x;
                w[2 * j + 1] = t.y;
            }
        } else {
            const float4 r0 = *reinterpret_cast<const float4 *>(wrow + o0);
            const float4 r1 = *reinterpret_cast<const float4 *>(wrow + o0 + 4);
            w[0] = r0.x, w[1] = r0.y, w[2] = r0.z, w[3] = r0.w;
            w[4] = r1.x, w[5] = r1.y, w[6] = r1.z, w[7] = r1.w;
        }
        const uint2 cr = *reinterpret_cast<const uint2 *>(crow + o0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c[j] = (cr.x >> (8 * j)) & 0xffu;
            c[4 + j] = (cr.y >> (8 * j)) & 0xffu;
        }
        return 0xffu;
    }
    uint32_t valid = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        w[j] = 0.f;
        c[j] = 0;
        if (o0 + j < d_out) {
            valid |= 1u << j;
            w[j] = load_as_f32<TW>(wrow, o0 + j);
            c[j] = crow[o0 + j];
        }
    }
    return valid;
}

template <typename TW>
__global__ __launch_bounds__(kT) void dequant_error_kernel(
    const TW *__restrict__ W, int64_t d_out, int64_t ldw, const float *__restrict__ centroids,
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ bits,
    const int32_t *__restrict__ out_idx, const int32_t *__restrict__ slices,
    double *__restrict__ err_ch, int vec_ok) {
    extern __shared__ uint32_t restored[];  // one bit per entry of the channel
    __shared__ float lut[CMPQ_KMAX];
    __shared__ double red[kT / CMPQ_WAVE];
    __shared__ int seg[2];
    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    const int b = bits[i];
    const bool whole = b < 1 || b > 4;  // a channel of O_act: every entry restored
    const int words = (int)((d_out + 31) / 32);
    for (int w = tid; w < words; w += kT) restored[w] = 0;
    if (tid < CMPQ_KMAX) lut[tid] = centroids[i * CMPQ_KMAX + tid];
    if (tid == 0) {
        seg[0] = slices ? slices[i] : 0;
        seg[1] = slices ? slices[i + 1] : 0;
    }
    __syncthreads();
    for (int e = seg[0] + tid; e < seg[1]; e += kT) {
        const int o = (int)(out_idx[e] - i * d_out);
        atomicOr(&restored[o >> 5], 1u << (o & 31));
    }
    __syncthreads();
    const TW *wrow = W + i * ldw;
    const uint8_t *crow = codes + i * d_out;
    double s = 0.0;
    // a lane takes 8 consecutive weights per step, two steps in flight
    for (int64_t o0 = (int64_t)tid * 8; o0 < d_out; o0 += 2 * kT * 8) {
        float w[2][8];
        uint32_t c[2][8], valid[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t o = o0 + (int64_t)u * kT * 8;
            valid[u] = o < d_out ? load8<TW>(wrow, crow, o, d_out, vec_ok, w[u], c[u]) : 0u;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t o = o0 + (int64_t)u * kT * 8;
            if (!valid[u]) continue;
            // o is a multiple of 8: the 8 flags sit in one byte of the bitmap
            const uint32_t back = whole ? 0xffu : (restored[o >> 5] >> (o & 31)) & 0xffu;
            // the eight levels first, without conditions, so that the look-ups go out together
            float level[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) level[j] = lut[c[u][j] & 15u];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // a restored entry is the weight rounded to FP16 (itself for FP16 input); an entry
                // past the end of the channel counts as exact
                float what = level[j];
                if ((back >> j) & 1u)
                    what = sizeof(TW) == 2 ? w[u][j] : __half2float(__float2half_rn(w[u][j]));
                if (!((valid[u] >> j) & 1u)) what = w[u][j];
                const double e = (double)w[u][j] - (double)what;
                s = fma(e, e, s);
            }
        }
    }
    s = wave_sum_f64(s);
    if ((tid & 63) == 0) red[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int w = 0; w < kT / CMPQ_WAVE; ++w) t += red[w];
        err_ch[i] = t;
    }
}

// totals[0] = sum_i sumsq[i]*err_ch[i], totals[1] = sum_i err_ch[i]; one workgroup,
// fixed order.
__global__ __launch_bounds__(1024) void error_totals_kernel(const double *__restrict__ err_ch,
                                                            const float *__restrict__ sumsq,
                                                            int64_t d_in,
                                                            double *__restrict__ totals) {
    __shared__ double red[2][16];
    double tw = 0.0, tu = 0.0;
    for (int64_t i = threadIdx.x; i < d_in; i += blockDim.x) {
        const double e = err_ch[i];
        tw = fma(sumsq ? (double)sumsq[i] : 1.0, e, tw);
        tu += e;
    }
    tw = wave_sum_f64(tw);
    tu = wave_sum_f64(tu);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = tw;
        red[1][threadIdx.x >> 6] = tu;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, c = 0.0;
        for (int w = 0; w < 16; ++w) {
            a += red[0][w];
            c += red[1][w];
        }
        totals[0] = a;
        totals[1] = c;
    }
}

}  // namespace

int launch_dequant_error_rows(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                              const float *centroids, const uint8_t *codes, const uint8_t *bits,
                              const int32_t *out_idx, const int32_t *slices, double *err_ch, hipStream_t s) {
    if (d_in <= 0) return CMPQ_OK;
    const size_t lds = (size_t)cdiv(d_out > 0 ? d_out : 1, 32) * 4;
    const int esz = dtype == CMPQ_F16 ? 2 : 4;
    const int vec_ok = reinterpret_cast<uintptr_t>(W) % 16 == 0 && (ldw * esz) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(codes) % 8 == 0 && d_out % 8 == 0;
    if (dtype == CMPQ_F16)
        dequant_error_kernel<__half><<<(unsigned)d_in, kT, lds, s>>>(
            static_cast<const __half *>(W), d_out, ldw, centroids, codes, bits, out_idx, slices, err_ch, vec_ok);
    else
        dequant_error_kernel<float><<<(unsigned)d_in, kT, lds, s>>>(
            static_cast<const float *>(W), d_out, ldw, centroids, codes, bits, out_idx, slices, err_ch, vec_ok);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

int launch_error_totals(const double *err_ch, const float *sumsq, int64_t d_in, double *totals, hipStream_t s) {
    error_totals_kernel<<<1, 1024, 0, s>>>(err_ch, sumsq, d_in, totals);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

size_t cmpq_ws_dequant_error(int64_t d_in) {
    return align_up((size_t)(d_in + 1) * sizeof(int32_t), 256);  // slice offsets of out_idx
}

extern "C" int cmpq_dequant_error(const void *W, int dtype, int64_t d_in, int64_t d_out,
                                  int64_t ldw, const float *centroids, const uint8_t *codes,
                                  const uint8_t *bits, const int32_t *out_idx, int64_t n_out,
                                  const float *sumsq, double *err_ch, double *err_total, void *ws,
                                  size_t ws_bytes, void *stream) {
    if (d_in < 0 || d_out < 0 || n_out < 0) return CMPQ_EINVAL;
    if (dtype != CMPQ_F16 && dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (!bits || !centroids || !err_ch || !err_total || (n_out > 0 && !out_idx)) return CMPQ_EINVAL;
    if (d_in > 0 && d_out > 0 && (!W || !codes)) return CMPQ_EINVAL;
    if (ldw < d_out) return CMPQ_ESHAPE;
    if (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;
    if (d_out > 1 << 20) return CMPQ_ESHAPE;  // the per-channel bitmap lives in LDS
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int32_t *slices = nullptr;
    if (d_in > 0 && n_out > 0) {
        if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_dequant_error(d_in))
            return CMPQ_EWORKSPACE;
        const int rc = launch_segment_offsets(out_idx, n_out, d_in, d_out, static_cast<int32_t *>(ws), s);
        if (rc != CMPQ_OK) return rc;
        slices = static_cast<const int32_t *>(ws);
    }
    if (const int rc = launch_dequant_error_rows(W, dtype, d_in, d_out, ldw, centroids, codes, bits, out_idx,
                                                 slices, err_ch, s))
        return rc;
    return launch_error_totals(err_ch, sumsq, d_in, err_total, s);
}
