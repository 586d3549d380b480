// cmpq_rtn_quantize: CMPQ with the uniform quantizer of Sec. 3 of arXiv 2410.13056 in place of
// K-means (App. A.2, Tab. 10): round-to-nearest on the grid min + k * Delta,
// Delta = (max - min) / (2^N - 1), per group of consecutive outputs of an input channel, with
// the channel's width N from Algorithm 1.
//
// HBM bound: 2 (or 4) bytes of W read, 1 byte of code written per weight, two floats per
// group.  One workgroup per channel; a lane takes 8 consecutive weights per step (one 16-byte
// load, one 8-byte store), so a group of g weights is g / 8 neighbouring lanes and its range
// is found with a butterfly of lane exchanges - min and max do not depend on the order.  The
// code is decided in fp32 from the correctly rounded quotient (w - min) / Delta; the squared
// error is summed in fp64 per lane and reduced in a fixed order.
#include "common.h"

namespace {

constexpr int kT = 256;
constexpr int kPer = 8;  // weights per lane and step

// Eight consecutive weights of one channel, by a vector load when the addresses allow it.
// Returns the mask of entries that exist (o0 + j < d_out).
template <typename TW>
__device__ __forceinline__ uint32_t load8w(const TW *__restrict__ wrow, int64_t o0, int64_t d_out, bool vec_ok,
                                           float (&w)[kPer]) {
    if (o0 >= d_out) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) w[j] = 0.f;
        return 0u;
    }
    if (vec_ok && o0 + kPer <= d_out) {
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
        return 0xffu;
    }
    uint32_t valid = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        w[j] = 0.f;
        if (o0 + j < d_out) {
            valid |= 1u << j;
            w[j] = load_as_f32<TW>(wrow, o0 + j);
        }
    }
    return valid;
}

// lanes_per_group: a power of two in 1..64 (group / 8).  VEC: rows are read and written in
// whole 8-weight pieces (aligned, d_out a multiple of 8), so a lane's piece exists entirely
// or not at all and no entry needs a test of its own.
template <typename TW, bool WITH_ERR, bool VEC>
__global__ __launch_bounds__(kT) void rtn_kernel(const TW *__restrict__ W, int64_t d_out, int64_t ldw,
                                                  const uint8_t *__restrict__ bits, int lanes_per_group,
                                                  int64_t n_groups, uint8_t *__restrict__ codes,
                                                  float *__restrict__ scale, float *__restrict__ zero,
                                                  double *__restrict__ err_ch, int32_t *__restrict__ status) {
    constexpr int vec_ok = VEC ? 1 : 0;
    __shared__ double red[kT / CMPQ_WAVE];
    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    const int N = bits[i];
    const bool kept = N < 1 || N > 4;  // a channel of O_act: stays FP16, no codes
    const float top = (float)((1 << (kept ? 1 : N)) - 1);
    const TW *wrow = W + i * ldw;
    uint8_t *crow = codes + i * d_out;
    double s = 0.0;
    bool bad = false;
    for (int64_t base = 0; base < d_out; base += (int64_t)kT * kPer) {
        const int64_t o0 = base + (int64_t)tid * kPer;
        float w[kPer];
        const uint32_t valid = load8w<TW>(wrow, o0, d_out, vec_ok, w);
        auto has = [&](int j) -> bool { return VEC ? valid != 0u : ((valid >> j) & 1u) != 0u; };
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (has(j)) {
                lo = fminf(lo, w[j]);
                hi = fmaxf(hi, w[j]);
                bad |= !isfinite(w[j]);
            }
        // range of the group: every lane of the wavefront takes part, also those past the end
        for (int off = 1; off < lanes_per_group; off <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, off));
            hi = fmaxf(hi, __shfl_xor(hi, off));
        }
        if (!valid) continue;
        float r[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) r[j] = 0.f;
        if (kept) {
            if (WITH_ERR) {
#pragma unroll
                for (int j = 0; j < kPer; ++j)
                    if (has(j)) {
                        const double d = (double)w[j] - (double)__half2float(__float2half_rn(w[j]));
                        s = fma(d, d, s);
                    }
            }
            lo = 0.f;
            hi = 0.f;
        }
        const float delta = (hi - lo) / top;
        if ((tid & (lanes_per_group - 1)) == 0) {
            const int64_t g = o0 / ((int64_t)lanes_per_group * kPer);
            scale[i * n_groups + g] = delta;
            zero[i * n_groups + g] = lo;
        }
        if (!kept && delta != 0.f) {
            // The correctly rounded quotient (w - lo) / delta.  With delta well inside the
            // normal range this is the usual division sequence - reciprocal estimate, one
            // Newton step, then two residual corrections of the quotient - with the part that
            // only depends on delta done once per step instead of once per weight; no
            // intermediate can leave the normal range for a quotient that rounds to a code
            // above 0.  Other steps (tiny or huge delta) divide in the ordinary way.
            float quo[kPer];
            if (delta >= 0x1p-60f && delta <= 0x1p60f) {
                const float y0 = __builtin_amdgcn_rcpf(delta);
                const float y = fmaf(fmaf(-delta, y0, 1.f), y0, y0);
#pragma unroll
                for (int j = 0; j < kPer; ++j) {
                    const float a = w[j] - lo;
                    const float m = a * y;
                    const float q1 = fmaf(fmaf(-delta, m, a), y, m);
                    quo[j] = fmaf(fmaf(-delta, q1, a), y, q1);
                }
            } else {
#pragma unroll
                for (int j = 0; j < kPer; ++j) quo[j] = (w[j] - lo) / delta;
            }
#pragma unroll
            for (int j = 0; j < kPer; ++j)
                if (has(j)) r[j] = fminf(fmaxf(rintf(quo[j]), 0.f), top);
        }
        if (WITH_ERR && !kept) {
#pragma unroll
            for (int j = 0; j < kPer; ++j)
                if (has(j)) {
                    const double d = (double)w[j] - fma((double)r[j], (double)delta, (double)lo);
                    s = fma(d, d, s);
                }
        }
        // r holds whole numbers in 0..15: the conversion packs them as bytes
        uint2 out = make_uint2(0u, 0u);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            out.x = __builtin_amdgcn_cvt_pk_u8_f32(r[j], j, out.x);
            out.y = __builtin_amdgcn_cvt_pk_u8_f32(r[4 + j], j, out.y);
        }
        if (VEC) {
            *reinterpret_cast<uint2 *>(crow + o0) = out;
        } else {
#pragma unroll
            for (int j = 0; j < kPer; ++j)
                if ((valid >> j) & 1u) crow[o0 + j] = (uint8_t)(((j < 4 ? out.x : out.y) >> (8 * (j & 3))) & 0xffu);
        }
    }
    if (status && __syncthreads_or(bad) && tid == 0) atomicOr(status, CMPQ_STATUS_NONFINITE);
    if (WITH_ERR) {
        s = wave_sum_f64(s);
        if ((tid & 63) == 0) red[tid >> 6] = s;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int wv = 0; wv < kT / CMPQ_WAVE; ++wv) t += red[wv];
            err_ch[i] = t;
        }
    }
}

}  // namespace

extern "C" int cmpq_rtn_quantize(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                                 const uint8_t *bits, int64_t group, uint8_t *codes, float *scale,
                                 float *zero, double *err_ch, int32_t *status, void *stream) {
    if (d_in < 0 || d_out < 0 || (dtype != CMPQ_F16 && dtype != CMPQ_F32)) return CMPQ_EINVAL;
    if (group < 8 || group > 512 || (group & (group - 1)) != 0) return CMPQ_EINVAL;
    if (d_in == 0 || d_out == 0) return CMPQ_OK;
    if (!W || !bits || !codes || !scale || !zero) return CMPQ_EINVAL;
    if (ldw < d_out) return CMPQ_ESHAPE;
    if (d_in > 0x7fffffff) return CMPQ_ESHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int esz = dtype == CMPQ_F16 ? 2 : 4;
    const int vec_ok = reinterpret_cast<uintptr_t>(W) % 16 == 0 && (ldw * esz) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(codes) % 8 == 0 && d_out % 8 == 0;
    const int lpg = (int)(group / kPer);
    const int64_t n_groups = cdiv(d_out, group);
    const unsigned grid = (unsigned)d_in;
#define CMPQ_RTN_LAUNCH(TW, ERR, VEC)                                                                          \
    rtn_kernel<TW, ERR, VEC><<<grid, kT, 0, s>>>(static_cast<const TW *>(W), d_out, ldw, bits, lpg, n_groups, \
                                                 codes, scale, zero, err_ch, status)
#define CMPQ_RTN_PICK(TW)                                        \
    do {                                                         \
        if (err_ch && vec_ok) CMPQ_RTN_LAUNCH(TW, true, true);   \
        else if (err_ch) CMPQ_RTN_LAUNCH(TW, true, false);       \
        else if (vec_ok) CMPQ_RTN_LAUNCH(TW, false, true);       \
        else CMPQ_RTN_LAUNCH(TW, false, false);                  \
    } while (0)
    if (dtype == CMPQ_F16) CMPQ_RTN_PICK(__half);
    else CMPQ_RTN_PICK(float);
#undef CMPQ_RTN_PICK
#undef CMPQ_RTN_LAUNCH
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
