// cmpq_pack: the stored format of Sec. 5.1 / Fig. 4 (arXiv 2410.13056): channels are
// grouped by width, each group is one bit-packed code matrix with a row per channel,
// plus the channel list and the FP16 look-up table of each row.
//
// HBM bound: 1 byte per weight in, bits/8 bytes out.  A lane packs 32 codes (two
// 16-byte loads) into `b` whole words, so rows never share a word between lanes and
// neighbouring lanes write neighbouring words.
#include "common.h"

namespace {

// row_of[i] = row of channel i inside its width group, -1 when it stores no row.  One pass: the
// flags of up to four widths are scanned together, two 16-bit fields to a word (a step covers
// 1024 channels, so no field overflows).
__global__ __launch_bounds__(1024) void pack_index_kernel(const uint8_t *__restrict__ bits,
                                                          int64_t d_in, PackPtrs p,
                                                          int32_t *__restrict__ row_of) {
    __shared__ uint32_t scan[34];
    uint32_t run[4] = {0, 0, 0, 0};
    for (int64_t base = 0; base < d_in; base += blockDim.x) {
        const int64_t i = base + threadIdx.x;
        int j = -1;
        if (i < d_in) {
            const int w = bits[i];
            for (int t = 0; t < p.n_set; ++t)
                if (w == p.width[t]) j = t;
        }
        const uint32_t a = j == 0 ? 1u : (j == 1 ? 0x10000u : 0u), b = j == 2 ? 1u : (j == 3 ? 0x10000u : 0u);
        uint32_t a_excl, b_excl, a_total, b_total;
        block_scan_excl_2xu32(a, b, scan, a_excl, b_excl, a_total, b_total);
        if (j >= 0) {
            const uint32_t field = j < 2 ? a_excl : b_excl;
            const uint32_t before = j == 0 ? run[0] : (j == 1 ? run[1] : (j == 2 ? run[2] : run[3]));
            const uint32_t row = before + ((j & 1) ? field >> 16 : field & 0xffffu);
            int32_t *list = j == 0 ? p.chan_idx[0] : (j == 1 ? p.chan_idx[1] : (j == 2 ? p.chan_idx[2] : p.chan_idx[3]));
            row_of[i] = (int32_t)row;
            if (list) list[row] = (int32_t)i;
        } else if (i < d_in) {
            row_of[i] = -1;
        }
        run[0] += a_total & 0xffffu, run[1] += a_total >> 16, run[2] += b_total & 0xffffu, run[3] += b_total >> 16;
    }
}

template <int B>
__device__ __forceinline__ void pack32(const uint8_t (&c)[32], uint32_t (&w)[B]) {
#pragma unroll
    for (int t = 0; t < B; ++t) w[t] = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int bit = j * B, word = bit >> 5, sh = bit & 31;
        const uint32_t v = c[j] & ((1u << B) - 1u);
        w[word] |= v << sh;
        if (sh + B > 32) w[word + 1] |= v >> (32 - sh);
    }
}

template <int B>
__device__ void pack_row(const uint8_t *__restrict__ crow, int64_t d_out, uint32_t *__restrict__ dst,
                         bool vec_ok) {
    const int64_t wpr = (d_out * B + 31) / 32, groups = (d_out + 31) / 32;
    for (int64_t g = (int64_t)blockIdx.y * blockDim.x + threadIdx.x; g < groups;
         g += (int64_t)gridDim.y * blockDim.x) {
        const int64_t o0 = g * 32;
        uint8_t c[32];
        if (vec_ok && o0 + 32 <= d_out) {
            const uint4 r0 = load16_stream(crow + o0);
            const uint4 r1 = load16_stream(crow + o0 + 16);
            const uint32_t r[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
            for (int j = 0; j < 32; ++j) c[j] = (r[j >> 2] >> (8 * (j & 3))) & 0xffu;
        } else {
#pragma unroll
            for (int j = 0; j < 32; ++j) c[j] = o0 + j < d_out ? crow[o0 + j] : 0;
        }
        uint32_t w[B];
        pack32<B>(c, w);
#pragma unroll
        for (int t = 0; t < B; ++t)
            if (g * B + t < wpr) dst[g * B + t] = w[t];
    }
}

__global__ __launch_bounds__(256) void pack_codes_kernel(const uint8_t *__restrict__ codes,
                                                         int64_t d_out,
                                                         const uint8_t *__restrict__ bits,
                                                         const float *__restrict__ centroids,
                                                         const int32_t *__restrict__ row_of,
                                                         PackPtrs p, int vec_ok) {
    const int64_t i = blockIdx.x;
    const int32_t row = row_of[i];
    if (row < 0) return;
    const int b = bits[i];
    int j = 0;
    while (j < p.n_set && p.width[j] != b) ++j;
    if (j == p.n_set) return;
    if (blockIdx.y == 0 && p.lut[j] && threadIdx.x < (1 << b))
        p.lut[j][(int64_t)row * (1 << b) + threadIdx.x] =
            __half_as_ushort(__float2half_rn(centroids[i * CMPQ_KMAX + threadIdx.x]));
    if (!p.packed[j]) return;
    const uint8_t *crow = codes + i * d_out;
    uint32_t *dst = p.packed[j] + (int64_t)row * ((d_out * b + 31) / 32);
    switch (b) {
        case 1: pack_row<1>(crow, d_out, dst, vec_ok); break;
        case 2: pack_row<2>(crow, d_out, dst, vec_ok); break;
        case 3: pack_row<3>(crow, d_out, dst, vec_ok); break;
        default: pack_row<4>(crow, d_out, dst, vec_ok); break;
    }
}

// ---- stored format and error in one pass over the codes --------------------------------
//
// cmpq_pack reads a byte per weight and cmpq_dequant_error reads the same byte again with
// the weight.  Here one workgroup per channel fetches 32 codes and 32 weights per lane and
// step, writes the `b` packed words and adds the squared errors: 3 (5 for fp32) bytes in and
// b/8 out per weight instead of 4 (6) in.  The kernel takes channels that are a whole number
// of 32 entries long with 16-byte aligned rows; the entry point sends other shapes through
// the two separate kernels.

constexpr int kPeT = 256;

// Squared errors of eight consecutive entries: levels by code, the weight itself (rounded to
// FP16 for fp32 input) where the entry is restored.
template <typename TW>
__device__ __forceinline__ double error8(const float (&w)[8], uint32_t c_lo, uint32_t c_hi, uint32_t back,
                                         const float *lut, double s) {
    // the eight levels first, without conditions, so that the look-ups go out together
    float level[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) level[j] = lut[((j < 4 ? c_lo : c_hi) >> (8 * (j & 3))) & 15u];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float what = level[j];
        if ((back >> j) & 1u) what = sizeof(TW) == 2 ? w[j] : __half2float(__float2half_rn(w[j]));
        const double d = (double)w[j] - (double)what;
        s = fma(d, d, s);
    }
    return s;
}

// The codes and weights of 32 consecutive entries of a channel as loaded: two 16-byte words
// of codes, 64 (fp16) or 128 (fp32) bytes of weights.
template <typename TW>
struct PeStep {
    static constexpr int kPer = 16 / (int)sizeof(TW);  // weights per 16-byte load
    uint4 code[2];
    uint4 raw[32 / kPer];
};

template <typename TW>
__device__ __forceinline__ void pe_fetch(PeStep<TW> &st, const TW *__restrict__ wrow,
                                         const uint8_t *__restrict__ crow, int64_t g) {
    const int64_t o0 = g * 32;
    st.code[0] = load16_stream(crow + o0);
    st.code[1] = load16_stream(crow + o0 + 16);
#pragma unroll
    for (int q = 0; q < 32 / PeStep<TW>::kPer; ++q)
        st.raw[q] = load16_stream(wrow + o0 + PeStep<TW>::kPer * q);
}

// The 32 codes of r[0..8), four to a word, as B whole words of the bit stream.
template <int B>
__device__ __forceinline__ void pack32_words(const uint32_t (&r)[8], uint32_t (&w)[B]) {
#pragma unroll
    for (int t = 0; t < B; ++t) w[t] = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t f = squeeze4<B>(r[q]);
        const int bit = q * 4 * B, word = bit >> 5, sh = bit & 31;
        w[word] |= f << sh;
        if (sh + 4 * B > 32) w[word + 1] |= f >> (32 - sh);
    }
}

// 32 codes packed and written as B words.
template <int B>
__device__ __forceinline__ void pack_store(const uint32_t (&r)[8], uint32_t *__restrict__ dst) {
    uint32_t pw[B];
    pack32_words<B>(r, pw);
#pragma unroll
    for (int t = 0; t < B; ++t) dst[t] = pw[t];
}

// One channel of d_out = 32 * groups entries: a lane takes 32 consecutive entries per step.
template <typename TW>
__device__ __forceinline__ double pack_error_row(const TW *__restrict__ wrow, const uint8_t *__restrict__ crow,
                                                 int64_t groups, uint32_t *__restrict__ dst, int b,
                                                 const uint32_t *restored, const float *lut, bool whole) {
    double s = 0.0;
    for (int64_t g = threadIdx.x; g < groups; g += kPeT) {
        PeStep<TW> cur;
        pe_fetch<TW>(cur, wrow, crow, g);
        // the 32 flags of the step are one word of the bitmap
        const uint32_t back = whole ? 0xffffffffu : restored[g];
        const uint32_t r[8] = {cur.code[0].x, cur.code[0].y, cur.code[0].z, cur.code[0].w,
                               cur.code[1].x, cur.code[1].y, cur.code[1].z, cur.code[1].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float w[8];
            if constexpr (sizeof(TW) == 2) {
                const __half2 *hp = reinterpret_cast<const __half2 *>(&cur.raw[q]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float2 t = __half22float2(hp[j]);
                    w[2 * j] = t.x;
                    w[2 * j + 1] = t.y;
                }
            } else {
                const float *fp = reinterpret_cast<const float *>(&cur.raw[2 * q]);
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = fp[j];
            }
            s = error8<TW>(w, r[2 * q], r[2 * q + 1], (back >> (8 * q)) & 0xffu, lut, s);
        }
        if (dst) {  // the error code above is shared by all widths; only this step differs
            switch (b) {
                case 1: pack_store<1>(r, dst + g); break;
                case 2: pack_store<2>(r, dst + g * 2); break;
                case 3: pack_store<3>(r, dst + g * 3); break;
                default: pack_store<4>(r, dst + g * 4); break;
            }
        }
    }
    return s;
}

template <typename TW>
__global__ __launch_bounds__(kPeT) void pack_error_kernel(
    const TW *__restrict__ W, int64_t d_out, int64_t ldw, const uint8_t *__restrict__ codes,
    const uint8_t *__restrict__ bits, const float *__restrict__ centroids,
    const int32_t *__restrict__ row_of, PackPtrs p, const int32_t *__restrict__ out_idx,
    const int32_t *__restrict__ slices, double *__restrict__ err_ch) {
    extern __shared__ uint32_t restored[];  // one bit per entry of the channel
    __shared__ float lut[CMPQ_KMAX];
    __shared__ double red[kPeT / CMPQ_WAVE];
    __shared__ int seg[2];
    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    const TW *wrow = W + i * ldw;
    const uint8_t *crow = codes + i * d_out;
    const int words = (int)(d_out / 32);
    const int b = bits[i];
    const bool whole = b < 1 || b > 4;  // a channel of O_act: every entry restored, no row stored
    for (int w = tid; w < words; w += kPeT) restored[w] = 0;
    if (tid < CMPQ_KMAX) lut[tid] = centroids[i * CMPQ_KMAX + tid];
    if (tid == 0) {
        seg[0] = slices ? slices[i] : 0;
        seg[1] = slices ? slices[i + 1] : 0;
    }
    __syncthreads();
    for (int e = seg[0] + tid; e < seg[1]; e += kPeT) {
        const int o = (int)(out_idx[e] - i * d_out);
        atomicOr(&restored[o >> 5], 1u << (o & 31));
    }
    // the row of the channel in its width group, its table, and where its words go
    const int32_t row = row_of[i];
    int j = 0;
    while (j < p.n_set && p.width[j] != b) ++j;
    uint32_t *dst = nullptr;
    if (row >= 0 && j < p.n_set) {
        if (p.lut[j] && tid < (1 << b))
            p.lut[j][(int64_t)row * (1 << b) + tid] =
                __half_as_ushort(__float2half_rn(centroids[i * CMPQ_KMAX + tid]));
        if (p.packed[j]) dst = p.packed[j] + (int64_t)row * (words * b);
    }
    __syncthreads();
    double s = pack_error_row<TW>(wrow, crow, words, dst, b, restored, lut, whole);
    s = wave_sum_f64(s);
    if ((tid & 63) == 0) red[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int w = 0; w < kPeT / CMPQ_WAVE; ++w) t += red[w];
        err_ch[i] = t;
    }
}

}  // namespace

int gather_pack_ptrs(int64_t d_in, int64_t d_out, const int32_t *bit_set, int n_set, const int64_t *counts_host,
                     uint32_t *const *packed, int32_t *const *chan_idx, uint16_t *const *lut, PackPtrs &p) {
    if (n_set < 1 || n_set > 4) return CMPQ_EBUDGET;
    p.n_set = n_set;
    for (int j = 0; j < 4; ++j) {
        p.packed[j] = nullptr;
        p.chan_idx[j] = nullptr;
        p.lut[j] = nullptr;
        p.width[j] = 0;
    }
    for (int j = 0; j < n_set; ++j) {
        if (bit_set[j] < 1 || bit_set[j] > 4 || (j && bit_set[j] <= bit_set[j - 1])) return CMPQ_EBUDGET;
        if (counts_host[j] < 0 || counts_host[j] > d_in) return CMPQ_EINVAL;
        p.width[j] = bit_set[j];
        if (counts_host[j] > 0) {
            if (!packed || !chan_idx || !lut) return CMPQ_EINVAL;
            p.packed[j] = packed[j];
            p.chan_idx[j] = chan_idx[j];
            p.lut[j] = lut[j];
            if (!p.chan_idx[j] || !p.lut[j] || (d_out > 0 && !p.packed[j])) return CMPQ_EINVAL;
        }
    }
    return CMPQ_OK;
}

int launch_pack_index(const uint8_t *bits, int64_t d_in, const PackPtrs &p, int32_t *row_of, hipStream_t s) {
    pack_index_kernel<<<1, 1024, 0, s>>>(bits, d_in, p, row_of);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

size_t cmpq_ws_pack(int64_t d_in) { return align_up((size_t)(d_in > 0 ? d_in : 1) * sizeof(int32_t), 256); }

extern "C" int cmpq_pack(const uint8_t *codes, int64_t d_in, int64_t d_out, const uint8_t *bits,
                         const float *centroids, const int32_t *bit_set, int n_set,
                         const int64_t *counts_host, uint32_t *const *packed,
                         int32_t *const *chan_idx, uint16_t *const *lut, void *ws, size_t ws_bytes,
                         void *stream) {
    if (d_in < 0 || d_out < 0 || !bits || !bit_set || !counts_host) return CMPQ_EINVAL;
    if (n_set < 1 || n_set > 4) return CMPQ_EBUDGET;
    if (d_in >= (int64_t)1 << 31) return CMPQ_ESHAPE;
    PackPtrs p;
    if (const int rc = gather_pack_ptrs(d_in, d_out, bit_set, n_set, counts_host, packed, chan_idx, lut, p)) return rc;
    if (d_in == 0) return CMPQ_OK;
    if (!centroids || (d_out > 0 && !codes)) return CMPQ_EINVAL;
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_pack(d_in))
        return CMPQ_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *row_of = static_cast<int32_t *>(ws);
    pack_index_kernel<<<1, 1024, 0, s>>>(bits, d_in, p, row_of);
    const int vec_ok = reinterpret_cast<uintptr_t>(codes) % 16 == 0 && d_out % 16 == 0;
    int64_t gy = cdiv(cdiv(d_out, 32), 256);
    if (gy < 1) gy = 1;
    if (gy > 64) gy = 64;
    dim3 grid((unsigned)d_in, (unsigned)gy);
    pack_codes_kernel<<<grid, 256, 0, s>>>(codes, d_out, bits, centroids, row_of, p, vec_ok);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

size_t cmpq_ws_pack_with_error(int64_t d_in) {
    const int64_t n = d_in > 0 ? d_in : 1;
    return align_up((size_t)n * sizeof(int32_t), 256) + align_up((size_t)(n + 1) * sizeof(int32_t), 256);
}

extern "C" int cmpq_pack_with_error(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                                    const uint8_t *codes, const uint8_t *bits, const float *centroids,
                                    const int32_t *bit_set, int n_set, const int64_t *counts_host,
                                    uint32_t *const *packed, int32_t *const *chan_idx,
                                    uint16_t *const *lut, const int32_t *out_idx, int64_t n_out,
                                    const float *sumsq, double *err_ch, double *err_total, void *ws,
                                    size_t ws_bytes, void *stream) {
    if (d_in < 0 || d_out < 0 || n_out < 0 || !bits || !bit_set || !counts_host) return CMPQ_EINVAL;
    if (dtype != CMPQ_F16 && dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (!centroids || !err_ch || !err_total || (n_out > 0 && !out_idx)) return CMPQ_EINVAL;
    if (d_in > 0 && d_out > 0 && (!W || !codes)) return CMPQ_EINVAL;
    if (ldw < d_out) return CMPQ_ESHAPE;
    if (d_in >= (int64_t)1 << 31 || (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in)) return CMPQ_ESHAPE;
    if (d_out > 1 << 20) return CMPQ_ESHAPE;  // the per-channel bitmap lives in LDS
    PackPtrs p;
    if (const int rc = gather_pack_ptrs(d_in, d_out, bit_set, n_set, counts_host, packed, chan_idx, lut, p)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d_in > 0) {
        if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_pack_with_error(d_in))
            return CMPQ_EWORKSPACE;
        int32_t *row_of = static_cast<int32_t *>(ws);
        int32_t *seg = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + align_up((size_t)d_in * sizeof(int32_t), 256));
        pack_index_kernel<<<1, 1024, 0, s>>>(bits, d_in, p, row_of);
        CMPQ_LAUNCH_CHECK();
        const int32_t *slices = nullptr;
        if (n_out > 0) {
            const int rc = launch_segment_offsets(out_idx, n_out, d_in, d_out, seg, s);
            if (rc != CMPQ_OK) return rc;
            slices = seg;
        }
        const int esz = dtype == CMPQ_F16 ? 2 : 4;
        const bool one_pass = d_out > 0 && d_out % 32 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0 &&
                              (ldw * esz) % 16 == 0 && reinterpret_cast<uintptr_t>(codes) % 16 == 0;
        if (one_pass) {
            const size_t lds = (size_t)(d_out / 32) * 4;
            cmpq_timing_before(CMPQ_KERNEL_PACK_ERROR, s);
            if (dtype == CMPQ_F16)
                pack_error_kernel<__half><<<(unsigned)d_in, kPeT, lds, s>>>(
                    static_cast<const __half *>(W), d_out, ldw, codes, bits, centroids, row_of, p, out_idx, slices,
                    err_ch);
            else
                pack_error_kernel<float><<<(unsigned)d_in, kPeT, lds, s>>>(
                    static_cast<const float *>(W), d_out, ldw, codes, bits, centroids, row_of, p, out_idx, slices,
                    err_ch);
            cmpq_timing_after(CMPQ_KERNEL_PACK_ERROR, s);
            CMPQ_LAUNCH_CHECK();
        } else {  // ragged or unaligned rows: the kernels of the two separate calls
            const int vec_ok = reinterpret_cast<uintptr_t>(codes) % 16 == 0 && d_out % 16 == 0;
            int64_t gy = cdiv(cdiv(d_out, 32), 256);
            if (gy < 1) gy = 1;
            if (gy > 64) gy = 64;
            pack_codes_kernel<<<dim3((unsigned)d_in, (unsigned)gy), 256, 0, s>>>(codes, d_out, bits, centroids,
                                                                                  row_of, p, vec_ok);
            CMPQ_LAUNCH_CHECK();
            if (const int rc = launch_dequant_error_rows(W, dtype, d_in, d_out, ldw, centroids, codes, bits,
                                                         out_idx, slices, err_ch, s))
                return rc;
        }
    }
    return launch_error_totals(err_ch, sumsq, d_in, err_total, s);
}
