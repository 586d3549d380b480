// cmpq_pack: the stored format of Sec. 5.1 / Fig. 4 (arXiv 2410.13056): channels are
// grouped by width, each group is one bit-packed code matrix with a row per channel,
// plus the channel list and the FP16 look-up table of each row.
//
// HBM bound: 1 byte per weight in, bits/8 bytes out.  A lane packs 32 codes (two
// 16-byte loads) into `b` whole words, so rows never share a word between lanes and
// neighbouring lanes write neighbouring words.
#include "common.h"

namespace {

struct PackPtrs {
    uint32_t *packed[4];
    int32_t *chan_idx[4];
    uint16_t *lut[4];
    int width[4];
    int n_set;
};

// row_of[i] = row of channel i inside its width group, -1 when it stores no row.
__global__ __launch_bounds__(1024) void pack_index_kernel(const uint8_t *__restrict__ bits,
                                                          int64_t d_in, PackPtrs p,
                                                          int32_t *__restrict__ row_of) {
    __shared__ uint32_t scan[17];
    for (int64_t i = threadIdx.x; i < d_in; i += blockDim.x) row_of[i] = -1;
    __syncthreads();
    for (int j = 0; j < p.n_set; ++j) {
        uint32_t run = 0;
        for (int64_t base = 0; base < d_in; base += blockDim.x) {
            const int64_t i = base + threadIdx.x;
            const uint32_t f = i < d_in && bits[i] == p.width[j];
            uint32_t total;
            const uint32_t row = run + block_scan_excl_u32(f, scan, &total);
            if (f) {
                row_of[i] = (int32_t)row;
                if (p.chan_idx[j]) p.chan_idx[j][row] = (int32_t)i;
            }
            run += total;
        }
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
            const uint4 r0 = *reinterpret_cast<const uint4 *>(crow + o0);
            const uint4 r1 = *reinterpret_cast<const uint4 *>(crow + o0 + 16);
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

}  // namespace

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
