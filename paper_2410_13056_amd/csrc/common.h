// Internal helpers shared by the HIP translation units of libcmpq (gfx950 only).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "cmpq.h"

#define CMPQ_WAVE 64

#define CMPQ_LAUNCH_CHECK()                                   \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return CMPQ_EHIP; \
    } while (0)

// Measurement hook of cmpq_time_kernel: brackets a launch of `kernel` with the events the
// calling thread armed, if any.
void cmpq_timing_before(int kernel, hipStream_t s);
void cmpq_timing_after(int kernel, hipStream_t s);

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
__device__ __forceinline__ size_t align_up_dev(size_t x) { return (x + 15) & ~(size_t)15; }

// seg[i] = number of entries of the ascending list idx[0..n) below i*d_out, i = 0..d_in.
int launch_segment_offsets(const int32_t *idx, int64_t n, int64_t d_in, int64_t d_out, int32_t *seg,
                           hipStream_t s);

// err_ch[i] = sum_o (W - W_hat)^2 of cmpq_dequant_error, one workgroup per channel; `slices`
// (nullable) cuts out_idx by channel.
int launch_dequant_error_rows(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                              const float *centroids, const uint8_t *codes, const uint8_t *bits,
                              const int32_t *out_idx, const int32_t *slices, double *err_ch, hipStream_t s);
// totals[0] = sum_i sumsq[i] * err_ch[i] (sumsq null: weight 1), totals[1] = sum_i err_ch[i].
int launch_error_totals(const double *err_ch, const float *sumsq, int64_t d_in, double *totals, hipStream_t s);

// Where the stored format of cmpq_pack goes: per width of the bit set the packed rows, the
// channel list and the FP16 tables (device pointers; null for a width without channels).
struct PackPtrs {
    uint32_t *packed[4];
    int32_t *chan_idx[4];
    uint16_t *lut[4];
    int width[4];
    int n_set;
};
// Checks the host arrays of cmpq_pack and gathers the device pointers.
int gather_pack_ptrs(int64_t d_in, int64_t d_out, const int32_t *bit_set, int n_set, const int64_t *counts_host,
                     uint32_t *const *packed, int32_t *const *chan_idx, uint16_t *const *lut, PackPtrs &p);
// row_of[i] = row of channel i inside its width group (-1: it stores no row); fills the channel lists.
int launch_pack_index(const uint8_t *bits, int64_t d_in, const PackPtrs &p, int32_t *row_of, hipStream_t s);

// Carves aligned pieces out of the caller's workspace; `need` ends up as the total.
struct WsCarver {
    char *base;
    size_t off = 0;
    explicit WsCarver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t count) {
        off = align_up(off, 256);
        T *p = reinterpret_cast<T *>(base + off);
        off += count * sizeof(T);
        return p;
    }
    size_t need() const { return align_up(off, 256); }
};

// The wavefront's number inside its workgroup, as a value the compiler knows to be the same
// in every lane: counters and addresses derived from it (row ranges, units, wave-chunks) then
// live in scalar registers and the loop control costs no vector instructions.
// 16 bytes of a stream that the kernel reads once (16-byte aligned): loaded past the caches'
// keep-for-later policy, which on this machine runs a read-once pass 7-15 % faster.
__device__ __forceinline__ uint4 load16_stream(const void *p) {
    typedef uint32_t U4 __attribute__((ext_vector_type(4)));
    const U4 v = __builtin_nontemporal_load(static_cast<const U4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ int wave_index() {
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x / CMPQ_WAVE));
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_down(v, s, CMPQ_WAVE);
    return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_down(v, s, CMPQ_WAVE);
    return v;
}

// Inclusive scan over the lanes of a wave, on the DPP data path: shifts by 1, 2, 4, 8
// inside each row of 16 lanes (lanes shifted in from outside a row read 0), then the last
// lane of row 0 / 2 into rows 1 / 3 and the last lane of the lower half into the upper.
__device__ __forceinline__ uint32_t wave_scan_incl_u32(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31 -> rows 2, 3
    return v;
}

// Exclusive scan of one value per thread over a block of up to 1024 threads.
// `scratch` holds at least 17 uint32 in LDS.  Returns the exclusive prefix and
// leaves the block total in *total.  Contains barriers: call from all threads.
__device__ __forceinline__ uint32_t block_scan_excl_u32(uint32_t v, uint32_t *scratch,
                                                        uint32_t *total) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = threadIdx.x / CMPQ_WAVE;
    const int nwave = (blockDim.x + CMPQ_WAVE - 1) / CMPQ_WAVE;
    uint32_t incl = wave_scan_incl_u32(v);
    __syncthreads();  // scratch may still be read from a previous call
    if (lane == CMPQ_WAVE - 1) scratch[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        uint32_t w = lane < nwave ? scratch[lane] : 0;
        uint32_t wi = wave_scan_incl_u32(w);
        if (lane < nwave) scratch[lane] = wi - w;
        if (lane == nwave - 1) scratch[16] = wi;
    }
    __syncthreads();
    *total = scratch[16];
    return scratch[wave] + incl - v;
}

// Exclusive scan of two values per thread at once (one set of barriers).  `scratch`
// holds at least 34 uint32 in LDS.  Contains barriers: call from all threads.
__device__ __forceinline__ void block_scan_excl_2xu32(uint32_t a, uint32_t b, uint32_t *scratch,
                                                      uint32_t &a_excl, uint32_t &b_excl,
                                                      uint32_t &a_total, uint32_t &b_total) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = threadIdx.x / CMPQ_WAVE;
    const int nwave = (blockDim.x + CMPQ_WAVE - 1) / CMPQ_WAVE;
    const uint32_t ai = wave_scan_incl_u32(a), bi = wave_scan_incl_u32(b);
    __syncthreads();  // scratch may still be read from a previous call
    if (lane == CMPQ_WAVE - 1) {
        scratch[wave] = ai;
        scratch[17 + wave] = bi;
    }
    __syncthreads();
    if (wave == 0) {
        const uint32_t wa = lane < nwave ? scratch[lane] : 0, wb = lane < nwave ? scratch[17 + lane] : 0;
        const uint32_t wai = wave_scan_incl_u32(wa), wbi = wave_scan_incl_u32(wb);
        if (lane < nwave) {
            scratch[lane] = wai - wa;
            scratch[17 + lane] = wbi - wb;
        }
        if (lane == nwave - 1) {
            scratch[16] = wai;
            scratch[33] = wbi;
        }
    }
    __syncthreads();
    a_total = scratch[16];
    b_total = scratch[33];
    a_excl = scratch[wave] + ai - a;
    b_excl = scratch[17 + wave] + bi - b;
}

// Four B-bit codes, one per byte of `r`, moved together into the low 4*B bits.
template <int B>
__device__ __forceinline__ uint32_t squeeze4(uint32_t r) {
    constexpr uint32_t m = (1u << B) - 1u, m2 = (1u << (2 * B)) - 1u;
    uint32_t x = r & (m * 0x01010101u);
    x = (x | (x >> (8 - B))) & (m2 * 0x00010001u);
    return (x | (x >> (16 - 2 * B))) & ((1u << (4 * B)) - 1u);
}

// fp32 bit pattern -> unsigned key with the same order as the value.
__device__ __forceinline__ uint32_t f32_ordered_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float f32_from_ordered_key(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

template <typename T>
__device__ __forceinline__ float load_as_f32(const T *p, int64_t i);
template <>
__device__ __forceinline__ float load_as_f32<__half>(const __half *p, int64_t i) {
    return __half2float(p[i]);
}
template <>
__device__ __forceinline__ float load_as_f32<float>(const float *p, int64_t i) {
    return p[i];
}
