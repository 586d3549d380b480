// Order keys of fp16 values and the exact level arithmetic of the histogram K-means
// (Sec. 3.2.1 of arXiv 2410.13056; nearest level of Sec. 3 eq. Q(x) in exact arithmetic):
// shared by the per-channel bucket kernel and the per-layer clustering of the table centres.
#pragma once
#include "common.h"

namespace {

constexpr uint32_t kKeyInf = 0xffffu;     // boundary above every key
constexpr uint32_t kFill4 = 0x80808080u;  // four filler bytes: above every place (<= 127)

// Order key of an fp16 bit pattern: unsigned key order = value order.  -0 comes out one
// key below +0 (0x7fff, 0x8000); nothing else lies between, and boundary_key never
// returns 0x7fff, so the two zeros always share a cell.
__device__ __forceinline__ uint32_t key_of_half(uint32_t h) {
    return (h & 0x8000u) ? (~h & 0xffffu) : (h | 0x8000u);
}
__device__ __forceinline__ uint32_t half_of_key(uint32_t k) {
    return (k & 0x8000u) ? (k & 0x7fffu) : (~k & 0xffffu);
}
__device__ __forceinline__ float value_of_key(uint32_t k) {
    return __half2float(__ushort_as_half((unsigned short)half_of_key(k)));
}
// Two fp16 patterns in one word -> their two keys: flip the sign bit of a non-negative
// value, every bit of a negative one.
__device__ __forceinline__ uint32_t keys_of_half2(uint32_t w) {
    const uint32_t neg = (w >> 15) & 0x00010001u;
    return w ^ (__umul24(neg, 0x7fffu) + 0x80008000u);
}
// Bits 15 and 31 of the result are set where the exponent field is all ones.
__device__ __forceinline__ uint32_t nonfinite_of_half2(uint32_t w) {
    return (w & 0x7c007c00u) + 0x04000400u;
}

// x*2^24 of the first key of bucket b, and the step per place inside the bucket.
// For a normal half (e >= 1) x*2^24 = (1024 + m) << (e - 1); a subnormal gives m.
template <int LB>
__device__ __forceinline__ void bucket_affine(uint32_t b, long long &q0, long long &step) {
    const uint32_t h = half_of_key(b << LB);
    const uint32_t e = (h >> 10) & 31u, m = h & 1023u;
    const uint32_t sh = (e > 1 ? e : 1) - 1;
    step = 1ll << sh;
    const long long mag = (long long)((e ? 1024u : 0u) + m) << sh;
    q0 = (h & 0x8000u) ? -mag : mag;
}

// Sum of x*2^24 over n keys of bucket b whose places add up to l (n <= 32768, places <= 127):
// (n * q0 + step * l) of bucket_affine, formed as a 32-bit product and one 64-bit shift
// (|mantissa * n| < 2^26 and l < 2^23, so their sum fits 32 bits).
template <int LB>
__device__ __forceinline__ long long bucket_sum(uint32_t b, uint32_t n, uint32_t l) {
    const uint32_t h = half_of_key(b << LB);
    const uint32_t e = (h >> 10) & 31u;
    const uint32_t sh = (e > 1 ? e : 1) - 1;
    const int mant = (int)((e ? 1024u : 0u) + (h & 1023u));
    const int t = __mul24((h & 0x8000u) ? -mant : mant, (int)n) + (int)l;
    return (long long)((unsigned long long)(long long)t << sh);
}

// Value of the lane below / above inside a row of 16 lanes; 0 at the row's edge.
__device__ __forceinline__ uint32_t row_from_below(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);  // row_shr:1
}
__device__ __forceinline__ uint32_t row_from_above(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x101, 0xF, 0xF, true);  // row_shl:1
}

// Sum over aligned groups of L lanes (L a power of two, 4..64); every lane gets its group's sum.
template <int L>
__device__ __forceinline__ uint32_t group_sum(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    if constexpr (L >= 8) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    if constexpr (L >= 16) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false); // row_mirror
    if constexpr (L >= 32) v += __shfl_xor(v, 16, CMPQ_WAVE);
    if constexpr (L >= 64) v += __shfl_xor(v, 32, CMPQ_WAVE);
    return v;
}

__device__ __forceinline__ unsigned long long wave_scan_incl_u64(unsigned long long v) {
    // Three limbs of 22, 22 and 20 bits: the 64 partial sums of a limb stay below 2^28, so
    // each limb is scanned on the DPP path, and the limbs are joined modulo 2^64 (sums of
    // two's complement values come out right).
    const uint32_t l0 = (uint32_t)v & 0x3fffffu, l1 = (uint32_t)(v >> 22) & 0x3fffffu, l2 = (uint32_t)(v >> 44);
    const uint32_t s0 = wave_scan_incl_u32(l0), s1 = wave_scan_incl_u32(l1), s2 = wave_scan_incl_u32(l2);
    return (unsigned long long)s0 + ((unsigned long long)s1 << 22) + ((unsigned long long)s2 << 44);
}

// Exclusive scan of a (count, sum) pair per thread over the workgroup, one set of
// barriers for both.  scratch32 / scratch64 hold 17 entries each.
__device__ __forceinline__ void block_scan_excl_pair(uint32_t n, unsigned long long v, uint32_t *scratch32,
                                                     unsigned long long *scratch64, uint32_t &n_excl,
                                                     unsigned long long &v_excl, uint32_t &n_total,
                                                     unsigned long long &v_total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwave = (blockDim.x + 63) >> 6;
    const uint32_t n_incl = wave_scan_incl_u32(n);
    const unsigned long long v_incl = wave_scan_incl_u64(v);
    if (lane == 63) {
        scratch32[wave] = n_incl;
        scratch64[wave] = v_incl;
    }
    __syncthreads();
    if (wave == 0) {
        const uint32_t wn = lane < nwave ? scratch32[lane] : 0u;
        const unsigned long long wv = lane < nwave ? scratch64[lane] : 0ull;
        const uint32_t wni = wave_scan_incl_u32(wn);
        const unsigned long long wvi = wave_scan_incl_u64(wv);
        if (lane < nwave) {
            scratch32[lane] = wni - wn;
            scratch64[lane] = wvi - wv;
        }
        if (lane == nwave - 1) {
            scratch32[16] = wni;
            scratch64[16] = wvi;
        }
    }
    __syncthreads();
    n_total = scratch32[16];
    v_total = scratch64[16];
    n_excl = scratch32[wave] + n_incl - n;
    v_excl = scratch64[wave] + v_incl - v;
}

// Number of boundary keys below `key` (boundaries ascending, repeats allowed).
template <int K>
__device__ __forceinline__ uint32_t cell_of(uint32_t q, const uint32_t (&t)[CMPQ_KMAX]) {
    if constexpr (K == 2) {
        return q > t[0];
    } else if constexpr (K == 4) {
        const bool c1 = q > t[1];
        const uint32_t u = c1 ? t[2] : t[0];
        return 2u * c1 + (q > u);
    } else if constexpr (K == 8) {
        const bool c2 = q > t[3];
        const uint32_t u1 = c2 ? t[5] : t[1];
        const bool c1 = q > u1;
        const uint32_t a = c1 ? t[2] : t[0], b = c1 ? t[6] : t[4];
        const uint32_t u0 = c2 ? b : a;
        return 4u * c2 + 2u * c1 + (q > u0);
    } else {
        const bool c3 = q > t[7];
        const uint32_t u2 = c3 ? t[11] : t[3];
        const bool c2 = q > u2;
        const uint32_t a1 = c2 ? t[5] : t[1], b1 = c2 ? t[13] : t[9];
        const uint32_t u1 = c3 ? b1 : a1;
        const bool c1 = q > u1;
        const uint32_t x0 = c1 ? t[2] : t[0], x1 = c1 ? t[6] : t[4];
        const uint32_t x2 = c1 ? t[10] : t[8], x3 = c1 ? t[14] : t[12];
        const uint32_t y0 = c2 ? x1 : x0, y1 = c2 ? x3 : x2;
        const uint32_t u0 = c3 ? y1 : y0;
        return 8u * c3 + 4u * c2 + 2u * c1 + (q > u0);
    }
}

// The largest fp16 value that is not above x (x finite, |x| < 65504), as its bit pattern: the
// two narrowing conversions run with the rounding mode set to "towards minus infinity" (both
// precision groups of the mode register), which is put back to "nearest even" - the mode this
// library's kernels run in - before the block ends.  Rounding down twice is rounding down once.
__device__ __forceinline__ uint32_t floor_half_of_double(double x) {
    uint32_t h;
    float f;
    asm volatile(
        "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 4), 0xa\n\t"
        "s_nop 1\n\t"
        "v_cvt_f32_f64 %1, %2\n\t"
        "s_nop 0\n\t"
        "v_cvt_f16_f32 %0, %1\n\t"
        "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 4), 0x0\n\t"
        "s_nop 1"
        : "=v"(h), "=&v"(f)
        : "v"(x));
    return h & 0xffffu;
}

// Key of the largest fp16 value that belongs to `lo` rather than `hi` (lo < hi): values
// below the midpoint, and the midpoint itself when lo has the smaller level index.
// Never the key of -0: a boundary there would part the two zeros.
__device__ __forceinline__ uint32_t boundary_key(float lo, float hi, int owner_lo, int owner_hi) {
    const double mid = ((double)lo + (double)hi) * 0.5;  // exact
    uint32_t h = floor_half_of_double(mid);
    h = h == 0x8000u ? 0u : h;  // -0 is +0 here
    uint32_t key = key_of_half(h);
    key -= ((double)value_of_key(key) == mid && owner_hi < owner_lo) ? 1u : 0u;
    return key == 0x7fffu ? 0x7ffeu : key;
}

// Wave 0: levels by level index (lane j holds c for j < K) -> per sorted position p
// (lane p): value, owning level, next distinct value above and the owners for the tie
// rule.  Handles repeated values and any order.
template <int K>
__device__ __forceinline__ void rank_levels(float c, float &sorted, int &own, float &hi,
                                            int &owner_lo, int &owner_hi, bool &have_hi) {
    const int j = threadIdx.x & 63;
    int rank = 0;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const float cl = __shfl(c, l, CMPQ_WAVE);
        rank += (cl < c) || (cl == c && l < j);
    }
    sorted = INFINITY;
    own = j;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const int rl = __shfl(rank, l, CMPQ_WAVE);
        const float cl = __shfl(c, l, CMPQ_WAVE);
        if (rl == j) {
            sorted = cl;
            own = l;
        }
    }
    hi = INFINITY;
    owner_lo = own;
    owner_hi = 0;
    bool have_lo = false;
    have_hi = false;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const float sl = __shfl(sorted, l, CMPQ_WAVE);
        const int pl = __shfl(own, l, CMPQ_WAVE);
        if (!have_lo && sl == sorted) {
            owner_lo = pl;
            have_lo = true;
        }
        if (!have_hi && l > j && sl > sorted) {
            hi = sl;
            owner_hi = pl;
            have_hi = true;
        }
    }
    if (j >= K - 1) have_hi = false;
}

}  // namespace
