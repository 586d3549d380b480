// cmpq_lut4_quantize: the look-up tables of a layer held in 4 bits (Sec. 5.1 / Tab. 7 of
// arXiv 2410.13056: the variant whose overhead is (1*4 + 8*4)/4096 bits per weight).
//
// The paper does not say how the centres are quantized; its figure leaves 4 bits per table
// entry and no room for anything per channel, and Tab. 7 reports a loss of at most 1.5 %.
//
// Default reading (CMPQ_LUT4_CODEBOOK): the 4 bits index one 16-entry table per layer, found
// by the paper's own non-uniform quantizer (Sec. 3 eq. Q(x), K-means with K = 16) over all
// FP16 centres of the layer.  The centres are FP16 values, so the whole clustering runs on a
// histogram over the 65536 order keys: one kernel counts, one workgroup turns the counts into
// cumulative counts and exact integer sums of x * 2^24, and one wavefront then runs the rounds
// - a boundary between two levels reads its count and sum straight off the cumulative arrays,
// the new level is the exact sum divided in fp64 and rounded once to fp32 (what an fp64
// reference computes).  A last kernel codes every table entry.
//
// Alternative (CMPQ_LUT4_UNIFORM): one uniform 16-level grid per layer - the uniform quantizer
// of Sec. 3 with N = 4 over all centres at once.  Two small kernels: the range of all centres,
// then code and rebuilt level of every entry; the code is decided in fp32 with one IEEE
// division, the rebuilt level is min + code * Delta formed exactly and rounded once to fp32.
#include "kmeans_keys.h"

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

// ---- the per-layer table (CMPQ_LUT4_CODEBOOK) ---------------------------------------------

constexpr int kKeys = 65536;

struct Lut4Ws {
    uint32_t *hist;      // [kKeys] entries per order key
    uint32_t *cum_n;     // [kKeys + 1] entries with a smaller key
    long long *cum_s;    // [kKeys + 1] and the sum of their x * 2^24
    uint32_t *tk;        // [16] final boundary keys by sorted position
    uint32_t *code_of;   // [16] level index of each sorted position
    size_t bytes;
};

Lut4Ws lut4_carve(void *ws) {
    WsCarver c(ws);
    Lut4Ws w;
    w.hist = c.take<uint32_t>(kKeys);
    w.cum_n = c.take<uint32_t>(kKeys + 1);
    w.cum_s = c.take<long long>(kKeys + 1);
    w.tk = c.take<uint32_t>(CMPQ_KMAX);
    w.code_of = c.take<uint32_t>(CMPQ_KMAX);
    w.bytes = c.need();
    return w;
}

// FP16 pattern of a centre as the stored table holds it (round to nearest even), -0 as +0.
__device__ __forceinline__ uint32_t stored_half(float c) {
    const uint32_t h = __half_as_ushort(__float2half_rn(c));
    return h == 0x8000u ? 0u : h;
}

__global__ __launch_bounds__(1024) void lut4_zero_kernel(uint32_t *__restrict__ hist) {
    hist[blockIdx.x * 1024 + threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void lut4_count_kernel(const float *__restrict__ centroids,
                                                         const uint8_t *__restrict__ bits, int64_t d_in,
                                                         uint32_t *__restrict__ hist) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d_in * CMPQ_KMAX) return;
    const int b = bits[e / CMPQ_KMAX];
    if (b < 1 || b > 4 || (int)(e % CMPQ_KMAX) >= (1 << b)) return;
    const uint32_t h = stored_half(centroids[e]);
    if ((h & 0x7c00u) == 0x7c00u) return;  // a non-finite centre takes no part
    atomicAdd(&hist[key_of_half(h)], 1u);
}

// x * 2^24 of the fp16 value with order key `key` (an integer: fp16 values are multiples of 2^-24).
__device__ __forceinline__ long long q24_of_key(uint32_t key) {
    long long q0, step;
    bucket_affine<0>(key, q0, step);
    return q0;
}

// One workgroup: cumulative tables, then wavefront 0 runs the quantile start and the rounds.
__global__ __launch_bounds__(1024) void lut4_cluster_kernel(const uint32_t *__restrict__ hist,
                                                            uint32_t *__restrict__ cum_n,
                                                            long long *__restrict__ cum_s, int iters,
                                                            float *__restrict__ table, uint32_t *__restrict__ tk_out,
                                                            uint32_t *__restrict__ code_of_out) {
    __shared__ uint32_t scan32[17];
    __shared__ unsigned long long scan64[17];
    constexpr int kPer = kKeys / 1024;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t k0 = (uint32_t)tid * kPer;
    uint32_t n_loc = 0;
    long long s_loc = 0;
    for (int r = 0; r < kPer; ++r) {
        const uint32_t n = hist[k0 + r];
        n_loc += n;
        s_loc += (long long)n * q24_of_key(k0 + r);
    }
    uint32_t n_run, M;
    unsigned long long s_run_u, s_tot_u;
    block_scan_excl_pair(n_loc, (unsigned long long)s_loc, scan32, scan64, n_run, s_run_u, M, s_tot_u);
    long long s_run = (long long)s_run_u;
    for (int r = 0; r < kPer; ++r) {
        const uint32_t n = hist[k0 + r];
        cum_n[k0 + r] = n_run;
        cum_s[k0 + r] = s_run;
        n_run += n;
        s_run += (long long)n * q24_of_key(k0 + r);
    }
    if (tid == 1023) {
        cum_n[kKeys] = n_run;
        cum_s[kKeys] = s_run;
    }
    __syncthreads();  // the tables are read below by wavefront 0 of this same workgroup
    if (tid >= 64) return;
    const long long S = (long long)s_tot_u;
    // quantile start: level j = order statistic floor((2j+1)M/32), i.e. the key whose bin holds that rank
    float c0 = lane < CMPQ_KMAX ? 0.0f : INFINITY;
    if (lane < CMPQ_KMAX && M > 0) {
        const uint32_t r = (uint32_t)(((uint64_t)(2 * lane + 1) * M) / 32u);
        uint32_t lo = 0, hi = kKeys - 1;  // largest key with cum_n[key] <= r: its bin is not empty
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (cum_n[mid] <= r) lo = mid; else hi = mid - 1;
        }
        c0 = value_of_key(lo);
        if (c0 == 0.0f) c0 = 0.0f;
    }
    float c_sorted = 0.0f, hi_v = 0.0f;
    int own = lane, owner_lo = 0, owner_hi = 0;
    bool have_hi = false;
    {
        const float c0_up = __uint_as_float(row_from_above(__float_as_uint(c0)));
        if (__ballot(lane < CMPQ_KMAX - 1 && !(c0 < c0_up)) == 0ull) {
            c_sorted = c0;
            hi_v = c0_up;
            owner_lo = lane;
            owner_hi = lane + 1;
            have_hi = lane < CMPQ_KMAX - 1;
        } else {
            rank_levels<CMPQ_KMAX>(c0, c_sorted, own, hi_v, owner_lo, owner_hi, have_hi);
        }
    }
    uint32_t tk_prev = 0xffffffffu;
    for (int round = 0;; ++round) {
        uint32_t tk = kKeyInf;
        if (have_hi) tk = boundary_key(c_sorted, hi_v, owner_lo, owner_hi);
        const bool moved = __ballot(lane < CMPQ_KMAX - 1 && tk != tk_prev) != 0ull;
        tk_prev = tk;
        if (round == iters || !moved) break;  // a fixed point repeats itself
        uint32_t n_below = M;
        long long s_below = S;
        if (lane < CMPQ_KMAX - 1 && tk != kKeyInf) {
            n_below = cum_n[tk + 1];
            s_below = cum_s[tk + 1];
        }
        const uint32_t n_prev = row_from_below(n_below);
        const long long s_prev = (long long)(((unsigned long long)row_from_below((uint32_t)((unsigned long long)s_below >> 32)) << 32) |
                                             row_from_below((uint32_t)s_below));
        const uint32_t n_cell = n_below - n_prev;
        const long long s_cell = s_below - s_prev;
        float c = c_sorted;
        if (lane < CMPQ_KMAX && n_cell > 0)
            c = (float)(((double)s_cell * 5.9604644775390625e-08) / (double)n_cell);
        const float c_up = __uint_as_float(row_from_above(__float_as_uint(c)));
        const int own_up = (int)row_from_above((uint32_t)own);
        if (__ballot(lane < CMPQ_KMAX - 1 && !(c < c_up)) == 0ull) {
            c_sorted = c;
            hi_v = c_up;
            owner_lo = own;
            owner_hi = own_up;
            have_hi = lane < CMPQ_KMAX - 1;
        } else {
            float c_level = INFINITY;
#pragma unroll
            for (int l = 0; l < CMPQ_KMAX; ++l) {
                const int ol = __shfl(own, l, CMPQ_WAVE);
                const float cl = __shfl(c, l, CMPQ_WAVE);
                if (ol == lane) c_level = cl;
            }
            rank_levels<CMPQ_KMAX>(c_level, c_sorted, own, hi_v, owner_lo, owner_hi, have_hi);
        }
    }
    if (lane < CMPQ_KMAX) {
        table[own] = c_sorted;
        tk_out[lane] = tk_prev;
        code_of_out[lane] = (uint32_t)own;
    }
}

__global__ __launch_bounds__(256) void lut4_assign_kernel(const float *__restrict__ centroids,
                                                          const uint8_t *__restrict__ bits, int64_t d_in,
                                                          const float *__restrict__ table,
                                                          const uint32_t *__restrict__ tk,
                                                          const uint32_t *__restrict__ code_of,
                                                          uint8_t *__restrict__ codes4,
                                                          float *__restrict__ centroids_q) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d_in * CMPQ_KMAX) return;
    const int b = bits[e / CMPQ_KMAX];
    uint8_t code = 0;
    float cq = INFINITY;
    if (b >= 1 && b <= 4 && (int)(e % CMPQ_KMAX) < (1 << b)) {
        uint32_t thr[CMPQ_KMAX];
#pragma unroll
        for (int p = 0; p < CMPQ_KMAX; ++p) thr[p] = tk[p];
        const uint32_t h = stored_half(centroids[e]);
        code = (uint8_t)code_of[cell_of<CMPQ_KMAX>(key_of_half(h), thr)];
        cq = __half2float(__float2half_rn(table[code]));
    }
    codes4[e] = code;
    centroids_q[e] = cq;
}

}  // namespace

size_t cmpq_ws_lut4() { return lut4_carve(nullptr).bytes; }

extern "C" int cmpq_lut4_quantize(int mode, const float *centroids, const uint8_t *bits, int64_t d_in, int iters,
                                  uint8_t *codes4, float *table, float *centroids_q, void *ws, size_t ws_bytes,
                                  void *stream) {
    if (d_in < 0 || !table || iters < 0) return CMPQ_EINVAL;
    if (mode != CMPQ_LUT4_CODEBOOK && mode != CMPQ_LUT4_UNIFORM) return CMPQ_EINVAL;
    if (d_in > 0 && (!centroids || !bits || !codes4 || !centroids_q)) return CMPQ_EINVAL;
    if (d_in > ((int64_t)1 << 27)) return CMPQ_ESHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == CMPQ_LUT4_UNIFORM) {
        lut4_range_kernel<<<1, kT, 0, s>>>(centroids, bits, d_in, table);
        if (d_in > 0)
            lut4_code_kernel<<<(unsigned)cdiv(d_in * CMPQ_KMAX, 256), 256, 0, s>>>(centroids, bits, d_in, table,
                                                                                    codes4, centroids_q);
        CMPQ_LAUNCH_CHECK();
        return CMPQ_OK;
    }
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_lut4()) return CMPQ_EWORKSPACE;
    const Lut4Ws w = lut4_carve(ws);
    const unsigned entry_blocks = (unsigned)cdiv(d_in * CMPQ_KMAX, 256);
    lut4_zero_kernel<<<kKeys / 1024, 1024, 0, s>>>(w.hist);
    if (d_in > 0) lut4_count_kernel<<<entry_blocks, 256, 0, s>>>(centroids, bits, d_in, w.hist);
    lut4_cluster_kernel<<<1, 1024, 0, s>>>(w.hist, w.cum_n, w.cum_s, iters, table, w.tk, w.code_of);
    if (d_in > 0)
        lut4_assign_kernel<<<entry_blocks, 256, 0, s>>>(centroids, bits, d_in, table, w.tk, w.code_of, codes4,
                                                         centroids_q);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
