// Fixed-point k-means for the common case of cmpq_kmeans_quantize: fp16 weights, unit
// importance (Sec. 3.2.1 of arXiv 2410.13056; entries of O_q removed as in Sec. 3.2.2).
//
// Every finite fp16 value is an integer multiple of 2^-24.  A channel whose magnitudes
// stay below 128 therefore maps exactly to 32-bit integers q = x * 2^24, kept with a
// bias of 2^31 as unsigned q' so that unsigned order is value order.  Everything the
// Lloyd rounds need becomes integer work on registers:
//   * the lane keeps its weights as q' in VGPRs for the whole kernel (one HBM read);
//   * the cell of a weight is the number of integer thresholds below it, found by a
//     branch-free binary search over K-1 thresholds held in VGPRs (log2 K compares and
//     K-1-log2 K selects) - thresholds are floor(midpoint * 2^24), adjusted for the
//     tie rule, so the cell is the nearest level in exact arithmetic (Sec. 3 eq. Q(x));
//   * sum and count of a cell travel in one 64-bit word (count above bit 47, biased
//     sum below) added with a single LDS atomic into a (cell, lane) table; integer
//     addition is exact and order-free, so results are reproducible bit for bit;
//   * entries of O_q are not masked in the loop: the few of them are subtracted again
//     from the table after the loop, which leaves the loop free of predicates.
// The new level is the exact integer sum divided in fp64 and rounded once to fp32,
// which is what an fp64 reference computes.
//
// A channel that does not fit (|x| >= 128, NaN, infinity) is flagged and left to the
// general kernel.
#include "kmeans_args.h"

namespace {

constexpr int kExclCap = 1024;          // entries of O_q per channel staged in LDS
constexpr uint32_t kBias = 0x80000000u;
constexpr int kCountShift = 47;         // count field of the packed accumulator
constexpr uint32_t kHiOne = 1u << (kCountShift - 32);

struct FastShared {
    unsigned long long acc[CMPQ_KMAX * 64];  // (cell, lane) packed sums
    uint32_t hist[CMPQ_KMAX * 256];          // start-up histograms
    uint32_t excl_q[kExclCap];               // q' of removed entries
    unsigned short excl_key[kExclCap];       // their 16-bit order keys
    unsigned long long tot[CMPQ_KMAX];       // per cell: packed total
    uint32_t thr[CMPQ_KMAX];                 // thresholds in q' units, ascending
    uint32_t grp_of_top[256];                // start-up: top byte -> histogram slot
    float cent[CMPQ_KMAX];                   // levels by level index
    int perm[CMPQ_KMAX];                     // sorted position -> level index
    uint32_t q_rank[CMPQ_KMAX], q_top[CMPQ_KMAX];
    int q_lead[CMPQ_KMAX];
    int seg_lo, n_excl, identity;
};

__device__ __forceinline__ uint32_t half_key(uint32_t h) {  // 16-bit pattern -> ordered key
    return (h & 0x8000u) ? (~h & 0xffffu) : (h | 0x8000u);
}
__device__ __forceinline__ float half_from_key(uint32_t k) {
    const uint32_t h = (k & 0x8000u) ? (k & 0x7fffu) : (~k & 0xffffu);
    return __half2float(__ushort_as_half((unsigned short)h));
}

// Decodes one fp16 pattern: q' for the arithmetic, the 16-bit key for the start-up.
// Returns false when the value does not fit the fixed-point range.
__device__ __forceinline__ bool decode(uint32_t h, uint32_t &qb, uint32_t &key) {
    if (h == 0x8000u) h = 0;  // -0 reads as +0
    const float f = __half2float(__ushort_as_half((unsigned short)h));
    key = half_key(h);
    qb = (uint32_t)(int)(f * 16777216.0f) ^ kBias;
    return fabsf(f) < 128.0f;  // false for NaN and infinity too
}

// Number of thresholds below q (thresholds ascending, repeats allowed).
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

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_down(v, s, CMPQ_WAVE);
    return v;
}

// New levels from the cell totals, ranking of the levels and integer thresholds.
// Run by the first K lanes of wave 0; everything stays in registers (cross-lane reads
// with compile-time lane numbers) until the results are stored for the other waves.
template <int K>
__device__ __noinline__ void update_levels(FastShared &sm, bool first) {
    const int j = threadIdx.x;  // < 64
    float c = j < K ? sm.cent[j] : INFINITY;
    if (!first) {
        // cell p (sorted position) belongs to level perm[p]: bring the totals to level order
        int pos_of_level = 0;  // inverse of perm for this lane's level
#pragma unroll
        for (int p = 0; p < K; ++p) {
            const int lv = sm.perm[p];
            if (lv == j) pos_of_level = p;
        }
        if (j < K) {
            const unsigned long long tot = sm.tot[pos_of_level];
            const uint32_t n = (uint32_t)(tot >> kCountShift);
            if (n) {
                const long long sb = (long long)(tot & ((1ull << kCountShift) - 1));
                const long long ssum = sb - ((long long)n << 31);  // remove the bias
                c = (float)(((double)ssum * 5.9604644775390625e-08) / (double)n);
            }
        }
    }
    // rank by (value, level index)
    int rank = 0;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const float cl = __shfl(c, l, CMPQ_WAVE);
        rank += (cl < c) || (cl == c && l < j);
    }
    float sorted = INFINITY;
    int perm = j;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const int rl = __shfl(rank, l, CMPQ_WAVE);
        const float cl = __shfl(c, l, CMPQ_WAVE);
        if (rl == j) {
            sorted = cl;
            perm = l;
        }
    }
    // for sorted position j: owner of its value group, and the next distinct value
    float hi = INFINITY;
    int owner_lo = perm, owner_hi = 0;
    bool have_lo = false, have_hi = false;
#pragma unroll
    for (int l = 0; l < K; ++l) {
        const float sl = __shfl(sorted, l, CMPQ_WAVE);
        const int pl = __shfl(perm, l, CMPQ_WAVE);
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
    uint32_t t = 0xffffffffu;  // no cell above: nothing exceeds it
    if (j < K - 1 && have_hi) {
        // x goes above iff q > floor(mid * 2^24); an exact tie goes to the smaller level index
        const double m24 = ((double)sorted + (double)hi) * 8388608.0;  // midpoint * 2^24, exact
        double fl = floor(m24);
        if (fl == m24 && owner_hi < owner_lo) fl -= 1.0;
        fl = fmin(fmax(fl, -2147483648.0), 2147483647.0);
        t = (uint32_t)(int)fl ^ kBias;
    }
    if (j < K) {
        sm.cent[j] = c;
        sm.perm[j] = perm;
        sm.thr[j] = t;
    }
    const unsigned long long moved = __ballot(j < K && perm != j);
    if (j == 0) sm.identity = moved == 0ull;
}

template <int G, int K>
__device__ __forceinline__ void lloyd_fast(const KmArgs &a, int64_t i, FastShared &sm, const uint32_t (&q)[4 * G],
                           int n_groups) {
    const int T = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = T >> 6;
    const int kfull = n_groups / T, rem = n_groups % T;  // group k is whole for k < kfull
    const int n_ex = sm.n_excl;
    const int32_t *ex_idx = a.out_idx + sm.seg_lo;
    const __half *wrow = static_cast<const __half *>(a.W) + i * a.ldw;
    for (int round = 0; round <= a.iters; ++round) {
        if (wave == 0) update_levels<K>(sm, round == 0);
        __syncthreads();
        uint32_t thr[CMPQ_KMAX];
#pragma unroll
        for (int p = 0; p < K - 1; ++p) thr[p] = sm.thr[p];
        if (round == a.iters) {  // final coding: 4 codes per lane and store
            uint32_t *crow = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
            const bool ident = sm.identity;
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const int g = k * T + tid;
                if (g < n_groups) {
                    uint32_t word = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uint32_t pos = cell_of<K>(q[4 * k + e], thr);
                        if (!ident) pos = (uint32_t)sm.perm[pos];
                        word |= pos << (8 * e);
                    }
                    crow[g] = word;
                }
            }
            break;
        }
        unsigned long long *slot = sm.acc + lane;
#pragma unroll
        for (int k = 0; k < G; ++k) {
            if (k < kfull || (k == kfull && tid < rem)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t v = q[4 * k + e];
                    const uint32_t pos = cell_of<K>(v, thr);
                    atomicAdd(slot + pos * 64, ((unsigned long long)kHiOne << 32) | v);
                }
            }
        }
        // entries of O_q were counted like the rest: take them out again
        for (int e = tid; e < n_ex; e += T) {
            uint32_t v, key;
            if (e < kExclCap) {
                v = sm.excl_q[e];
            } else {
                decode(__half_as_ushort(wrow[ex_idx[e] - (int32_t)(i * a.d_out)]), v, key);
            }
            const uint32_t pos = cell_of<K>(v, thr);
            atomicAdd(slot + pos * 64, 0ull - (((unsigned long long)kHiOne << 32) | v));
        }
        __syncthreads();
        for (int p = wave; p < K; p += nw) {
            unsigned long long v = sm.acc[p * 64 + lane];
            sm.acc[p * 64 + lane] = 0ull;
            v = wave_sum_u64(v);
            if (lane == 0) sm.tot[p] = v;
        }
        __syncthreads();
    }
}

template <int G>
__global__ __launch_bounds__(1024) void kmeans_fast_kernel(KmArgs a) {
    __shared__ FastShared sm;
    const int64_t i = blockIdx.x;
    const int T = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = T >> 6;
    const int d_out = (int)a.d_out, n_groups = d_out >> 2;
    const int b = a.bits[i];
    float *crow = a.centroids + i * CMPQ_KMAX;
    if (b < 1 || b > 4) {  // a channel of O_act: no levels, no codes
        if (tid < CMPQ_KMAX) crow[tid] = INFINITY;
        uint32_t *c32 = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
        for (int g = tid; g < n_groups; g += T) c32[g] = 0;
        if (tid == 0) a.deferred[i] = 0;
        return;
    }
    const int K = 1 << b;
    // ---- load the channel into registers: lane owns groups g = k*T + tid of 4 weights
    const uint2 *wrow = reinterpret_cast<const uint2 *>(static_cast<const __half *>(a.W) + i * a.ldw);
    uint32_t q[4 * G];
    uint32_t keys[2 * G];  // two 16-bit order keys per word, start-up only
    int fits = 1;
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        uint2 raw = make_uint2(0, 0);
        if (g < n_groups) raw = wrow[g];
        const uint32_t h[4] = {raw.x & 0xffffu, raw.x >> 16, raw.y & 0xffffu, raw.y >> 16};
        uint32_t ky[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) fits &= (int)decode(h[e], q[4 * k + e], ky[e]);
        keys[2 * k] = ky[0] | (ky[1] << 16);
        keys[2 * k + 1] = ky[2] | (ky[3] << 16);
    }
    // ---- the slice of out_idx inside this channel
    if (tid == 0) {
        sm.seg_lo = a.seg ? a.seg[i] : 0;
        const int64_t lo = a.seg ? a.seg[i + 1] : 0;
        sm.n_excl = (int)lo - sm.seg_lo;
    }
    if (!__syncthreads_and(fits)) {  // leave the channel to the general kernel
        if (tid == 0) a.deferred[i] = 1;
        return;
    }
    if (tid == 0) a.deferred[i] = 0;
    const int n_ex = sm.n_excl;
    const int32_t *ex_idx = a.out_idx + sm.seg_lo;
    const __half *w16 = static_cast<const __half *>(a.W) + i * a.ldw;
    for (int e = tid; e < n_ex && e < kExclCap; e += T) {
        uint32_t v, key;
        decode(__half_as_ushort(w16[ex_idx[e] - (int32_t)(i * a.d_out)]), v, key);
        sm.excl_q[e] = v;
        sm.excl_key[e] = (unsigned short)key;
    }
    for (int s = tid; s < CMPQ_KMAX * 64; s += T) sm.acc[s] = 0ull;
    const uint32_t M = (uint32_t)(d_out - n_ex);
    const int kfull = n_groups / T, rem = n_groups % T;

    // ---- start-up: level j = order statistic floor((2j+1)M/(2K)) of the kept weights,
    //      by a two-digit radix select on the 16-bit keys, all K ranks at once
    if (M == 0) {
        if (tid < K) sm.cent[tid] = 0.0f;
    } else {
        for (int s = tid; s < 512; s += T) sm.hist[s] = 0;
        for (int s = tid; s < 256; s += T) sm.grp_of_top[s] = 0xffu;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < G; ++k) {
            if (k < kfull || (k == kfull && tid < rem)) {
                atomicAdd(&sm.hist[(keys[2 * k] >> 8) & 255u], 1u);
                atomicAdd(&sm.hist[keys[2 * k] >> 24], 1u);
                atomicAdd(&sm.hist[(keys[2 * k + 1] >> 8) & 255u], 1u);
                atomicAdd(&sm.hist[keys[2 * k + 1] >> 24], 1u);
            }
        }
        for (int e = tid; e < n_ex; e += T) {
            uint32_t v, key;
            if (e < kExclCap) key = sm.excl_key[e];
            else decode(__half_as_ushort(w16[ex_idx[e] - (int32_t)(i * a.d_out)]), v, key);
            atomicSub(&sm.hist[key >> 8], 1u);
        }
        __syncthreads();
        if (wave == 0) {  // inclusive prefix of the 256 counts into hist[256..511]
            uint32_t c4[4], s = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s += sm.hist[4 * lane + r];
                c4[r] = s;
            }
            const uint32_t before = wave_scan_incl_u32(s) - s;
#pragma unroll
            for (int r = 0; r < 4; ++r) sm.hist[256 + 4 * lane + r] = before + c4[r];
        }
        __syncthreads();
        if (tid < K) {
            const uint32_t rank = (uint32_t)(((uint64_t)(2 * tid + 1) * M) / (uint64_t)(2 * K));
            int lo = 0, hi = 255;  // smallest bin whose inclusive count exceeds rank
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (sm.hist[256 + mid] > rank) hi = mid; else lo = mid + 1;
            }
            sm.q_top[tid] = (uint32_t)lo;
            sm.q_rank[tid] = rank - (sm.hist[256 + lo] - sm.hist[lo]);
        }
        __syncthreads();
        if (tid < K) {  // ranks with the same top byte share one histogram slot
            int lead = tid;
            for (int l = tid - 1; l >= 0; --l)
                if (sm.q_top[l] == sm.q_top[tid]) lead = l;
            sm.q_lead[tid] = lead;
            if (lead == tid) sm.grp_of_top[sm.q_top[tid]] = (uint32_t)tid;
        }
        __syncthreads();
        for (int s = tid; s < K * 256; s += T) sm.hist[s] = 0;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < G; ++k) {
            if (k < kfull || (k == kfull && tid < rem)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t key = (keys[2 * k + (e >> 1)] >> (16 * (e & 1))) & 0xffffu;
                    const uint32_t grp = sm.grp_of_top[key >> 8];
                    if (grp != 0xffu) atomicAdd(&sm.hist[grp * 256 + (key & 255u)], 1u);
                }
            }
        }
        for (int e = tid; e < n_ex; e += T) {
            uint32_t v, key;
            if (e < kExclCap) key = sm.excl_key[e];
            else decode(__half_as_ushort(w16[ex_idx[e] - (int32_t)(i * a.d_out)]), v, key);
            const uint32_t grp = sm.grp_of_top[key >> 8];
            if (grp != 0xffu) atomicSub(&sm.hist[grp * 256 + (key & 255u)], 1u);
        }
        __syncthreads();
        for (int gslot = wave; gslot < K; gslot += nw) {  // inclusive prefix inside each used slot
            if (sm.q_lead[gslot] != gslot) continue;
            uint32_t *h = sm.hist + gslot * 256;
            uint32_t c4[4], s = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s += h[4 * lane + r];
                c4[r] = s;
            }
            const uint32_t before = wave_scan_incl_u32(s) - s;
#pragma unroll
            for (int r = 0; r < 4; ++r) h[4 * lane + r] = before + c4[r];
        }
        __syncthreads();
        if (tid < K) {
            const uint32_t *h = sm.hist + sm.q_lead[tid] * 256;
            const uint32_t rank = sm.q_rank[tid];
            int lo = 0, hi = 255;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (h[mid] > rank) hi = mid; else lo = mid + 1;
            }
            sm.cent[tid] = half_from_key((sm.q_top[tid] << 8) | (uint32_t)lo);
        }
    }
    __syncthreads();

    switch (K) {
        case 2: lloyd_fast<G, 2>(a, i, sm, q, n_groups); break;
        case 4: lloyd_fast<G, 4>(a, i, sm, q, n_groups); break;
        case 8: lloyd_fast<G, 8>(a, i, sm, q, n_groups); break;
        default: lloyd_fast<G, 16>(a, i, sm, q, n_groups); break;
    }
    if (tid < CMPQ_KMAX) crow[tid] = tid < K ? sm.cent[tid] : INFINITY;
}

}  // namespace

bool kmeans_fast_eligible(const KmArgs &a, int dtype) {
    return dtype == CMPQ_F16 && a.ew == nullptr && a.d_out >= 4 && a.d_out % 4 == 0 &&
           a.ldw % 4 == 0 && reinterpret_cast<uintptr_t>(a.W) % 8 == 0 &&
           reinterpret_cast<uintptr_t>(a.codes) % 4 == 0 && a.d_out <= 32768;
}

int launch_kmeans_fast(const KmArgs &a, hipStream_t s) {
    // lanes needed at 32, 16, 8 or 4 weights per lane; the widest that still fills a wave
    const int64_t groups = a.d_out / 4;
    int G = 8;
    while (G > 1 && groups < (int64_t)G * 64) G >>= 1;
    int64_t T = cdiv(groups, G);
    T = cdiv(T, 64) * 64;
    if (T > 1024) return CMPQ_ESHAPE;
    const dim3 grid((unsigned)a.d_in), block((unsigned)T);
    switch (G) {
        case 8: kmeans_fast_kernel<8><<<grid, block, 0, s>>>(a); break;
        case 4: kmeans_fast_kernel<4><<<grid, block, 0, s>>>(a); break;
        case 2: kmeans_fast_kernel<2><<<grid, block, 0, s>>>(a); break;
        default: kmeans_fast_kernel<1><<<grid, block, 0, s>>>(a); break;
    }
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}
