// Bucket k-means for the common case of cmpq_kmeans_quantize: fp16 weights, unit
// importance (Sec. 3.2.1 of arXiv 2410.13056; entries of O_q removed as in Sec. 3.2.2).
//
// A Lloyd round on a line only needs, for each boundary between two neighbouring
// levels, how many weights lie below it and what they sum to.  The kernel arranges the
// channel once so that each round reads these numbers instead of recounting them:
//
//   * every weight becomes its 16-bit order key (unsigned order = value order); the top
//     10 bits name one of 1024 buckets, the low 6 bits the place inside it;
//   * one pass counts the buckets and sums the places, a scan turns this into exclusive
//     prefixes of the count and of the exact integer sum of x*2^24 (inside a bucket
//     x*2^24 is affine in the place: sign, exponent and top mantissa bits are shared);
//   * a second pass scatters the keys into an LDS array ordered by bucket (any order
//     inside a bucket);
//   * a round then costs, per boundary, the prefix of its bucket plus a scan of that one
//     bucket's keys (a wavefront per boundary), a cell is the difference of two
//     boundaries, and the new level is the exact integer sum divided in fp64 and rounded
//     once to fp32 - the value an fp64 reference computes;
//   * when no boundary moved the iteration has reached its fixed point and the remaining
//     rounds, which would repeat it, are skipped.
//
// All sums are integers, so the result is reproducible bit for bit and identical to the
// brute-force kernels.  Boundaries are exact: between distinct neighbouring levels
// lo < hi the boundary key is that of the largest fp16 value below the real midpoint (or
// equal to it when the tie rule gives the midpoint to lo).  Levels are ranked by (value,
// index) whenever their order may have changed; they need not stay ascending because a
// level without members keeps a stale value.
//
// The weights stay in registers as packed keys for the final coding (branch-free search
// over K-1 key boundaries).  A channel with NaN or infinity is flagged and left to the
// general kernel.
#include "kmeans_args.h"

namespace {

constexpr int kLowBits = 6;
constexpr int kBuckets = 1 << (16 - kLowBits);
constexpr int kLows = 1 << kLowBits;
constexpr uint32_t kKeyInf = 0xffffu;  // boundary above every key

struct BucketShared {
    long long scum[kBuckets + 1];   // exclusive prefix over buckets of sum(x * 2^24)
    uint32_t ncum[kBuckets + 1];    // counts, then their exclusive prefix
    uint32_t thr[CMPQ_KMAX];        // boundary keys by sorted position
    uint32_t part_n[CMPQ_KMAX];     // per boundary: kept weights of its bucket not above it
    uint32_t part_l[CMPQ_KMAX];     //               and the sum of their places
    float cent[CMPQ_KMAX];          // levels by level index
    int perm[CMPQ_KMAX];            // sorted position -> level index
    uint32_t scan32[17];
    unsigned long long scan64[17];
    int seg_lo, n_excl, identity, done;
};

__device__ __forceinline__ uint32_t key_of_half(uint32_t h) {
    return (h & 0x8000u) ? (~h & 0xffffu) : (h | 0x8000u);
}
__device__ __forceinline__ uint32_t half_of_key(uint32_t k) {
    return (k & 0x8000u) ? (k & 0x7fffu) : (~k & 0xffffu);
}
__device__ __forceinline__ float value_of_key(uint32_t k) {
    return __half2float(__ushort_as_half((unsigned short)half_of_key(k)));
}

// x*2^24 of the first key of bucket b, and the step per place inside the bucket.
__device__ __forceinline__ void bucket_affine(uint32_t b, long long &q0, long long &step) {
    const uint32_t key0 = b << kLowBits;
    const uint32_t e = (half_of_key(key0) >> 10) & 31u;
    step = 1ll << ((e > 1 ? e : 1) - 1);
    q0 = (long long)((double)value_of_key(key0) * 16777216.0);
}

__device__ __forceinline__ unsigned long long wave_scan_incl_u64(unsigned long long v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const unsigned long long t = __shfl_up(v, s, CMPQ_WAVE);
        if (lane >= s) v += t;
    }
    return v;
}

__device__ __forceinline__ unsigned long long block_scan_excl_u64(unsigned long long v,
                                                                  unsigned long long *scratch,
                                                                  unsigned long long *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwave = (blockDim.x + 63) >> 6;
    const unsigned long long incl = wave_scan_incl_u64(v);
    __syncthreads();
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const unsigned long long w = lane < nwave ? scratch[lane] : 0ull;
        const unsigned long long wi = wave_scan_incl_u64(w);
        if (lane < nwave) scratch[lane] = wi - w;
        if (lane == nwave - 1) scratch[16] = wi;
    }
    __syncthreads();
    *total = scratch[16];
    return scratch[wave] + incl - v;
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

// Key of the largest fp16 value that belongs to `lo` rather than `hi` (lo < hi): values
// below the midpoint, and the midpoint itself when lo has the smaller level index.
__device__ __forceinline__ uint32_t boundary_key(float lo, float hi, int owner_lo, int owner_hi) {
    const double mid = ((double)lo + (double)hi) * 0.5;
    float f = (float)mid;  // round down to fp32 ...
    if ((double)f > mid) {
        uint32_t u = __float_as_uint(f);
        if (f > 0.0f) u -= 1; else if (f == 0.0f) u = 0x80000001u; else u += 1;
        f = __uint_as_float(u);
    }
    uint32_t h = __half_as_ushort(__float2half_rn(f));  // ... then down to fp16
    if (h == 0x8000u) h = 0;                            // -0 is +0 here; checked below against f
    uint32_t key = key_of_half(h);
    if (value_of_key(key) > f) key -= 1;
    if ((double)value_of_key(key) == mid && owner_hi < owner_lo) key -= 1;
    return key;
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

template <int G>
__device__ __forceinline__ uint32_t elem_key(const uint32_t (&keys)[2 * G], int k, int e) {
    return (keys[2 * k + (e >> 1)] >> (16 * (e & 1))) & 0xffffu;
}

// One wavefront: among the keys arr[begin, end), how many are <= tk, and the sum of
// their places.  Result valid in every lane.
__device__ __forceinline__ void scan_bucket(const unsigned short *arr, uint32_t begin, uint32_t end,
                                            uint32_t tk, uint32_t &n, uint32_t &l) {
    const int lane = threadIdx.x & 63;
    uint32_t cn = 0, cl = 0;
    for (uint32_t j = begin + lane; j < end; j += 64) {
        const uint32_t key = arr[j];
        const bool in = key <= tk;
        cn += in;
        cl += in ? (key & (kLows - 1)) : 0u;
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) {
        cn += __shfl_xor(cn, s, CMPQ_WAVE);
        cl += __shfl_xor(cl, s, CMPQ_WAVE);
    }
    n = cn;
    l = cl;
}

template <int G, int K>
__device__ __forceinline__ void lloyd_bucket(const KmArgs &a, int64_t i, BucketShared &sm,
                                             const unsigned short *arr, uint32_t *fine,
                                             const uint32_t (&keys)[2 * G], int n_groups, uint32_t M) {
    const int T = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = T >> 6;

    // ---- start-up: level j = order statistic floor((2j+1)M/(2K)) of the kept weights.
    //      A wavefront per rank: locate the bucket by its prefix, count its 64 places.
    for (int j = wave; j < K; j += nw) {
        float c = 0.0f;
        if (M > 0) {
            const uint32_t r = (uint32_t)(((uint64_t)(2 * j + 1) * M) / (uint64_t)(2 * K));
            int lo = 0, hi_b = kBuckets - 1;  // largest b with ncum[b] <= r
            while (lo < hi_b) {
                const int mid = (lo + hi_b + 1) >> 1;
                if (sm.ncum[mid] <= r) lo = mid; else hi_b = mid - 1;
            }
            const uint32_t b = (uint32_t)lo, r_in = r - sm.ncum[lo];
            uint32_t *f = fine + wave * kLows;
            f[lane] = 0;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            for (uint32_t e = sm.ncum[b] + lane; e < sm.ncum[b + 1]; e += 64)
                atomicAdd(&f[arr[e] & (kLows - 1)], 1u);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            __builtin_amdgcn_wave_barrier();
            const uint32_t incl = wave_scan_incl_u32(f[lane]);
            // smallest place whose inclusive count exceeds the rank inside the bucket
            const unsigned long long over = __ballot(incl > r_in);
            const int place = __ffsll((long long)over) - 1;
            c = value_of_key((b << kLowBits) | (uint32_t)place);
        }
        if (lane == 0) sm.cent[j] = c;
    }
    __syncthreads();

    // ---- wave 0 state: lane p = sorted position p
    float c_sorted = INFINITY, hi = INFINITY;
    int own = lane, owner_lo = lane, owner_hi = 0;
    bool have_hi = false;
    uint32_t tk = kKeyInf, tk_prev = 0xffffffffu;
    if (wave == 0) {
        const float c = lane < K ? sm.cent[lane] : INFINITY;
        rank_levels<K>(c, c_sorted, own, hi, owner_lo, owner_hi, have_hi);
    }

    for (int round = 0;; ++round) {
        if (wave == 0) {
            tk = kKeyInf;
            if (have_hi) tk = boundary_key(c_sorted, hi, owner_lo, owner_hi);
            // no boundary moved: the iteration sits on its fixed point
            const unsigned long long moved = __ballot(lane < K - 1 && tk != tk_prev);
            tk_prev = tk;
            if (lane < K) {
                sm.thr[lane] = tk;
                sm.perm[lane] = own;
                sm.cent[own] = c_sorted;
            }
            const unsigned long long shuffled = __ballot(lane < K && own != lane);
            if (lane == 0) {
                sm.identity = shuffled == 0ull;
                sm.done = round == a.iters || moved == 0ull;
            }
        }
        __syncthreads();
        if (sm.done) break;
        // a wavefront per boundary: the part of its bucket that lies below it
        for (int p = wave; p < K - 1; p += nw) {
            const uint32_t t = sm.thr[p];
            uint32_t n = 0, l = 0;
            if (t != kKeyInf) {
                const uint32_t b = t >> kLowBits;
                scan_bucket(arr, sm.ncum[b], sm.ncum[b + 1], t, n, l);
            }
            if (lane == 0) {
                sm.part_n[p] = n;
                sm.part_l[p] = l;
            }
        }
        __syncthreads();
        if (wave == 0) {
            // cumulative count and sum at each boundary; the last position takes everything
            uint32_t n_below = M;
            long long s_below = sm.scum[kBuckets];
            if (lane < K - 1 && tk != kKeyInf) {
                const uint32_t b = tk >> kLowBits;
                const uint32_t cnt = sm.part_n[lane];
                long long q0, step;
                bucket_affine(b, q0, step);
                n_below = sm.ncum[b] + cnt;
                s_below = sm.scum[b] + (long long)cnt * q0 + step * (long long)sm.part_l[lane];
            }
            uint32_t n_prev = __shfl_up(n_below, 1, CMPQ_WAVE);
            long long s_prev = __shfl_up(s_below, 1, CMPQ_WAVE);
            if (lane == 0) {
                n_prev = 0;
                s_prev = 0;
            }
            const uint32_t n_cell = n_below - n_prev;
            const long long s_cell = s_below - s_prev;
            float c = c_sorted;
            if (lane < K && n_cell > 0)
                c = (float)(((double)s_cell * 5.9604644775390625e-08) / (double)n_cell);
            // usual case: the levels are still strictly ascending in the old order
            const float c_up = __shfl_down(c, 1, CMPQ_WAVE);
            const int own_up = __shfl_down(own, 1, CMPQ_WAVE);
            const unsigned long long bad = __ballot(lane < K - 1 && !(c < c_up));
            if (bad == 0ull) {
                c_sorted = c;
                hi = c_up;
                owner_lo = own;
                owner_hi = own_up;
                have_hi = lane < K - 1;
            } else {
                // bring the values back to level order and rank them again
                float c_level = INFINITY;
#pragma unroll
                for (int l = 0; l < K; ++l) {
                    const int ol = __shfl(own, l, CMPQ_WAVE);
                    const float cl = __shfl(c, l, CMPQ_WAVE);
                    if (ol == lane) c_level = cl;
                }
                rank_levels<K>(c_level, c_sorted, own, hi, owner_lo, owner_hi, have_hi);
            }
        }
    }

    // ---- final coding: 4 codes per lane and store
    uint32_t thr[CMPQ_KMAX];
#pragma unroll
    for (int p = 0; p < K - 1; ++p) thr[p] = sm.thr[p];
    uint32_t *crow = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
    const bool ident = sm.identity;
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        if (g < n_groups) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t pos = cell_of<K>(elem_key<G>(keys, k, e), thr);
                if (!ident) pos = (uint32_t)sm.perm[pos];
                word |= pos << (8 * e);
            }
            crow[g] = word;
        }
    }
}

template <int G, int TMAX>
__global__ __launch_bounds__(TMAX) void kmeans_bucket_kernel(KmArgs a) {
    // dynamic LDS: keys ordered by bucket | removed-entry bitmap (one bit per weight) |
    // a table used three times in a row: per-bucket sums of places, then the scatter
    // cursors, then one 64-entry table per wavefront for the start-up
    extern __shared__ __align__(16) unsigned char dyn[];
    __shared__ BucketShared sm;
    const int64_t i = blockIdx.x;
    const int T = blockDim.x, tid = threadIdx.x;
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
    unsigned short *arr = reinterpret_cast<unsigned short *>(dyn);
    uint32_t *removed = reinterpret_cast<uint32_t *>(dyn + (((size_t)d_out * 2 + 15) & ~(size_t)15));
    const int n_words = (d_out + 31) >> 5;
    uint32_t *fine = removed + ((n_words + 3) & ~3);
    uint32_t *lsum = fine;

    // ---- load: lane owns groups g = k*T + tid of 4 weights, kept as packed 16-bit keys
    const uint2 *wrow = reinterpret_cast<const uint2 *>(static_cast<const __half *>(a.W) + i * a.ldw);
    uint32_t keys[2 * G];
    int finite = 1;
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        uint2 raw = make_uint2(0, 0);
        if (g < n_groups) raw = wrow[g];
        uint32_t h[4] = {raw.x & 0xffffu, raw.x >> 16, raw.y & 0xffffu, raw.y >> 16};
        uint32_t ky[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            finite &= (h[e] & 0x7c00u) != 0x7c00u;
            if (h[e] == 0x8000u) h[e] = 0;  // -0 reads as +0
            ky[e] = key_of_half(h[e]);
        }
        keys[2 * k] = ky[0] | (ky[1] << 16);
        keys[2 * k + 1] = ky[2] | (ky[3] << 16);
    }
    if (tid == 0) {  // the slice of out_idx inside this channel
        const int64_t first = i * a.d_out, last = first + a.d_out;
        int64_t lo = 0, hi = a.n_out;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.out_idx[mid] < first) lo = mid + 1; else hi = mid;
        }
        sm.seg_lo = (int)lo;
        hi = a.n_out;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.out_idx[mid] < last) lo = mid + 1; else hi = mid;
        }
        sm.n_excl = (int)lo - sm.seg_lo;
    }
    for (int s = tid; s <= kBuckets; s += T) sm.ncum[s] = 0;
    for (int s = tid; s < kBuckets; s += T) lsum[s] = 0;
    for (int s = tid; s < n_words; s += T) removed[s] = 0;
    if (!__syncthreads_and(finite)) {  // leave the channel to the general kernel
        if (tid == 0) a.deferred[i] = 1;
        return;
    }
    if (tid == 0) a.deferred[i] = 0;
    const int n_ex = sm.n_excl;
    const int32_t *ex_idx = a.out_idx + sm.seg_lo;
    const int32_t chan_base = (int32_t)(i * a.d_out);
    for (int e = tid; e < n_ex; e += T) {  // entries of O_q do not take part in the clustering
        const int o = ex_idx[e] - chan_base;
        atomicOr(&removed[o >> 5], 1u << (o & 31));
    }
    __syncthreads();

    // ---- bucket tables: counts and sums of places of the kept weights
    uint32_t kept[G];  // 4 bits per group: which of its weights are kept
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        kept[k] = 0;
        if (g < n_groups) {
            kept[k] = ~(removed[g >> 3] >> ((g & 7) * 4)) & 0xfu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if ((kept[k] >> e) & 1u) {
                    const uint32_t key = elem_key<G>(keys, k, e);
                    atomicAdd(&sm.ncum[key >> kLowBits], 1u);
                    atomicAdd(&lsum[key >> kLowBits], key & (kLows - 1));
                }
            }
        }
    }
    __syncthreads();
    // ---- exclusive prefixes over buckets of count and exact sum; scatter cursors
    {
        const int per = kBuckets / T > 0 ? kBuckets / T : 1;  // T is a power of two <= 1024
        const int b0 = tid * per;
        uint32_t n_loc = 0;
        long long s_loc = 0;
        if (b0 < kBuckets) {
            for (int r = 0; r < per; ++r) {
                const uint32_t n = sm.ncum[b0 + r];
                long long q0, step;
                bucket_affine((uint32_t)(b0 + r), q0, step);
                n_loc += n;
                s_loc += (long long)n * q0 + step * (long long)lsum[b0 + r];
            }
        }
        uint32_t n_tot;
        unsigned long long s_tot;
        uint32_t n_run = block_scan_excl_u32(n_loc, sm.scan32, &n_tot);
        long long s_run = (long long)block_scan_excl_u64((unsigned long long)s_loc, sm.scan64, &s_tot);
        if (b0 < kBuckets) {
            for (int r = 0; r < per; ++r) {
                const uint32_t n = sm.ncum[b0 + r];
                long long q0, step;
                bucket_affine((uint32_t)(b0 + r), q0, step);
                const long long sb = (long long)n * q0 + step * (long long)lsum[b0 + r];
                sm.ncum[b0 + r] = n_run;
                lsum[b0 + r] = n_run;  // from here on: where the next key of the bucket goes
                sm.scum[b0 + r] = s_run;
                n_run += n;
                s_run += sb;
            }
        }
        if (tid == 0) {
            sm.ncum[kBuckets] = n_tot;
            sm.scum[kBuckets] = (long long)s_tot;
        }
    }
    __syncthreads();
    const uint32_t M = sm.ncum[kBuckets];
    // ---- scatter the kept keys, ordered by bucket
#pragma unroll
    for (int k = 0; k < G; ++k) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if ((kept[k] >> e) & 1u) {
                const uint32_t key = elem_key<G>(keys, k, e);
                const uint32_t pos = atomicAdd(&lsum[key >> kLowBits], 1u);
                arr[pos] = (unsigned short)key;
            }
        }
    }
    __syncthreads();

    switch (K) {
        case 2: lloyd_bucket<G, 2>(a, i, sm, arr, fine, keys, n_groups, M); break;
        case 4: lloyd_bucket<G, 4>(a, i, sm, arr, fine, keys, n_groups, M); break;
        case 8: lloyd_bucket<G, 8>(a, i, sm, arr, fine, keys, n_groups, M); break;
        default: lloyd_bucket<G, 16>(a, i, sm, arr, fine, keys, n_groups, M); break;
    }
    if (tid < CMPQ_KMAX) crow[tid] = tid < K ? sm.cent[tid] : INFINITY;
}

size_t bucket_dyn_lds(int64_t d_out, int64_t T) {
    size_t b = ((size_t)d_out * 2 + 15) & ~(size_t)15;
    b += (size_t)((((d_out + 31) >> 5) + 3) & ~3) * 4;
    const size_t table = (size_t)(T / 64) * kLows;
    b += (table > (size_t)kBuckets ? table : (size_t)kBuckets) * 4;
    return b;
}

template <int G, int TMAX>
int launch_variant(const KmArgs &a, int64_t T, hipStream_t s) {
    auto kern = kmeans_bucket_kernel<G, TMAX>;
    const size_t lds = bucket_dyn_lds(a.d_out, T);
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return CMPQ_EHIP;
    }
    kern<<<dim3((unsigned)a.d_in), dim3((unsigned)T), lds, s>>>(a);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

int launch_kmeans_hist(const KmArgs &a, hipStream_t s) {
    // a power-of-two workgroup with at most 32 weights per lane
    const int64_t groups = a.d_out / 4;
    int64_t T = 64;
    while (T < 1024 && T * 8 < groups) T <<= 1;
    if (T * 8 < groups) return CMPQ_ESHAPE;
    const int64_t per_lane = cdiv(groups, T);
    if (per_lane > 4) {
        if (T > 256) return launch_variant<8, 1024>(a, T, s);
        return launch_variant<8, 256>(a, T, s);
    }
    if (per_lane > 2) return launch_variant<4, 64>(a, T, s);
    if (per_lane > 1) return launch_variant<2, 64>(a, T, s);
    return launch_variant<1, 64>(a, T, s);
}
