// Bucket k-means for the common case of cmpq_kmeans_quantize: fp16 weights, unit
// importance (Sec. 3.2.1 of arXiv 2410.13056; entries of O_q removed as in Sec. 3.2.2).
//
// A Lloyd round on a line only needs, for each boundary between two neighbouring
// levels, how many weights lie below it and what they sum to.  The kernel arranges the
// channel once so that each round reads these numbers instead of recounting them:
//
//   * every weight becomes its 16-bit order key (unsigned order = value order); the top
//     bits name a bucket (1024 buckets of 64 places, or 512 of 128 for short channels),
//     the low bits the place inside it;
//   * one pass counts the buckets and sums the places, a scan turns this into exclusive
//     prefixes of the count and of the exact integer sum of x*2^24 (inside a bucket
//     x*2^24 is affine in the place: sign, exponent and top mantissa bits are shared);
//   * a second pass scatters the places into an LDS byte array ordered by bucket (any
//     order inside a bucket); a bucket's stretch starts on a 4-byte boundary and its
//     unused tail holds a filler above every place, so a scan reads whole words;
//   * a round then costs, per boundary, the prefix of its bucket plus a scan of that one
//     bucket (a group of lanes per boundary, four places per word compared at once), a
//     cell is the difference of two boundaries, and the new level is the exact integer sum
//     divided in fp64 and rounded once to fp32 - the value an fp64 reference computes;
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
// The kernel is bound by instruction issue, not by latency: the serial part of a round
// runs on one wavefront while the others sleep at barriers, and several workgroups share
// a compute unit.  A channel with NaN or infinity raises the status flag and gets levels 0
// and codes 0.
#include <type_traits>

#include "kmeans_args.h"
#include "kmeans_keys.h"

namespace {

// Bytes of the place array: one per weight plus up to 3 of filler per non-empty bucket.
__host__ __device__ inline size_t bucket_arr_bytes(int64_t d_out, int lb) {
    const int64_t buckets = (int64_t)1 << (16 - lb);
    const int64_t pad = 3 * (d_out < buckets ? d_out : buckets);
    return ((size_t)(d_out + pad) + 15) & ~(size_t)15;
}

template <int LB>
struct BucketShared {
    static constexpr int kBuckets = 1 << (16 - LB);
    long long scum[kBuckets + 1];   // count << 32 | sum of places; then the exclusive prefix
                                    // over buckets of sum(x * 2^24)
    uint16_t ncum[kBuckets + 2];    // exclusive prefix over buckets of the counts
    uint16_t start[kBuckets + 2];   // where a bucket's stretch of the byte array begins
    uint32_t part_n[2][CMPQ_KMAX];  // by round parity, per boundary: kept weights of its bucket
    uint32_t part_l[2][CMPQ_KMAX];  //   not above it, and the sum of their places
    float cent[CMPQ_KMAX];          // levels by level index
    uint32_t tk[2][CMPQ_KMAX];      // by round parity: boundary keys by sorted position
    uint32_t code_of[CMPQ_KMAX];    // level index that each sorted position stands for
    int go[2];                      // by round parity: another round follows
    uint32_t scan32[17];
    unsigned long long scan64[17];
    int seg_lo, n_excl;
    double cent64[CMPQ_KMAX];       // final levels by level index, as the error sum reads them
};

// Two order keys in one word -> the two fp16 patterns they stand for (inverse of keys_of_half2).
__device__ __forceinline__ uint32_t halves_of_keys2(uint32_t kk) {
    const uint32_t pos = (kk >> 15) & 0x00010001u;  // key of a non-negative value: only the sign bit was flipped
    return kk ^ (0xffffffffu ^ __umul24(pos, 0x7fffu));
}

template <int G>
__device__ __forceinline__ uint32_t elem_key(const uint32_t (&keys)[2 * G], int k, int e) {
    return (keys[2 * k + (e >> 1)] >> (16 * (e & 1))) & 0xffffu;
}

// A group of L lanes: among the places of one bucket, arr[begin, end) with begin and end
// multiples of 4 and filler in the unused tail, how many are <= pl, and their sum (U words
// per lane in flight).  Four places per word are compared at once: a byte plus (127 - pl) reaches bit 7 exactly when
// it is above pl (places and pl are at most 127, the filler is 128: no carry leaves a
// byte).  The inverted bits 7 are counted, and a dot product of the word's bytes with them
// gives 128 times the sum of the places they mark (below 2^32 for any channel: at most
// 32 768 places of at most 127).  Result valid in every lane of the group.
template <int L, int U = 4>
__device__ __forceinline__ void scan_bucket(const unsigned char *arr, uint32_t begin, uint32_t end,
                                            uint32_t pl, uint32_t &n, uint32_t &l) {
    const int sub = threadIdx.x & (L - 1);
    const uint32_t *words = reinterpret_cast<const uint32_t *>(arr);
    const uint32_t w_end = end >> 2;
    const uint32_t bias = 0x7f7f7f7fu - pl * 0x01010101u;
    uint32_t cn = 0, cl7 = 0;
    for (uint32_t j = (begin >> 2) + sub; j < w_end; j += U * L) {  // U reads in flight
        uint32_t x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = j + u * L < w_end ? words[j + u * L] : kFill4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t le7 = ~(x[u] + bias) & 0x80808080u;  // bit 7 per byte <= pl
            cn += (uint32_t)__builtin_popcount(le7);
            cl7 = __builtin_amdgcn_udot4(x[u], le7, cl7, false);
        }
    }
    n = group_sum<L>(cn);
    l = group_sum<L>(cl7) >> 7;
}

// Counts the buckets and sums the places of the kept weights (packed 64-bit LDS atomics).
template <int G, int T, int LB, bool MASKED>
__device__ __forceinline__ void count_buckets(const uint32_t (&keys)[2 * G], const uint32_t *removed,
                                              long long *scum, int n_groups) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        if (g < n_groups) {
            uint32_t kept = 0xfu;  // 4 bits of the bitmap per group of 4 weights
            if constexpr (MASKED) kept = ~(removed[g >> 3] >> ((g & 7) * 4)) & 0xfu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (!MASKED || ((kept >> e) & 1u)) {
                    const uint32_t key = elem_key<G>(keys, k, e);
                    atomicAdd(reinterpret_cast<unsigned long long *>(&scum[key >> LB]),
                              (1ull << 32) | (key & ((1u << LB) - 1)));
                }
            }
        }
    }
}

// Puts the place of every kept weight into its bucket's stretch of the byte array.
template <int G, int T, int LB, bool MASKED>
__device__ __forceinline__ void scatter_places(const uint32_t (&keys)[2 * G], const uint32_t *removed,
                                               uint32_t *cursor, unsigned char *arr, int n_groups) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int g = k * T + tid;
        if (g < n_groups) {
            uint32_t kept = 0xfu;
            if constexpr (MASKED) kept = ~(removed[g >> 3] >> ((g & 7) * 4)) & 0xfu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (!MASKED || ((kept >> e) & 1u)) {
                    const uint32_t key = elem_key<G>(keys, k, e);
                    const uint32_t pos = atomicAdd(&cursor[key >> LB], 1u);
                    arr[pos] = (unsigned char)(key & ((1u << LB) - 1));
                }
            }
        }
    }
}

// The coding table over the buckets (many levels, long channels): a bucket with no boundary
// inside has one code; with one boundary, a code on either side of it; with more (rare) the
// entry sends the weight to the search.  An entry: byte 0 the code at or below the boundary,
// byte 1 the low byte of the boundary's key (0xff: nothing lies above it), byte 2 the code
// above it, bit 24 the flag for more than one boundary.  A key and a boundary of the same
// bucket share all bits above the place, so their low bytes compare like their places.
constexpr uint32_t kTblMulti = 0x1000000u;

template <int K, int T, int LB>
__device__ __forceinline__ int build_code_table(const uint32_t (&thr)[CMPQ_KMAX], const uint32_t *code_of,
                                                const uint32_t *tk, uint32_t *tbl) {
    constexpr int kLows = 1 << LB, kBuckets = 1 << (16 - LB);
    int multi = 0;
    for (int bk = threadIdx.x; bk < kBuckets; bk += T) {
        const uint32_t first = (uint32_t)bk << LB;
        const uint32_t p0 = cell_of<K>(first, thr), p1 = cell_of<K>(first + kLows - 1, thr);
        uint32_t ent = code_of[p0] | (code_of[p1] << 16);
        if (p1 == p0) {
            ent |= 0xff00u;
        } else {
            ent |= (tk[p0] & 0xffu) << 8;
            if (p1 > p0 + 1) {
                ent |= kTblMulti;
                multi = 1;
            }
        }
        tbl[bk] = ent;
    }
    return multi;
}

// (v << 2) + base in one instruction (the compiler's own form of extract-shift-add is a
// shift, a mask and an add); base is the same in every lane.
__device__ __forceinline__ uint32_t shl2_add(uint32_t v, uint32_t base) {
    uint32_t r;
    asm("v_lshl_add_u32 %0, %1, 2, %2" : "=v"(r) : "v"(v), "s"(base));
    return r;
}

// LDS address (byte offset inside the workgroup's LDS) of a pointer into shared memory.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)reinterpret_cast<uintptr_t>(p);
}

// The table entry of the key in half `half` (0: low, 1: high) of the packed pair kk; the
// table starts at LDS address tbl_at.
template <int LB>
__device__ __forceinline__ uint32_t table_entry(uint32_t tbl_at, uint32_t kk, int half) {
    typedef const uint32_t __attribute__((address_space(3))) *LdsWord;
    const uint32_t bucket = __builtin_amdgcn_ubfe(kk, 16 * half + LB, 16 - LB);
    return *(LdsWord)(uintptr_t)shl2_add(bucket, tbl_at);
}

// The code that entry `ent` gives the same key (when its flag for several boundaries is clear).
__device__ __forceinline__ uint32_t code_from_entry(uint32_t ent, uint32_t kk, int half) {
    const uint32_t low = (kk >> (16 * half)) & 0xffu;
    return low > ((ent >> 8) & 0xffu) ? (ent >> 16) & 0xffu : ent & 0xffu;
}

// The coding pass with the stored format and the error folded in (Sec. 5.1; App. B.3): every
// lane takes groups g = tid, tid + T, ... of 4 weights (fetched again: the place array cannot
// give a weight's position back), finds their codes, adds (w - level)^2 in fp64 - nothing for an
// entry of O_q, whose FP16 weight is restored - and puts the group's 4 * B code bits into the
// channel's row of the bit stream, which is built in the place array the rounds no longer need.
// A rolled loop: its fp64 temporaries would not fit the register budget of the unrolled one.
// Returns the lane's share of the error.  Contains a barrier: called by all threads.
template <int G, int K, int T, int LB>
__device__ __forceinline__ double coding_pass_fused(const KmArgs &a, int64_t i, BucketShared<LB> &sm,
                                                    unsigned char *arr, uint32_t *tbl, const uint32_t *removed,
                                                    int n_ex, int n_groups, int par) {
    constexpr int kLowBits = LB, kLows = 1 << LB, kBuckets = 1 << (16 - LB);
    constexpr int B = K == 2 ? 1 : (K == 4 ? 2 : (K == 8 ? 3 : 4));
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t tk_fin = sm.tk[par][lane & (CMPQ_KMAX - 1)];
    uint32_t thr[CMPQ_KMAX];
#pragma unroll
    for (int p = 0; p < K - 1; ++p) thr[p] = (uint32_t)__builtin_amdgcn_readlane((int)tk_fin, p);
    if (tid < CMPQ_KMAX) sm.cent64[tid] = (double)sm.cent[tid];
    // bytes of the row that the groups below do not write: zero, up to whole words
    const int row_bytes = (int)(((int64_t)a.d_out * B + 31) / 32) * 4;
    const int coded = B == 4 ? 2 * n_groups : (B == 2 ? n_groups : (B == 3 ? 3 * ((n_groups + 1) >> 1) : (n_groups + 1) >> 1));
    for (int x = coded + tid; x < row_bytes; x += T) arr[x] = 0;
    // a table over the buckets replaces the search where there are many levels
    constexpr bool kTable = K >= 8 && G * T >= 2 * kBuckets;  // worth it for long channels only
    int multi = 0;
    if constexpr (kTable) multi = build_code_table<K, T, LB>(thr, sm.code_of, sm.tk[par], tbl);
    const bool any_multi = __syncthreads_or(multi) != 0;  // also the barrier before the groups below
    const uint32_t tbl_at = lds_address(tbl);
    const uint2 *wrow = reinterpret_cast<const uint2 *>(static_cast<const __half *>(a.W) + i * a.ldw);
    uint32_t *crow = a.codes ? reinterpret_cast<uint32_t *>(a.codes + i * a.d_out) : nullptr;
    double err = 0.0;
    const int n_steps = (n_groups + T - 1) / T;  // the same for every lane: the neighbour exchange below needs all of them
    // the weights of the next few groups are fetched while the current ones are worked on: this
    // pass may be the first to touch the row (when the tables came from an earlier run)
    constexpr int kAhead = 4;
    // two copies of the loop: only a channel that has a bucket with several boundaries (rare)
    // pays for looking at each entry's flag
    auto all_groups = [&](auto with_search) {
    constexpr bool kSearch = decltype(with_search)::value;
    uint2 nxt[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
        const int g = u * T + tid;
        nxt[u] = g < n_groups ? wrow[g] : make_uint2(0, 0);
    }
#pragma unroll 1
    for (int step0 = 0; step0 < n_steps; step0 += kAhead) {
        uint2 chunk[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            chunk[u] = nxt[u];
            const int gn = (step0 + kAhead + u) * T + tid;
            nxt[u] = gn < n_groups ? wrow[gn] : make_uint2(0, 0);
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (step0 + u >= n_steps) break;  // uniform over the workgroup
            const int g = (step0 + u) * T + tid;
            const bool in = g < n_groups;
            const uint2 cur = chunk[u];
            const uint32_t kk[2] = {keys_of_half2(cur.x), keys_of_half2(cur.y)};
            uint32_t code[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (kTable) {
                    const uint32_t ent = table_entry<LB>(tbl_at, kk[e >> 1], e & 1);
                    code[e] = code_from_entry(ent, kk[e >> 1], e & 1);
                    if (kSearch && (ent & kTblMulti))
                        code[e] = sm.code_of[cell_of<K>((kk[e >> 1] >> (16 * (e & 1))) & 0xffffu, thr)];
                } else {
                    code[e] = sm.code_of[cell_of<K>((kk[e >> 1] >> (16 * (e & 1))) & 0xffffu, thr)];
                }
            }
            const uint32_t word = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);  // one code per byte
            if (in && crow) crow[g] = word;
            // (w - level)^2 of the four entries; an entry of O_q (restored to its FP16 weight) and a
            // lane past the end add an exact zero: their difference is masked bit by bit
            uint32_t kept = in ? 0xfu : 0u;
            if (n_ex > 0 && in) kept = ~(removed[g >> 3] >> ((g & 7) * 4)) & 0xfu;
            const uint32_t hw[2] = {cur.x, cur.y};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float w = __half2float(__ushort_as_half((unsigned short)(hw[e >> 1] >> (16 * (e & 1)))));
                const double d = (double)w - sm.cent64[code[e]];
                const uint32_t m = (uint32_t)__builtin_amdgcn_sbfe((int)kept, e, 1);  // all ones or zero
                const unsigned long long db = (unsigned long long)__double_as_longlong(d);
                const double dm = __longlong_as_double((long long)(((unsigned long long)(m & (uint32_t)(db >> 32)) << 32) |
                                                                   (m & (uint32_t)db)));
                err = fma(dm, dm, err);
            }
            const uint32_t f = in ? squeeze4<B>(word) : 0u;
            if constexpr (B == 4) {
                if (in) reinterpret_cast<uint16_t *>(arr)[g] = (uint16_t)f;
            } else if constexpr (B == 2) {
                if (in) arr[g] = (unsigned char)f;
            } else {
                // 12 (4) bits: an even lane joins its own with those of the lane above it (the next
                // group: T is even, so a lane's groups keep its parity) into 3 (1) whole bytes
                const uint32_t v = f | (row_from_above(f) << (4 * B));
                if (in && (tid & 1) == 0) {
                    if constexpr (B == 3) {
                        unsigned char *dst = arr + 3 * (g >> 1);
                        dst[0] = (unsigned char)v;
                        dst[1] = (unsigned char)(v >> 8);
                        dst[2] = (unsigned char)(v >> 16);
                    } else {
                        arr[g >> 1] = (unsigned char)v;
                    }
                }
            }
        }
    }
    };
    if (any_multi) all_groups(std::true_type{});
    else all_groups(std::false_type{});
    __syncthreads();
    return err;
}

template <int G, int K, int T, int LB, bool FUSED>
__device__ __forceinline__ void lloyd_bucket(const KmArgs &a, int64_t i, BucketShared<LB> &sm,
                                             unsigned char *arr, uint32_t *tbl, const uint32_t *removed, int n_ex,
                                             const uint32_t (&keys)[2 * G], int n_groups, uint32_t M,
                                             double &err_out) {
    constexpr int L = T / 16;  // lanes that share one boundary in a round
    constexpr int kLowBits = LB, kLows = 1 << LB, kBuckets = 1 << (16 - LB);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Start-up and rounds are a chain of short dependent steps (half the lifetime of a
    // workgroup): they go first at instruction issue, ahead of the wide, latency-tolerant
    // passes of the other workgroups on the compute unit.
    __builtin_amdgcn_s_setprio(3);
    // ---- start-up: level j = order statistic floor((2j+1)M/(2K)) of the kept weights.
    //      L lanes per rank: locate the bucket by its prefix, then bisect on the place
    //      with counting scans of that bucket.  Not when the caller gave the levels: they
    //      are in place already.
    if (!a.start_given) {
        const int j = tid / L, sub = tid & (L - 1);
        if (j < K) {
            float c = 0.0f;
            if (M > 0) {
                const uint32_t r = (uint32_t)(((uint64_t)(2 * j + 1) * M) / (uint64_t)(2 * K));
                const int g0 = lane & ~(L - 1);  // first lane of this group inside its wavefront
                // largest b with ncum[b] <= r: the L lanes probe L evenly spaced buckets at a time
                // (ncum does not decrease, so the probes that pass come first)
                int lo = 0, hi_b = kBuckets - 1;
                while (lo < hi_b) {
                    const int step = (hi_b - lo + L - 1) / L;
                    const int probe = min(lo + (sub + 1) * step, hi_b);
                    const unsigned long long pass = __ballot(sm.ncum[probe] <= r) >> g0;
                    const int c_pass = __popcll(L < 64 ? pass & ((1ull << L) - 1) : pass);
                    const int nlo = c_pass > 0 ? min(lo + c_pass * step, hi_b) : lo;
                    if (c_pass < L) hi_b = min(lo + (c_pass + 1) * step, hi_b) - 1;
                    lo = nlo;
                }
                const uint32_t b = (uint32_t)lo, r_in = r - sm.ncum[b];
                const uint32_t begin = sm.start[b], end = sm.start[b + 1];
                // smallest place with more than r_in weights at or below it: bisection on the place.
                // The bucket's words are fetched once (4 per lane) when they fit; the counting
                // scans of the bisection then run on registers.
                const uint32_t w_begin = begin >> 2, w_end = end >> 2;
                const bool fits = w_end - w_begin <= 4u * L;
                const uint32_t *words = reinterpret_cast<const uint32_t *>(arr);
                uint32_t x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t at = w_begin + sub + u * L;
                    x[u] = at < w_end ? words[at] : kFill4;
                }
                int pl = 0, ph = kLows - 1;
                while (pl < ph) {
                    const int mid = (pl + ph) >> 1;
                    uint32_t n, l;
                    if (fits) {
                        const uint32_t bias = 0x7f7f7f7fu - (uint32_t)mid * 0x01010101u;
                        uint32_t cn = 0;
#pragma unroll
                        for (int u = 0; u < 4; ++u) cn += (uint32_t)__builtin_popcount(~(x[u] + bias) & 0x80808080u);
                        n = group_sum<L>(cn);
                    } else {
                        scan_bucket<L>(arr, begin, end, (uint32_t)mid, n, l);
                    }
                    if (n > r_in) ph = mid; else pl = mid + 1;
                }
                c = value_of_key((b << kLowBits) | (uint32_t)pl);
                if (c == 0.0f) c = 0.0f;  // a level never starts as -0
            }
            if (sub == 0) sm.cent[j] = c;
        }
    }
    __syncthreads();

    // ---- rounds.  Wavefront 0 alone carries the levels (lane p = sorted position p) and
    //      does the serial part of a round; the others only join in the per-boundary bucket
    //      scans and otherwise sleep at the two barriers, leaving the issue slots to the
    //      other workgroups of the compute unit.
    float c_sorted = 0.0f, hi = 0.0f;
    int own = lane, owner_lo = 0, owner_hi = 0;
    bool have_hi = false;
    if (wave == 0) {
        // starting levels that ascend strictly (the usual outcome of the quantile start) are
        // in sorted order already: each level's upper neighbour sits one lane up
        const float c0 = lane < K ? sm.cent[lane] : INFINITY;
        const float c0_up = __uint_as_float(row_from_above(__float_as_uint(c0)));
        if (__ballot(lane < K - 1 && !(c0 < c0_up)) == 0ull) {
            c_sorted = c0;
            hi = c0_up;
            owner_lo = lane;
            owner_hi = lane + 1;
            have_hi = lane < K - 1;
        } else {
            rank_levels<K>(c0, c_sorted, own, hi, owner_lo, owner_hi, have_hi);
        }
    }
    uint32_t tk_prev = 0xffffffffu;
    // lanes per boundary in the rounds, and words each of them has in flight: the 512-lane
    // workgroups give a boundary 16 lanes with 8 words (fewer wavefronts then execute the scan;
    // measured 2 % faster there, 3 % slower for 256 lanes)
    constexpr int LR = T >= 512 ? T / 32 : L;
    constexpr int UR = 4 * (L / LR);
    const int p_mine = tid / LR;  // the boundary this lane helps with
    int par = 0;

    for (int round = 0;; ++round) {
        par = round & 1;
        if (wave == 0) {
            uint32_t tk = kKeyInf;
            if (have_hi) tk = boundary_key(c_sorted, hi, owner_lo, owner_hi);
            // no boundary moved: the iteration sits on its fixed point
            const bool moved = __ballot(lane < K - 1 && tk != tk_prev) != 0ull;
            tk_prev = tk;
            const bool go = round != a.iters && moved;
            if (lane < CMPQ_KMAX) sm.tk[par][lane] = tk;
            if (lane == 0) sm.go[par] = go;
            if (!go) {  // results: the position -> level map and the levels by level index
                if (lane < CMPQ_KMAX) sm.code_of[lane] = (uint32_t)own;
                if (lane < K) sm.cent[own] = c_sorted;
            }
        }
        __syncthreads();
        if (!sm.go[par]) break;
        // L lanes per boundary: the part of its bucket that lies below it
        if (p_mine < K - 1) {
            const uint32_t t = sm.tk[par][p_mine];
            uint32_t n = 0, l = 0;
            if (t != kKeyInf) {
                const uint32_t b = t >> kLowBits;
                scan_bucket<LR, UR>(arr, sm.start[b], sm.start[b + 1], t & (kLows - 1), n, l);
            }
            if ((tid & (LR - 1)) == 0) {
                sm.part_n[par][p_mine] = n;
                sm.part_l[par][p_mine] = l;
            }
        }
        __syncthreads();
        if (wave != 0) continue;
        // cumulative count and sum at each boundary; the last position takes everything
        const uint32_t tk = tk_prev;
        uint32_t n_below = M;
        long long s_below = sm.scum[kBuckets];
        if (lane < K - 1 && tk != kKeyInf) {
            const uint32_t b = tk >> kLowBits;
            const uint32_t cnt = sm.part_n[par][lane];
            n_below = sm.ncum[b] + cnt;
            s_below = sm.scum[b] + bucket_sum<LB>(b, cnt, sm.part_l[par][lane]);
        }
        // sorted positions live in lanes 0..15, one DPP row: neighbours come by row shifts
        const uint32_t n_prev = row_from_below(n_below);
        const long long s_prev = (long long)(((unsigned long long)row_from_below((uint32_t)((unsigned long long)s_below >> 32)) << 32) |
                                             row_from_below((uint32_t)s_below));
        const uint32_t n_cell = n_below - n_prev;
        const long long s_cell = s_below - s_prev;
        float c = c_sorted;
        if (lane < K && n_cell > 0)
            c = (float)(((double)s_cell * 5.9604644775390625e-08) / (double)n_cell);
        // usual case: the levels are still strictly ascending in the old order
        const float c_up = __uint_as_float(row_from_above(__float_as_uint(c)));
        const int own_up = (int)row_from_above((uint32_t)own);
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

    __builtin_amdgcn_s_setprio(0);
    if constexpr (FUSED) {
        err_out = coding_pass_fused<G, K, T, LB>(a, i, sm, arr, tbl, removed, n_ex, n_groups, par);
        return;
    }
    if (!a.codes) {  // the caller wants the levels alone
        __syncthreads();
        return;
    }
    // ---- final coding: 4 codes per lane and store.  Every wavefront fetches the final
    //      boundaries and the position -> level map left by wavefront 0.
    const uint32_t tk_fin = sm.tk[par][lane & (CMPQ_KMAX - 1)];
    const int own_fin = (int)sm.code_of[lane & (CMPQ_KMAX - 1)];
    uint32_t thr[CMPQ_KMAX];
#pragma unroll
    for (int p = 0; p < K - 1; ++p) thr[p] = (uint32_t)__builtin_amdgcn_readlane((int)tk_fin, p);
    uint32_t *crow = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
    // Workgroups of 512 lanes fetch their weights again here (from cache) instead of holding
    // them in registers through the rounds: a third workgroup then fits a compute unit.
    constexpr bool kReload = T >= 512;
    uint32_t again[2 * G];
    if constexpr (kReload) {
        const uint2 *wrow = reinterpret_cast<const uint2 *>(static_cast<const __half *>(a.W) + i * a.ldw);
#pragma unroll
        for (int k = 0; k < G; ++k) {
            const int g = k * T + tid;
            uint2 raw = make_uint2(0, 0);
            if (g < n_groups) raw = wrow[g];
            again[2 * k] = keys_of_half2(raw.x);
            again[2 * k + 1] = keys_of_half2(raw.y);
        }
    }
    auto key_at = [&](int k, int e) -> uint32_t {
        if constexpr (kReload) return elem_key<G>(again, k, e);
        else return elem_key<G>(keys, k, e);
    };
    // Many weights per lane and many levels: a table over the buckets replaces the search.
    constexpr bool kTable = K >= 8 && G * T >= 2 * kBuckets;
    if constexpr (kTable) {
        const int multi = build_code_table<K, T, LB>(thr, sm.code_of, sm.tk[par], tbl);
        const uint32_t tbl_at = lds_address(tbl);
        auto pair_at = [&](int k, int e) -> uint32_t {
            if constexpr (kReload) return again[2 * k + (e >> 1)];
            else return keys[2 * k + (e >> 1)];
        };
        if (!__syncthreads_or(multi)) {
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const int g = k * T + tid;
                uint32_t word = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t kk = pair_at(k, e);
                    word |= code_from_entry(table_entry<LB>(tbl_at, kk, e & 1), kk, e & 1) << (8 * e);
                }
                if (g < n_groups) crow[g] = word;
            }
        } else {
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const int g = k * T + tid;
                uint32_t word = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t kk = pair_at(k, e);
                    const uint32_t ent = table_entry<LB>(tbl_at, kk, e & 1);
                    uint32_t code = code_from_entry(ent, kk, e & 1);
                    if (ent & kTblMulti) code = sm.code_of[cell_of<K>(key_at(k, e), thr)];
                    word |= code << (8 * e);
                }
                if (g < n_groups) crow[g] = word;
            }
        }
    } else {
        const bool ident = __ballot(lane < K && own_fin != lane) == 0ull;
#pragma unroll
        for (int k = 0; k < G; ++k) {
            const int g = k * T + tid;
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {  // all lanes take part: the level look-up crosses lanes
                uint32_t pos = cell_of<K>(key_at(k, e), thr);
                if (!ident) pos = (uint32_t)__shfl(own_fin, (int)pos, CMPQ_WAVE);
                word |= pos << (8 * e);
            }
            if (g < n_groups) crow[g] = word;
        }
    }
    __syncthreads();
}

// What a run may leave behind for a later run on the same channel (the final quantization of
// Sec. 3.2.2 differs from the preliminary one by the few entries of O_q): per channel a header
// word, the per-bucket (count << 32 | sum of places) table and the place array, as built from
// ALL weights of the channel.  The later run loads them instead of fetching, keying, counting
// and scattering the weights again, takes the entries of O_q out of the table and blanks one
// byte of the place array per such entry.
constexpr uint32_t kArrMagic = 0xC3A77A00u;  // + 1: an arrangement follows; + 2: the channel held a non-finite weight
__host__ __device__ inline size_t arrangement_stride(int64_t d_out, int lb) {
    return 16 + ((size_t)8 << (16 - lb)) + bucket_arr_bytes(d_out, lb);
}

constexpr int kModePlain = 0;  // codes only
constexpr int kModeFused = 1;  // the coding pass also writes the row of the stored format and the error
constexpr int kModeReuse = 2;  // starts from a kept arrangement; codes like kModeFused (outputs optional)

// One of the place bytes of bucket stretch [w0, w1) (words) that equals `place` becomes a filler.
// Lanes that remove equal values race for the bytes: compare-and-swap, try the next on a loss.
__device__ __forceinline__ void blank_one_place(uint32_t *words, uint32_t w0, uint32_t w1, uint32_t place) {
    const uint32_t pat = place * 0x01010101u;
    uint32_t j = w0;
    while (j < w1) {
        // The search and the exchange are separate loops: lanes of a wavefront find their
        // words after different numbers of steps, and an exchange inside the search would put
        // its round trip into every step that any lane ends on.
        uint32_t x = 0, zero = 0;
        for (; j < w1; j += 4) {  // four words per step, the last one again past the end
            uint32_t xs[4], zs[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) xs[u] = words[min(j + u, w1 - 1)];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t t = xs[u] ^ pat;
                zs[u] = (t - 0x01010101u) & ~t & 0x80808080u;  // lowest flag marks a byte that matches
            }
            if (zs[0] | zs[1] | zs[2] | zs[3]) {
                const uint32_t u = zs[0] ? 0u : (zs[1] ? 1u : (zs[2] ? 2u : 3u));
                x = zs[0] ? xs[0] : (zs[1] ? xs[1] : (zs[2] ? xs[2] : xs[3]));
                zero = zs[0] ? zs[0] : (zs[1] ? zs[1] : (zs[2] ? zs[2] : zs[3]));
                j = min(j + u, w1 - 1);
                break;
            }
        }
        if (!zero) return;
        for (;;) {
            const uint32_t sh = (uint32_t)(__ffs(zero) - 8);  // bit offset of that byte
            const uint32_t nw = (x & ~(0xffu << sh)) | (0x80u << sh);
            const uint32_t old = atomicCAS(&words[j], x, nw);
            if (old == x) return;
            x = old;  // another lane changed the word: look at it again
            const uint32_t t = x ^ pat;
            zero = (t - 0x01010101u) & ~t & 0x80808080u;
            if (!zero) break;
        }
        ++j;
    }
}

// Registers and occupancy.  The longest channels (16 groups a lane, 512 lanes) are bound by LDS:
// 3 workgroups = 6 wavefronts per SIMD at d_out = 28 672 whatever the registers; their budget is
// 64 per lane (72 for the fused final pass, which would spill at 64), so that what they leave
// free lets a wavefront of a memory-bound kernel on another stream in beside them.  Every other
// variant keeps the occupancy it has always run at, 7 wavefronts per SIMD (72 registers; 7
// workgroups of 256 lanes per compute unit).  Measured against budgets of 77 / 72 registers: the
// kernel alone 3-4 % shorter, the whole step with three streams 5 %.
constexpr int waves_per_simd(int G, int T, int MODE) {
    return G == 16 && T == 512 && MODE != kModeFused ? 8 : 7;
}
template <int G, int T, int LB, int MODE>
__global__ __launch_bounds__(T)
    __attribute__((amdgpu_waves_per_eu(waves_per_simd(G, T, MODE), waves_per_simd(G, T, MODE))))
void kmeans_bucket_kernel(KmArgs a) {
    constexpr int kBuckets = 1 << (16 - LB);
    constexpr bool kCodesFused = MODE != kModePlain;
    // dynamic LDS: places of the kept weights, ordered by bucket (a byte each; the bucket
    // follows from the position) | removed-entry bitmap (one bit per weight) | the scatter
    // cursors, later the coding table
    extern __shared__ __align__(16) unsigned char dyn[];
    __shared__ BucketShared<LB> sm;
    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    const int d_out = (int)a.d_out, n_groups = d_out >> 2;
    const int b = a.bits[i];
    float *crow = a.centroids + i * CMPQ_KMAX;
    if (b < 1 || b > 4) {  // a channel of O_act: no levels, no codes, no row; kept whole in FP16: no error
        if (tid < CMPQ_KMAX) crow[tid] = INFINITY;
        if (a.codes) {
            uint32_t *c32 = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
            for (int g = tid; g < n_groups; g += T) c32[g] = 0;
        }
        if (kCodesFused && a.err_ch && tid == 0) a.err_ch[i] = 0.0;
        return;
    }
    // where the channel's row of the stored format goes
    uint32_t *row_dst = nullptr;
    uint16_t *lut_dst = nullptr;
    const int row_words = (int)(((int64_t)d_out * b + 31) / 32);
    if (kCodesFused && a.fused) {
        const int32_t row = a.row_of[i];
        int j = 0;
        while (j < a.pack.n_set && a.pack.width[j] != b) ++j;
        if (row >= 0 && j < a.pack.n_set) {
            if (a.pack.packed[j]) row_dst = a.pack.packed[j] + (int64_t)row * row_words;
            if (a.pack.lut[j]) lut_dst = a.pack.lut[j] + ((int64_t)row << b);
        }
    }
    const int K = 1 << b;
    unsigned char *arr = dyn;
    const size_t arr_bytes = bucket_arr_bytes(d_out, LB);
    uint32_t *removed = reinterpret_cast<uint32_t *>(dyn + arr_bytes);
    const int n_words = (d_out + 31) >> 5;
    uint32_t *cursor = removed + ((n_words + 3) & ~3);
    const __half *wrow_h = static_cast<const __half *>(a.W) + i * a.ldw;
    const uint2 *wrow = reinterpret_cast<const uint2 *>(wrow_h);
    // the arrangement this run leaves (any mode but reuse) or starts from (reuse)
    unsigned char *keep = nullptr;
    if (MODE != kModeReuse && a.arr_keep) keep = static_cast<unsigned char *>(a.arr_keep) + i * a.arr_stride;
    const int per = kBuckets / T > 0 ? kBuckets / T : 1;  // buckets a lane owns in the prefix pass (T is a power of two)
    const int b0 = tid * per;

    uint32_t keys[2 * G];
    uint32_t n_orig[8];  // reuse: the kept arrangement's count of each bucket this lane owns (per <= 8)
    bool input_ok = true;
    uint32_t bad_status = CMPQ_STATUS_NONFINITE;
    if (tid == 0) {  // the slice of out_idx inside this channel
        sm.seg_lo = a.seg ? a.seg[i] : 0;
        const int64_t lo = a.seg ? a.seg[i + 1] : 0;
        sm.n_excl = (int)lo - sm.seg_lo;
    }
    for (int s = tid; s < n_words; s += T) removed[s] = 0;
    if constexpr (MODE == kModeReuse) {
        // ---- the kept arrangement: header, bucket table, place array
        const unsigned char *src = static_cast<const unsigned char *>(a.arr_reuse) + i * a.arr_stride;
        const uint32_t head = *reinterpret_cast<const uint32_t *>(src);
        if (head != kArrMagic + 1u) {
            input_ok = false;  // the earlier run flagged the channel, or this is no arrangement at all
            if (head != kArrMagic + 2u) bad_status = CMPQ_STATUS_ARRANGEMENT;
        } else {
            const unsigned long long *tsrc = reinterpret_cast<const unsigned long long *>(src + 16);
            if (b0 < kBuckets) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    if (r < per) {
                        const unsigned long long packed = tsrc[b0 + r];
                        n_orig[r] = (uint32_t)(packed >> 32);
                        sm.scum[b0 + r] = (long long)packed;
                    }
                }
            }
            const uint4 *asrc = reinterpret_cast<const uint4 *>(src + 16 + (size_t)kBuckets * 8);
            uint4 *a4 = reinterpret_cast<uint4 *>(arr);
            for (int s = tid; s < (int)(arr_bytes >> 4); s += T) a4[s] = asrc[s];
        }
    } else {
        // ---- load: lane owns groups g = k*T + tid of 4 weights, kept as packed 16-bit keys
        uint32_t nonfinite = 0;
#pragma unroll
        for (int k = 0; k < G; ++k) {
            const int g = k * T + tid;
            uint2 raw = make_uint2(0, 0);
            if (g < n_groups) raw = wrow[g];
            nonfinite |= nonfinite_of_half2(raw.x) | nonfinite_of_half2(raw.y);
            keys[2 * k] = keys_of_half2(raw.x);
            keys[2 * k + 1] = keys_of_half2(raw.y);
        }
        input_ok = (nonfinite & 0x80008000u) == 0u;
        for (int s = tid; s < kBuckets; s += T) sm.scum[s] = 0;  // first: count << 32 | sum of places
        uint4 *a4 = reinterpret_cast<uint4 *>(arr);
        for (int s = tid; s < (int)(arr_bytes >> 4); s += T) a4[s] = make_uint4(kFill4, kFill4, kFill4, kFill4);
    }
    bool bad_start = false;
    if (a.start_given && tid < K) {  // the caller's levels, in level order; -0 is taken as +0
        const float given = crow[tid];
        bad_start = !isfinite(given);
        sm.cent[tid] = given == 0.0f ? 0.0f : given;
    }
    if (!__syncthreads_and(input_ok && !bad_start)) {
        // a non-finite weight or starting level (or no usable arrangement): the caller's status
        // word says so; the channel gets defined outputs (all levels 0, all codes 0) instead of
        // a clustering of NaNs
        if (tid == 0 && a.status) atomicOr(a.status, (int)(input_ok ? CMPQ_STATUS_NONFINITE : bad_status));
        if (tid < CMPQ_KMAX) crow[tid] = tid < K ? 0.0f : INFINITY;
        if (a.codes) {
            uint32_t *c32 = reinterpret_cast<uint32_t *>(a.codes + i * a.d_out);
            for (int g = tid; g < n_groups; g += T) c32[g] = 0;
        }
        if constexpr (kCodesFused) {  // the row of all-zero codes, the table of zero levels, no number for the error
            if (row_dst) for (int w = tid; w < row_words; w += T) row_dst[w] = 0;
            if (lut_dst && tid < K) lut_dst[tid] = 0;
            if (a.err_ch && tid == 0) a.err_ch[i] = __longlong_as_double(0x7ff8000000000000ll);
        }
        if (keep && tid == 0) *reinterpret_cast<uint32_t *>(keep) = kArrMagic + 2u;
        return;
    }
    const int n_ex = sm.n_excl;
    uint32_t first_key = 0;  // reuse: the key of entry `tid` of O_q, for the second visit below
    if (n_ex > 0) {  // entries of O_q do not take part in the clustering
        const int32_t *ex_idx = a.out_idx + sm.seg_lo;
        const int32_t chan_base = (int32_t)(i * a.d_out);
        for (int e = tid; e < n_ex; e += T) {
            const int o = ex_idx[e] - chan_base;
            atomicOr(&removed[o >> 5], 1u << (o & 31));
            if constexpr (MODE == kModeReuse) {  // out of its bucket's count and sum of places
                const uint32_t key = key_of_half(__half_as_ushort(wrow_h[o]));
                if (e == tid) first_key = key;
                atomicAdd(reinterpret_cast<unsigned long long *>(&sm.scum[key >> LB]),
                          0ull - ((1ull << 32) | (key & ((1u << LB) - 1))));
            }
        }
        __syncthreads();
    }

    // ---- bucket tables: counts and sums of places of the kept weights
    if constexpr (MODE != kModeReuse) {
        if (n_ex > 0) count_buckets<G, T, LB, true>(keys, removed, sm.scum, n_groups);
        else count_buckets<G, T, LB, false>(keys, removed, sm.scum, n_groups);
        __syncthreads();
    }
    // ---- exclusive prefixes over buckets of count and exact sum; where each bucket's
    //      stretch of the byte array begins (counts rounded up to whole words; with a kept
    //      arrangement the stretches are those of its counts, the prefixes those of what is left)
    {
        unsigned long long *keep_tbl = keep ? reinterpret_cast<unsigned long long *>(keep + 16) : nullptr;
        uint32_t n_loc = 0;  // count | padded count << 16: both stay below 2^16
        long long s_loc = 0;
        if (b0 < kBuckets) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if (r < per) {
                    const unsigned long long packed = (unsigned long long)sm.scum[b0 + r];
                    const uint32_t n = (uint32_t)(packed >> 32);
                    const uint32_t n_place = MODE == kModeReuse ? n_orig[r] : n;
                    n_loc += n | (((n_place + 3) & ~3u) << 16);
                    s_loc += bucket_sum<LB>((uint32_t)(b0 + r), n, (uint32_t)packed);
                    if (keep_tbl) keep_tbl[b0 + r] = packed;
                }
            }
        }
        uint32_t n_run, n_tot;
        unsigned long long s_run_u, s_tot;
        block_scan_excl_pair(n_loc, (unsigned long long)s_loc, sm.scan32, sm.scan64, n_run, s_run_u, n_tot, s_tot);
        long long s_run = (long long)s_run_u;
        if (b0 < kBuckets) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if (r < per) {
                    const unsigned long long packed = (unsigned long long)sm.scum[b0 + r];
                    const uint32_t n = (uint32_t)(packed >> 32);
                    const uint32_t n_place = MODE == kModeReuse ? n_orig[r] : n;
                    const long long sb = bucket_sum<LB>((uint32_t)(b0 + r), n, (uint32_t)packed);
                    sm.ncum[b0 + r] = (uint16_t)(n_run & 0xffffu);
                    sm.start[b0 + r] = (uint16_t)(n_run >> 16);
                    cursor[b0 + r] = n_run >> 16;  // where the next place of the bucket goes
                    sm.scum[b0 + r] = s_run;
                    n_run += n | (((n_place + 3) & ~3u) << 16);
                    s_run += sb;
                }
            }
        }
        if (tid == 0) {
            sm.ncum[kBuckets] = (uint16_t)(n_tot & 0xffffu);
            sm.start[kBuckets] = (uint16_t)(n_tot >> 16);
            sm.scum[kBuckets] = (long long)s_tot;
        }
    }
    __syncthreads();
    const uint32_t M = sm.ncum[kBuckets];
    if constexpr (MODE == kModeReuse) {
        // ---- one place byte per entry of O_q becomes a filler
        if (n_ex > 0) {
            const int32_t *ex_idx = a.out_idx + sm.seg_lo;
            const int32_t chan_base = (int32_t)(i * a.d_out);
            for (int e = tid; e < n_ex; e += T) {
                const uint32_t key =
                    e == tid ? first_key : key_of_half(__half_as_ushort(wrow_h[ex_idx[e] - chan_base]));
                const uint32_t bk = key >> LB;
                blank_one_place(reinterpret_cast<uint32_t *>(arr), sm.start[bk] >> 2, sm.start[bk + 1] >> 2,
                                key & ((1u << LB) - 1));
            }
        }
    } else {
        // ---- scatter the places of the kept weights, ordered by bucket
        if (n_ex > 0) scatter_places<G, T, LB, true>(keys, removed, cursor, arr, n_groups);
        else scatter_places<G, T, LB, false>(keys, removed, cursor, arr, n_groups);
    }
    __syncthreads();
    if (keep) {  // the arrangement as it stands, for a later run on this channel
        const uint4 *a4 = reinterpret_cast<const uint4 *>(arr);
        uint4 *adst = reinterpret_cast<uint4 *>(keep + 16 + (size_t)kBuckets * 8);
        for (int s = tid; s < (int)(arr_bytes >> 4); s += T) adst[s] = a4[s];
        if (tid == 0) *reinterpret_cast<uint32_t *>(keep) = kArrMagic + 1u;
    }

    double err = 0.0;
    switch (K) {
        case 2: lloyd_bucket<G, 2, T, LB, kCodesFused>(a, i, sm, arr, cursor, removed, n_ex, keys, n_groups, M, err); break;
        case 4: lloyd_bucket<G, 4, T, LB, kCodesFused>(a, i, sm, arr, cursor, removed, n_ex, keys, n_groups, M, err); break;
        case 8: lloyd_bucket<G, 8, T, LB, kCodesFused>(a, i, sm, arr, cursor, removed, n_ex, keys, n_groups, M, err); break;
        default: lloyd_bucket<G, 16, T, LB, kCodesFused>(a, i, sm, arr, cursor, removed, n_ex, keys, n_groups, M, err); break;
    }
    if (tid < CMPQ_KMAX) crow[tid] = tid < K ? sm.cent[tid] : INFINITY;
    if constexpr (kCodesFused) {
        // the row is complete in the place array (the coding pass ends with a barrier): copy it
        // out, the table in FP16 beside it, and add the lanes' error sums in a fixed order
        if (row_dst) {
            const uint32_t *stage = reinterpret_cast<const uint32_t *>(arr);
            for (int w = tid; w < row_words; w += T) row_dst[w] = stage[w];
        }
        if (lut_dst && tid < K) lut_dst[tid] = __half_as_ushort(__float2half_rn(sm.cent[tid]));
        err = wave_sum_f64(err);
        double *red = reinterpret_cast<double *>(sm.scan64);
        if ((tid & 63) == 0) red[tid >> 6] = err;
        __syncthreads();
        if (tid == 0 && a.err_ch) {
            double t = 0.0;
            for (int w = 0; w < T / CMPQ_WAVE; ++w) t += red[w];
            a.err_ch[i] = t;
        }
    }
}

size_t bucket_dyn_lds(int64_t d_out, int lb) {
    size_t b = bucket_arr_bytes(d_out, lb);
    b += (size_t)((((d_out + 31) >> 5) + 3) & ~3) * 4;
    b += ((size_t)1 << (16 - lb)) * 4;
    return b;
}

template <int G, int T, int LB>
int launch_variant(const KmArgs &a, hipStream_t s) {
    auto kern = a.arr_reuse ? kmeans_bucket_kernel<G, T, LB, kModeReuse>
                            : (a.fused ? kmeans_bucket_kernel<G, T, LB, kModeFused> : kmeans_bucket_kernel<G, T, LB, kModePlain>);
    const size_t lds = bucket_dyn_lds(a.d_out, LB);
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return CMPQ_EHIP;
    }
    cmpq_timing_before(CMPQ_KERNEL_KMEANS, s);
    kern<<<dim3((unsigned)a.d_in), dim3((unsigned)T), lds, s>>>(a);
    cmpq_timing_after(CMPQ_KERNEL_KMEANS, s);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

#ifndef CMPQ_LB512
#define CMPQ_LB512 6
#endif
#ifndef CMPQ_LB256
#define CMPQ_LB256 7
#endif
// The launch shape launch_kmeans_hist picks for a channel length: lanes per workgroup, groups of
// 4 weights per lane, low bits of a key that name the place inside a bucket.  0 lanes: too long.
static void hist_variant(int64_t d_out, int &T_out, int &G_out, int &LB_out) {
    const int64_t groups = d_out / 4;
    int64_t T = 64;
    while (T < 512 && T * 8 < groups) T <<= 1;
    const int64_t per_lane = cdiv(groups, T);
    T_out = (int)T;
    LB_out = T == 512 ? CMPQ_LB512 : (T == 256 ? CMPQ_LB256 : 7);
    if (per_lane > 16) T_out = 0, G_out = 0;
    else if (per_lane > 8) G_out = 16, LB_out = CMPQ_LB512;
    else if (per_lane > 4) G_out = 8;
    else if (per_lane > 2) G_out = 4;
    else if (per_lane > 1) G_out = 2;
    else G_out = 1;
}

size_t kmeans_hist_arrangement_stride(int64_t d_out) {
    if (d_out < 4 || d_out % 4 != 0) return 0;
    int T, G, LB;
    hist_variant(d_out, T, G, LB);
    return T == 0 ? 0 : arrangement_stride(d_out, LB);
}

extern "C" int cmpq_kmeans_launch_shape(int64_t d_out, int64_t *shape) {
    if (!shape || d_out < 4 || d_out % 4 != 0) return CMPQ_EINVAL;
    int T, G, LB;
    hist_variant(d_out, T, G, LB);
    if (T == 0) return CMPQ_ESHAPE;
    shape[0] = T;
    shape[1] = G;
    shape[2] = LB;
    shape[3] = (int64_t)bucket_arr_bytes(d_out, LB);
    shape[4] = (int64_t)bucket_dyn_lds(d_out, LB);
    shape[5] = LB == 6 ? (int64_t)sizeof(BucketShared<6>) : (int64_t)sizeof(BucketShared<7>);
    return CMPQ_OK;
}

int launch_kmeans_hist(const KmArgs &a, hipStream_t s) {
    // A power-of-two workgroup of at most 512 lanes: up to 32 weights per lane, 64 for the
    // longest channels (two workgroups of 512 share a compute unit where one of 1024
    // would leave it idle at every barrier).
    int T, G, LB;
    hist_variant(a.d_out, T, G, LB);
    if (T == 0) return CMPQ_ESHAPE;
    if (G == 16) return launch_variant<16, 512, CMPQ_LB512>(a, s);
    if (G == 8) {
        switch (T) {
            case 512: return launch_variant<8, 512, CMPQ_LB512>(a, s);
            case 256: return launch_variant<8, 256, CMPQ_LB256>(a, s);
            case 128: return launch_variant<8, 128, 7>(a, s);
            default: return launch_variant<8, 64, 7>(a, s);
        }
    }
    if (G == 4) return launch_variant<4, 64, 7>(a, s);
    if (G == 2) return launch_variant<2, 64, 7>(a, s);
    return launch_variant<1, 64, 7>(a, s);
}
