// Rankings of the CMPQ path (arXiv 2410.13056): the activation outliers O_act and
// Algorithm 1 rank d_in channel statistics; the quantization-aware outliers O_q
// (Sec. 3.2.2) rank up to d_in*d_out residuals.  All three are "the k largest
// keys, equal keys by smaller index", done with a radix select on the fp32 bit
// pattern of the non-negative key: histogram a digit, locate the digit that holds
// the k-th key, descend.  Nothing is sorted; the selected set is then written in
// index order through ordered compaction (prefix sums), so the output is unique.
#include "common.h"

namespace {

// ------------------------------------------------------------------ one workgroup, d_in keys

constexpr int kSelThreads = 1024;

struct SelShared {
    uint32_t hist[256];
    uint32_t scan[34];
    uint32_t prefix, rem;
};

__device__ __forceinline__ uint32_t stat_key(float f) {
    return f == 0.0f ? 0u : __float_as_uint(f);  // -0 -> +0; the statistic is non-negative
}

// k-th largest key among entries with skip[i] == 0 (skip nullable).  After the
// call: select key > T, and of the keys == T the first `need` in index order.
__device__ void block_kth_largest(const float *__restrict__ keys, const uint8_t *__restrict__ skip,
                                  int64_t d, uint32_t k, SelShared &sh, uint32_t &T,
                                  uint32_t &need) {
    if (k == 0) {  // nothing: no key exceeds the all-ones pattern
        T = 0xffffffffu;
        need = 0;
        return;
    }
    if (threadIdx.x == 0) {
        sh.prefix = 0;
        sh.rem = k;
    }
    uint32_t have_mask = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int b = threadIdx.x; b < 256; b += blockDim.x) sh.hist[b] = 0;
        __syncthreads();
        const uint32_t prefix = sh.prefix;
        for (int64_t i = threadIdx.x; i < d; i += blockDim.x) {
            if (skip && skip[i]) continue;
            const uint32_t key = stat_key(keys[i]);
            if ((key & have_mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        {
            // walk the digits from the largest down, all at once: thread t looks at digit
            // 255 - t and owns it when the rank falls inside its count
            const uint32_t rem = sh.rem;
            const uint32_t v = threadIdx.x < 256 ? sh.hist[255 - threadIdx.x] : 0u;
            uint32_t total;
            const uint32_t before = block_scan_excl_u32(v, sh.scan, &total);
            if (threadIdx.x < 256 && v && before < rem && rem <= before + v) {
                sh.rem = rem - before;  // rank inside the chosen digit
                sh.prefix = prefix | ((uint32_t)(255 - threadIdx.x) << shift);
            }
        }
        have_mask |= 255u << shift;
        __syncthreads();
    }
    T = sh.prefix;
    need = sh.rem;
    __syncthreads();
}

__global__ __launch_bounds__(kSelThreads) void top_channels_kernel(
    const float *__restrict__ sumsq, int64_t d_in, uint32_t k, int32_t *__restrict__ idx_out,
    uint8_t *__restrict__ mask_out) {
    __shared__ SelShared sh;
    uint32_t T, need;
    block_kth_largest(sumsq, nullptr, d_in, k, sh, T, need);
    uint32_t tie_base = 0, out_base = 0;
    for (int64_t base = 0; base < d_in; base += blockDim.x) {
        const int64_t i = base + threadIdx.x;
        uint32_t key = 0;
        const bool in = i < d_in;
        if (in) key = stat_key(sumsq[i]);
        const uint32_t tie = in && key == T, gt = in && key > T;
        // ties are taken in index order until `need` are in, so the number of taken ties
        // before a position is min(ties before it, need): one scan gives both offsets
        uint32_t tie_excl, gt_excl, tie_total, gt_total;
        block_scan_excl_2xu32(tie, gt, sh.scan, tie_excl, gt_excl, tie_total, gt_total);
        const uint32_t tie_rank = tie_base + tie_excl;
        const uint32_t sel = gt || (tie && tie_rank < need);
        const uint32_t pos = out_base + gt_excl + (min(tie_rank, need) - min(tie_base, need));
        if (sel && idx_out) idx_out[pos] = (int32_t)i;
        if (in && mask_out) mask_out[i] = (uint8_t)sel;
        const uint32_t sel_total = gt_total + (min(tie_base + tie_total, need) - min(tie_base, need));
        tie_base += tie_total;
        out_base += sel_total;
    }
}

// bits[i] = w_hi for the k_hi most salient unprotected channels, w_mid for the
// next ones up to rank k_mid, w_lo for the rest; CMPQ_PROTECTED where chan_mask is set.
__global__ __launch_bounds__(kSelThreads) void allocate_bits_kernel(
    const float *__restrict__ sumsq, int64_t d_in, const uint8_t *__restrict__ chan_mask,
    uint32_t k_hi, uint32_t k_mid, int all_mid, int w_hi, int w_mid, int w_lo,
    uint8_t *__restrict__ bits) {
    __shared__ SelShared sh;
    uint32_t T1, need1, T2 = 0, need2 = 0;
    block_kth_largest(sumsq, chan_mask, d_in, k_hi, sh, T1, need1);
    if (!all_mid) block_kth_largest(sumsq, chan_mask, d_in, k_mid, sh, T2, need2);
    uint32_t tie1_base = 0, tie2_base = 0;
    for (int64_t base = 0; base < d_in; base += blockDim.x) {
        const int64_t i = base + threadIdx.x;
        const bool in = i < d_in;
        const bool prot = in && chan_mask && chan_mask[i];
        const bool live = in && !prot;
        uint32_t key = 0;
        if (live) key = stat_key(sumsq[i]);
        const uint32_t tie1 = live && key == T1, tie2 = live && !all_mid && key == T2;
        uint32_t t1_excl, t2_excl, t1_total, t2_total;
        block_scan_excl_2xu32(tie1, tie2, sh.scan, t1_excl, t2_excl, t1_total, t2_total);
        const uint32_t r1 = tie1_base + t1_excl, r2 = tie2_base + t2_excl;
        if (in) {
            int w;
            if (prot)
                w = CMPQ_PROTECTED;
            else if (key > T1 || (tie1 && r1 < need1))
                w = w_hi;
            else if (all_mid || key > T2 || (tie2 && r2 < need2))
                w = w_mid;
            else
                w = w_lo;
            bits[i] = (uint8_t)w;
        }
        tie1_base += t1_total;
        tie2_base += t2_total;
    }
}

// ------------------------------------------------------------------ whole layer, d_in*d_out keys
//
// Top-k of the scores of a whole layer, written in ascending linear index.  The data is
// shared out in wave-chunks (512 consecutive entries of one channel, 8 per lane); a unit
// is one wavefront with a contiguous run of wave-chunks, four consecutive units make a
// workgroup.
//
// Exact chain: three histogram passes over the data fix the threshold key digit by digit
// (11 + 11 + 10 bits).  The last pass also sets aside, unit by unit and in index order,
// every entry whose top 22 bits reach the prefix known by then - a superset of the answer
// a little over k entries long - and the result is written from this staging list.  When
// a unit's share of the list does not fit (many equal scores, or an unusual
// concentration), a flag sends the call down the full path: per-workgroup tables from the
// last pass and one more pass over the data.
//
// Fast chain, tried first: two histogram passes over a sample (every s-th wave-chunk)
// give a 22-bit prefix that, by the sample, a few percent more than k entries reach.  One
// pass over the data stages every entry that reaches it; the exact k-th key is then
// found inside the list (the same three digits, over the list only) and the answer
// written from the list.  The sample only guides the guess: if the list turns out to
// hold fewer than k entries or overflows, a flag is raised and the exact chain, whose
// kernels otherwise return at once, does the work.  Either way the result is the same set.

constexpr int kWThreads = 256;
constexpr int kWaves = kWThreads / CMPQ_WAVE;
constexpr int kWPerLane = 8;
constexpr int kWaveChunk = CMPQ_WAVE * kWPerLane;
constexpr int kMaxBlocks = 2048;
constexpr int kMaxUnits = kMaxBlocks * kWaves;
constexpr int kBins = 2048;
// histograms: 0-2 the digits of the exact chain, 3-4 the sample's, 5-7 the list's
constexpr int kHists = 8;

struct WselState {
    uint32_t T;         // final threshold key
    uint64_t need;      // ties (key == T) to take, in index order
    uint32_t overflow;  // exact chain: a unit's staging share was too small: take the full path
    // fast chain
    uint32_t fast_overflow;  // a unit's staging share was too small
    uint32_t fast_failed;    // the list does not settle the answer: the exact chain runs
    uint32_t guess22;        // staged: top 22 bits >= guess22
};

struct WselArgs {
    const void *W;
    const float *centroids;
    const uint8_t *codes;
    const uint8_t *bits;
    int64_t d_in, d_out, ldw;
    int64_t wc_per_channel, total_wc, wc_per_unit;
    int score;
    int vec_ok;  // 16-byte loads of W and 8-byte loads of codes are aligned
    unsigned long long *stage_ik;  // per unit `cap` entries: linear index << 32 | key
    uint16_t *stage_val;           //   and the entry's value as fp16 bits
    uint32_t *stage_cnt;           // entries staged per unit
    uint32_t cap;
    int64_t sample_stride, n_sample;  // sampled wave-chunks: q = j * stride, j < n_sample
    uint64_t sample_rank;             // rank in the sample that the guess aims at
};

struct WselPlan {
    int64_t wc_per_channel, total_wc, wc_per_unit;
    int nunits, nblocks;
    uint32_t cap;
    int64_t sample_stride, n_sample;
    uint64_t sample_rank;
};

WselPlan wsel_plan(int64_t d_in, int64_t d_out, int64_t k) {
    WselPlan p;
    p.wc_per_channel = cdiv(d_out, kWaveChunk);
    p.total_wc = p.wc_per_channel * d_in;
    int64_t nu = p.total_wc < kMaxUnits ? p.total_wc : kMaxUnits;
    if (nu < 1) nu = 1;
    p.wc_per_unit = cdiv(p.total_wc, nu);
    if (p.wc_per_unit < 1) p.wc_per_unit = 1;
    nu = cdiv(p.total_wc, p.wc_per_unit);
    if (nu < 1) nu = 1;
    p.nblocks = (int)cdiv(nu, kWaves);
    p.nunits = p.nblocks * kWaves;
    // four times a unit's even share of k, plus room for small inputs
    int64_t cap = 4 * cdiv(k, nu) + 256;
    if (cap > p.wc_per_unit * kWaveChunk) cap = p.wc_per_unit * kWaveChunk;
    p.cap = (uint32_t)cap;
    // sample: 8192 wave-chunks or more, a prime stride that does not divide the chunks of a
    // channel (so that every part of a channel is met); aim a margin above the sample's share
    // of k: 6 %, or 8 standard deviations of a count of that size if that is more
    static const int primes[] = {61, 59, 53, 47, 43, 41, 37, 31, 29, 23, 19, 17, 13, 11, 7, 5, 3};
    p.sample_stride = 1;
    for (int pr : primes) {
        if ((int64_t)pr * 8192 <= p.total_wc && p.wc_per_channel % pr != 0) {
            p.sample_stride = pr;
            break;
        }
    }
    p.n_sample = cdiv(p.total_wc, p.sample_stride);
    const double ks = (double)k * (double)p.n_sample / (double)(p.total_wc > 0 ? p.total_wc : 1);
    double margin = 8.0 / __builtin_sqrt(ks > 1.0 ? ks : 1.0);
    if (margin < 0.06) margin = 0.06;
    p.sample_rank = (uint64_t)(ks * (1.0 + margin)) + 8;
    return p;
}

// Eight consecutive entries of a channel as loaded: weights and codes still packed.
template <typename TW>
struct Raw8;
template <>
struct Raw8<__half> {
    uint4 w;
    uint2 c;
};
template <>
struct Raw8<float> {
    float4 w0, w1;
    uint2 c;
};

// (o0, a lane's first output of the wave-chunk, is a 32-bit offset from the channel's row, whose
// address is the same in every lane: loads take that address from scalar registers)
__device__ __forceinline__ uint2 fetch_codes8(const WselArgs &a, int64_t i, int o0, bool vec) {
    uint2 c = make_uint2(0, 0);
    if (!a.codes) return c;
    const uint8_t *crow = a.codes + i * a.d_out;
    const int d_out = (int)a.d_out;
    if (vec) {  // streamed: every pass over the layer reads it once
        typedef uint32_t U2 __attribute__((ext_vector_type(2)));
        const U2 nt = __builtin_nontemporal_load(reinterpret_cast<const U2 *>(crow + o0));
        return make_uint2(nt.x, nt.y);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (o0 + j < d_out) {
            const uint32_t b = crow[o0 + j];
            if (j < 4) c.x |= b << (8 * j); else c.y |= b << (8 * (j - 4));
        }
    }
    return c;
}

__device__ __forceinline__ void fetch8(const WselArgs &a, int64_t i, int o0, Raw8<__half> &r) {
    const uint16_t *wrow = static_cast<const uint16_t *>(a.W) + i * a.ldw;
    const int d_out = (int)a.d_out;
    const bool vec = a.vec_ok && o0 + 8 <= d_out;
    if (vec) {
        typedef uint32_t U4 __attribute__((ext_vector_type(4)));
        const U4 nt = __builtin_nontemporal_load(reinterpret_cast<const U4 *>(wrow + o0));
        r.w = make_uint4(nt.x, nt.y, nt.z, nt.w);
    } else {
        uint32_t h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = o0 + j < d_out ? wrow[o0 + j] : 0u;
        r.w = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
    r.c = fetch_codes8(a, i, o0, vec);
}

__device__ __forceinline__ void fetch8(const WselArgs &a, int64_t i, int o0, Raw8<float> &r) {
    const float *wrow = static_cast<const float *>(a.W) + i * a.ldw;
    const int d_out = (int)a.d_out;
    const bool vec = a.vec_ok && o0 + 8 <= d_out;
    if (vec) {
        r.w0 = *reinterpret_cast<const float4 *>(wrow + o0);
        r.w1 = *reinterpret_cast<const float4 *>(wrow + o0 + 4);
    } else {
        float f[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = o0 + j < d_out ? wrow[o0 + j] : 0.f;
        r.w0 = make_float4(f[0], f[1], f[2], f[3]);
        r.w1 = make_float4(f[4], f[5], f[6], f[7]);
    }
    r.c = fetch_codes8(a, i, o0, vec);
}

__device__ __forceinline__ void unpack8(const Raw8<__half> &r, float (&wv)[8]) {
    const uint32_t w4[4] = {r.w.x, r.w.y, r.w.z, r.w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        wv[2 * j] = __half2float(__ushort_as_half((uint16_t)w4[j]));
        // the upper half converted in place (the compiler would shift it down first)
        asm("v_cvt_f32_f16_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1"
            : "=v"(wv[2 * j + 1])
            : "v"(w4[j]));
    }
}
__device__ __forceinline__ void unpack8(const Raw8<float> &r, float (&wv)[8]) {
    wv[0] = r.w0.x, wv[1] = r.w0.y, wv[2] = r.w0.z, wv[3] = r.w0.w;
    wv[4] = r.w1.x, wv[5] = r.w1.y, wv[6] = r.w1.z, wv[7] = r.w1.w;
}

// Residual scores without codes (Sec. 3.2.2 with Q(x) of Sec. 3: the preliminary quantization
// puts every weight on its nearest level, so |w - Q(w)| is the smallest |w - level| over the
// channel's levels; rounding to fp32 keeps the order, so the smallest rounded difference is the
// rounded difference to the nearest level).  `cent` holds level (lane & 15), +inf past the
// channel's K levels: the number of finite lanes among the first 16 is K.
__device__ __forceinline__ int levels_in(float cent) {
    return (int)__popcll(__ballot(cent < INFINITY) & 0xffffull);
}
__device__ __forceinline__ float min3_abs(float x, float y, float m) {
    asm("v_min3_f32 %0, |%1|, |%2|, %0" : "+v"(m) : "v"(x), "v"(y));
    return m;
}
__device__ __forceinline__ float level_of_lane(float cent, int k) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cent), k));
}
template <int K>
__device__ __forceinline__ void nearest_abs8(const float (&wv)[8], float cent, float (&m)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) m[j] = INFINITY;
#pragma unroll
    for (int k = 0; k < K; k += 2) {
        const float s0 = level_of_lane(cent, k), s1 = level_of_lane(cent, k + 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) m[j] = min3_abs(wv[j] - s0, wv[j] - s1, m[j]);
    }
}
__device__ __forceinline__ void nearest_abs8(const float (&wv)[8], float cent, float (&m)[8]) {
    switch (levels_in(cent)) {  // uniform over the wavefront
        case 2: nearest_abs8<2>(wv, cent, m); break;
        case 4: nearest_abs8<4>(wv, cent, m); break;
        case 8: nearest_abs8<8>(wv, cent, m); break;
        default: nearest_abs8<16>(wv, cent, m); break;  // lanes past K hold +inf and never win
    }
}

// Score keys of the 8 entries.  `cent` holds level (lane & 15) of the channel: the level
// of a code comes from the lane of that number (all lanes of the wavefront take part).
template <typename TW>
__device__ __forceinline__ void score_keys8(const WselArgs &a, const Raw8<TW> &r, float cent,
                                            uint32_t (&key)[8], float (&wv)[8]) {
    unpack8(r, wv);
    if (a.score != CMPQ_SCORE_RESIDUAL) {
#pragma unroll
        for (int j = 0; j < 8; ++j) key[j] = __float_as_uint(fabsf(wv[j]));
        return;
    }
    if (!a.codes) {
        float m[8];
        nearest_abs8(wv, cent, m);
#pragma unroll
        for (int j = 0; j < 8; ++j) key[j] = __float_as_uint(m[j]);
        return;
    }
    // One branch for the whole piece, so that the eight lane exchanges below are issued back to
    // back.  Four codes per word, one per byte: the byte address of lane `code` (code * 4) is a
    // bit-field extract of the word shifted up by two.
    float level[8];
    const uint32_t c4[2] = {(r.c.x & 0x0f0f0f0fu) << 2, (r.c.y & 0x0f0f0f0fu) << 2};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t at;  // written out: the compiler turns the extract back into a shift and a mask
        asm("v_bfe_u32 %0, %1, %2, 6" : "=v"(at) : "v"(c4[j >> 2]), "n"(8 * (j & 3)));
        level[j] = __int_as_float(__builtin_amdgcn_ds_bpermute((int)at, __float_as_int(cent)));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) key[j] = __float_as_uint(fabsf(wv[j] - level[j]));
}

__device__ __forceinline__ uint32_t valid8(int o0, int64_t d_out64) {
    const int d_out = (int)d_out64;
    if (o0 + 8 <= d_out) return 0xffu;
    return o0 < d_out ? (1u << (d_out - o0)) - 1u : 0u;
}

__device__ __forceinline__ bool channel_live(const WselArgs &a, int64_t i) {
    const uint8_t b = a.bits[i];
    return b >= 1 && b <= 4;
}

__device__ __forceinline__ int64_t uniform_i64(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Calls body(i, o0, raw, cent) for every wave-chunk in [q0, q1) of a live channel, in order;
// o0 is this lane's first output, raw its 8 entries as loaded, cent level (lane & 15) of the
// channel.  The loads of the next wave-chunk are issued before the current one is worked on
// (two ahead was measured and is slower).
template <typename TW, typename F>
__device__ __forceinline__ void for_each_raw_chunk(const WselArgs &a, int64_t q0, int64_t q1, F &&body) {
    if (q0 >= q1) return;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1);
    // (the same in every lane, but out of a division the compiler does per lane: taken back into
    // scalar registers, so that the walk over channels and wave-chunks below is scalar work)
    int64_t i = uniform_i64(q0 / a.wc_per_channel);
    int c = __builtin_amdgcn_readfirstlane((int)(q0 % a.wc_per_channel));  // a channel has at most 2^31 / 512 wave-chunks
    const int wc_per_channel = (int)a.wc_per_channel, lane0 = lane * kWPerLane;
    bool live = channel_live(a, i);
    float cent = live && a.centroids ? a.centroids[i * CMPQ_KMAX + (lane & 15)] : 0.f;
    Raw8<TW> cur = {}, nxt = {};
    if (live) fetch8(a, i, c * kWaveChunk + lane0, cur);
    for (int64_t q = q0; q < q1; ++q) {
        int64_t ni = i;
        int nc = c + 1;
        bool live_n = live;
        float cent_n = cent;
        if (nc == wc_per_channel) {
            nc = 0;
            ++ni;
        }
        if (q + 1 < q1) {
            if (ni != i) {
                live_n = channel_live(a, ni);
                cent_n = live_n && a.centroids ? a.centroids[ni * CMPQ_KMAX + (lane & 15)] : 0.f;
            }
            if (live_n) fetch8(a, ni, nc * kWaveChunk + lane0, nxt);
        }
        if (live) body(i, c * kWaveChunk + lane0, cur, cent);
        cur = nxt;
        i = ni;
        c = nc;
        live = live_n;
        cent = cent_n;
    }
}

// The same with the score keys formed: body(i, o0, key, wv, valid).
template <typename TW, typename F>
__device__ __forceinline__ void for_each_wave_chunk(const WselArgs &a, int64_t q0, int64_t q1, F &&body) {
    for_each_raw_chunk<TW>(a, q0, q1, [&](int64_t i, int o0, const Raw8<TW> &raw, float cent) {
        uint32_t key[8];
        float wv[8];
        score_keys8<TW>(a, raw, cent, key, wv);
        body(i, o0, key, wv, valid8(o0, a.d_out));
    });
}

// w - level in fp32 straight from a packed FP16 weight (the conversion is part of the
// instruction: a fused multiply-add w * 1 - level with an FP16 first operand, rounded once,
// which is the subtraction's own rounding).  HI picks the upper half of the word.
template <int HI>
__device__ __forceinline__ float half_minus(uint32_t packed, float level) {
    float d;
    if (HI)
        asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(packed), "v"(level));
    else
        asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(packed), "v"(level));
    return d;
}

// Signed scores of the 8 FP16 entries: w - level (residual score) or w (magnitude score); the
// ranking key of an entry is the bit pattern of the magnitude of its score.
__device__ __forceinline__ void signed_scores8(const WselArgs &a, const Raw8<__half> &r, float cent, float (&d)[8]) {
    const uint32_t w4[4] = {r.w.x, r.w.y, r.w.z, r.w.w};
    float level[8];
    if (a.score == CMPQ_SCORE_RESIDUAL && !a.codes) {  // no codes: the magnitude itself, from the nearest level
        float wv[8];
        unpack8(r, wv);
        nearest_abs8(wv, cent, d);
        return;
    }
    if (a.score == CMPQ_SCORE_RESIDUAL) {
        // one branch for the whole piece, so that the eight lane exchanges are issued back to back
        const uint32_t c4[2] = {(r.c.x & 0x0f0f0f0fu) << 2, (r.c.y & 0x0f0f0f0fu) << 2};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t at;
            asm("v_bfe_u32 %0, %1, %2, 6" : "=v"(at) : "v"(c4[j >> 2]), "n"(8 * (j & 3)));
            level[j] = __int_as_float(__builtin_amdgcn_ds_bpermute((int)at, __float_as_int(cent)));
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) level[j] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        d[2 * j] = half_minus<0>(w4[j], level[2 * j]);
        d[2 * j + 1] = half_minus<1>(w4[j], level[2 * j + 1]);
    }
}

// Appends the entries of this wave-chunk flagged in `cand` (bit j: entry j of the lane) to
// the unit's staging list, in index order: a lane's entries follow those of the lanes
// below it.  Few lanes hold any and hardly one holds two: every lane with entries left
// stores its next one, until none is left.  Called by all lanes of the wavefront.
__device__ __forceinline__ void stage_chunk(uint32_t cand, int64_t i, int o0, int64_t d_out,
                                            const uint32_t (&key)[8], const float (&wv)[8],
                                            unsigned long long *__restrict__ stage_ik,
                                            uint16_t *__restrict__ stage_val, uint32_t cap,
                                            uint32_t &n_staged, bool &over) {
    const unsigned long long has = __ballot(cand != 0);
    if (has == 0ull) return;
    // usual case: no lane holds two - places come from the lane mask alone
    uint32_t excl, tot;
    if (__ballot((cand & (cand - 1)) != 0) == 0ull) {
        excl = __builtin_amdgcn_mbcnt_hi((uint32_t)(has >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)has, 0u));
        tot = (uint32_t)__popcll(has);
    } else {
        const uint32_t n_cand = __popc(cand);
        const uint32_t incl = wave_scan_incl_u32(n_cand);
        tot = __shfl(incl, CMPQ_WAVE - 1, CMPQ_WAVE);
        excl = incl - n_cand;
    }
    if (n_staged + tot <= cap) {
        uint32_t pos = n_staged + excl;
        while (__ballot(cand != 0) != 0ull) {
            if (cand) {
                const int j = __ffs(cand) - 1;
                cand &= cand - 1;
                uint32_t kj = key[0];
                float wj = wv[0];
#pragma unroll
                for (int t = 1; t < 8; ++t) {
                    if (j == t) {
                        kj = key[t];
                        wj = wv[t];
                    }
                }
                stage_ik[pos] = ((unsigned long long)((uint32_t)(i * d_out) + (uint32_t)(o0 + j)) << 32) | kj;
                stage_val[pos] = __half_as_ushort(__float2half_rn(wj));
                ++pos;
            }
        }
    } else {
        over = true;
    }
    n_staged += tot;
}

// stage_chunk for FP16 input: the key of a candidate is the magnitude of its signed score d,
// its value the packed FP16 weight itself.
__device__ __forceinline__ void stage_chunk_half(uint32_t cand, int64_t i, int o0, int64_t d_out,
                                                 const float (&d)[8], const uint4 &w,
                                                 unsigned long long *__restrict__ stage_ik,
                                                 uint16_t *__restrict__ stage_val, uint32_t cap,
                                                 uint32_t &n_staged, bool &over) {
    const unsigned long long has = __ballot(cand != 0);
    if (has == 0ull) return;
    uint32_t excl, tot;
    if (__ballot((cand & (cand - 1)) != 0) == 0ull) {  // usual case: no lane holds two
        excl = __builtin_amdgcn_mbcnt_hi((uint32_t)(has >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)has, 0u));
        tot = (uint32_t)__popcll(has);
    } else {
        const uint32_t n_cand = __popc(cand);
        const uint32_t incl = wave_scan_incl_u32(n_cand);
        tot = __shfl(incl, CMPQ_WAVE - 1, CMPQ_WAVE);
        excl = incl - n_cand;
    }
    if (n_staged + tot <= cap) {
        uint32_t pos = n_staged + excl;
        const uint32_t w4[4] = {w.x, w.y, w.z, w.w};
        while (__ballot(cand != 0) != 0ull) {
            if (cand) {
                const int j = __ffs(cand) - 1;
                cand &= cand - 1;
                float dj = d[0];
                uint32_t wj = w4[0];
#pragma unroll
                for (int t = 1; t < 8; ++t) {
                    if (j == t) dj = d[t];
                    if ((t & 1) == 0 && (j >> 1) == (t >> 1)) wj = w4[t >> 1];
                }
                stage_ik[pos] = ((unsigned long long)((uint32_t)(i * d_out) + (uint32_t)(o0 + j)) << 32) | __float_as_uint(fabsf(dj));
                stage_val[pos] = (uint16_t)(wj >> (16 * (j & 1)));
                ++pos;
            }
        }
    } else {
        over = true;
    }
    n_staged += tot;
}

// ---- staging without codes, FP16 weights: which weights can reach the threshold at all
//
// A weight stays below the threshold t iff it is closer than t to SOME level: the weights that do
// are, level by level, a run of consecutive FP16 values around the level (the rounded difference
// grows with the distance), and the runs of a channel's levels merge into a few intervals - one,
// where the levels lie closer together than 2t.  The intervals are found once per channel, by
// bisection on the very comparison the ranking makes (|fp32(w - level)| < t), so a weight is
// inside one exactly when its score is below t; a wave-chunk is then tested with three packed
// FP16 instructions per pair of weights and interval, and only the few weights outside every
// interval get a score.

// FP16 bit pattern <-> position in the order of the values (-0 just below +0).
__device__ __forceinline__ uint32_t ord_of_half(uint32_t h) { return (h & 0x8000u) ? (~h & 0xffffu) : (h | 0x8000u); }
__device__ __forceinline__ uint32_t half_of_ord(uint32_t o) { return (o & 0x8000u) ? (o & 0x7fffu) : (~o & 0xffffu); }
constexpr uint32_t kOrdLo = 0x0400u, kOrdHi = 0xfbffu;  // -65504 and +65504: the finite values

// What safe_intervals leaves for a channel: in lanes g < n the bounds of interval g (an FP16
// pattern in both halves of a word) and the smallest and largest level whose run it holds.
struct SafeIntervals {
    int n;       // intervals; 0: none (then every weight is a candidate)
    bool whole;  // every level has a run: a weight outside the intervals has one of the levels
                 // lo_level / hi_level as its nearest
    uint32_t lo_pk, hi_pk;
    float lo_level, hi_level;
};

// The intervals of channel levels `cent` (level lane & 15 in every lane; K of them) for threshold
// t (none when t is not positive: then every weight reaches it).  Called by all lanes of the
// wavefront.
__device__ __forceinline__ SafeIntervals safe_intervals(float cent, int K, float t) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), k = lane & 15;
    // lanes 0-15: the lower end of level k's run; lanes 16-31: its upper end, searched in
    // mirrored positions (0xffff - position) so that both searches look for a first position
    const bool upper = (lane & 16) != 0, mine = lane < 32 && k < K;
    auto reached = [&](uint32_t pos) -> bool {  // at or past the end searched for
        const float v = __half2float(__ushort_as_half((uint16_t)half_of_ord(upper ? 0xffffu - pos : pos)));
        return fabsf(v - cent) < t || (upper ? v <= cent : v >= cent);
    };
    // reached(a) false or a before the finite values; reached(b) true or b past them
    uint32_t a = kOrdLo - 1, b = kOrdHi + 1;
    uint32_t guess = ord_of_half(__half_as_ushort(__float2half_rn(upper ? cent + t : cent - t)));
    if (upper) guess = 0xffffu - guess;
    guess = min(max(guess, kOrdLo + 2), kOrdHi - 2);
    if (mine) {  // two positions either side of the rounded end bracket it, but for rare roundings
        if (!reached(guess - 2)) a = guess - 2;
        if (reached(guess + 2)) b = guess + 2;
    }
    while (__ballot(mine && b - a > 1) != 0ull) {
        if (mine && b - a > 1) {
            const uint32_t mid = (a + b) >> 1;
            if (reached(mid)) b = mid; else a = mid;
        }
    }
    const uint32_t end = upper ? 0xffffu - b : b;  // first position of the run / its last
    const uint32_t first = end, last = (uint32_t)__shfl((int)end, k + 16, CMPQ_WAVE);
    // (a level that is itself an FP16 value would be "inside" at t <= 0 by the second clause above)
    const bool valid = lane < 16 && k < K && first <= last && t > 0.f;
    SafeIntervals r;
    r.whole = (int)__popcll(__ballot(valid)) == K;
    // runs in ascending order of their levels (first and last positions ascend with the level):
    // rank by counting, send to the lane of the rank
    const uint32_t cb = __float_as_uint(cent);
    const uint32_t key = valid ? cb ^ ((cb >> 31) ? 0xffffffffu : 0x80000000u) : 0xffffffffu;
    uint32_t rank = 0;
    for (int j = 0; j < K; ++j) {  // (lanes past K hold the largest key and keep their places)
        const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)key, j);
        rank += (kj < key || (kj == key && j < k)) ? 1u : 0u;
    }
    if (k >= K) rank = (uint32_t)k;
    const int to = (lane < 16 ? (int)rank : lane) << 2;  // a permutation of the lanes
    const uint32_t sf = (uint32_t)__builtin_amdgcn_ds_permute(to, valid ? (int)first : 0x10000);
    const uint32_t sl = (uint32_t)__builtin_amdgcn_ds_permute(to, valid ? (int)last : 0);
    const float sc = __int_as_float(__builtin_amdgcn_ds_permute(to, __float_as_int(cent)));
    const bool svalid = lane < 16 && sf <= 0xffffu;
    // running largest last position; a run starts a new interval when an FP16 value lies between
    uint32_t run_max = svalid ? sl : 0u;
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)run_max, d, 16);
        if (k >= d) run_max = max(run_max, up);
    }
    const uint32_t before = (uint32_t)__shfl_up((int)run_max, 1, 16);
    const bool start = svalid && (lane == 0 || sf > before + 1u);
    const uint32_t smask = (uint32_t)__ballot(start) & 0xffffu, vmask = (uint32_t)__ballot(svalid) & 0xffffu;
    r.n = (int)__popc(smask);
    const int gid = (int)__popc(smask & ((2u << k) - 1u)) - 1;
    const bool stop = svalid && (((smask >> (k + 1)) & 1u) || !((vmask >> (k + 1)) & 1u));
    const int to_lo = (start ? gid : 63) << 2, to_hi = (stop ? gid : 63) << 2;
    r.lo_pk = half_of_ord((uint32_t)__builtin_amdgcn_ds_permute(to_lo, (int)sf)) * 0x10001u;
    r.hi_pk = half_of_ord((uint32_t)__builtin_amdgcn_ds_permute(to_hi, (int)run_max)) * 0x10001u;
    r.lo_level = __int_as_float(__builtin_amdgcn_ds_permute(to_lo, __float_as_int(sc)));
    r.hi_level = __int_as_float(__builtin_amdgcn_ds_permute(to_hi, __float_as_int(sc)));
    return r;
}

// The entries of the lane outside every interval: bit q for entry 2q, bit 16 + q for entry
// 2q + 1 (the two halves of word q).  0 in every lane of the wavefront in many wave-chunks.
__device__ __forceinline__ uint32_t outside_intervals8(const uint4 &w, const SafeIntervals &iv) {
    const uint32_t w4[4] = {w.x, w.y, w.z, w.w};
    uint32_t acc[4] = {~0u, ~0u, ~0u, ~0u};  // a half stays non-zero while no interval holds it
    for (int g = 0; g < iv.n; ++g) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)iv.lo_pk, g);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)iv.hi_pk, g);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t c;  // the pair clamped into the interval: unchanged halves are inside
            asm("v_pk_max_f16 %0, %1, %2" : "=v"(c) : "v"(w4[q]), "s"(lo));
            asm("v_pk_min_f16 %0, %1, %2" : "=v"(c) : "v"(c), "s"(hi));
            const uint32_t moved = c ^ w4[q];
            if (g == 0) acc[q] = moved;
            else asm("v_pk_min_u16 %0, %1, %2" : "=v"(acc[q]) : "v"(acc[q]), "v"(moved));
        }
    }
    if (__ballot((acc[0] | acc[1] | acc[2] | acc[3]) != 0u) == 0ull) return 0u;
    uint32_t out = 0;
#pragma unroll
    for (int q = 3; q >= 0; --q) {
        uint32_t one;  // 1 in each half that is not zero
        asm("v_pk_min_u16 %0, %1, %2" : "=v"(one) : "v"(acc[q]), "v"(0x00010001u));
        out = out + out + one;
    }
    return out;
}

// The same layout for "entry j exists" (bit j of valid8).
__device__ __forceinline__ uint32_t pairs_layout(uint32_t valid) {
    uint32_t out = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) out |= (((valid >> (2 * q)) & 1u) << q) | (((valid >> (2 * q + 1)) & 1u) << (16 + q));
    return out;
}

// The smallest |w - level| over the K levels in the first lanes of `cent` (K uniform).
__device__ __forceinline__ float nearest_abs1(float w, float cent, int K) {
    float m = INFINITY;
    for (int k = 0; k < K; k += 2) m = min3_abs(w - level_of_lane(cent, k), w - level_of_lane(cent, k + 1), m);
    return m;
}

// The score of a weight outside every interval, formed by all lanes of the wavefront (the levels
// cross lanes): such a weight lies below all levels of the interval above it and above all
// levels of the one below, so its nearest level is among the intervals' end levels.
__device__ __forceinline__ float outside_score(float wf, float cent, int K, const SafeIntervals &iv) {
    if (iv.whole && iv.n > 0) {
        float key = INFINITY;
        for (int g = 0; g < iv.n; ++g)
            key = min3_abs(wf - level_of_lane(iv.lo_level, g), wf - level_of_lane(iv.hi_level, g), key);
        return key;
    }
    return nearest_abs1(wf, cent, K);
}

// stage_chunk_half for staging without codes: `cand` in the layout of outside_intervals8; the
// key of a candidate is formed here.
__device__ __forceinline__ void stage_chunk_nearest(uint32_t cand, int64_t i, int o0, int64_t d_out, const uint4 &w,
                                                    float cent, int K, const SafeIntervals &iv,
                                                    unsigned long long *__restrict__ stage_ik,
                                                    uint16_t *__restrict__ stage_val, uint32_t cap,
                                                    uint32_t &n_staged, bool &over) {
    const unsigned long long has = __ballot(cand != 0);
    if (has == 0ull) return;
    const uint32_t w4[4] = {w.x, w.y, w.z, w.w};
    auto half_at = [&](int q, int hi) -> uint16_t {  // half `hi` of word q
        uint32_t wq = w4[0];
#pragma unroll
        for (int t = 1; t < 4; ++t)
            if (q == t) wq = w4[t];
        return (uint16_t)(wq >> (16 * hi));
    };
    const uint32_t base = (uint32_t)(i * d_out) + (uint32_t)o0;
    if (__ballot((cand & (cand - 1)) != 0) == 0ull) {  // usual case: no lane holds two
        const uint32_t tot = (uint32_t)__popcll(has);
        if (n_staged + tot <= cap) {
            const uint32_t pos = n_staged + __builtin_amdgcn_mbcnt_hi((uint32_t)(has >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)has, 0u));
            const int bit = cand ? __ffs(cand) - 1 : 0, q = bit & 15, hi = bit >> 4;
            const uint16_t hj = half_at(q, hi);
            const float key = outside_score(__half2float(__ushort_as_half(hj)), cent, K, iv);
            if (cand) {
                stage_ik[pos] = ((unsigned long long)(base + (uint32_t)(2 * q + hi)) << 32) | __float_as_uint(key);
                stage_val[pos] = hj;
            }
        } else {
            over = true;
        }
        n_staged += tot;
        return;
    }
    const uint32_t n_cand = __popc(cand);
    const uint32_t incl = wave_scan_incl_u32(n_cand);
    const uint32_t tot = __shfl(incl, CMPQ_WAVE - 1, CMPQ_WAVE);
    if (n_staged + tot <= cap) {
        // index order inside the lane: entry 2q before 2q + 1 before 2q + 2
        uint32_t order = 0;  // bit j: entry j
#pragma unroll
        for (int q = 0; q < 4; ++q) order |= (((cand >> q) & 1u) << (2 * q)) | (((cand >> (16 + q)) & 1u) << (2 * q + 1));
        uint32_t pos = n_staged + incl - n_cand;
        while (__ballot(order != 0) != 0ull) {
            const int j = order ? __ffs(order) - 1 : 0;
            const uint16_t hj = half_at(j >> 1, j & 1);
            const float key = outside_score(__half2float(__ushort_as_half(hj)), cent, K, iv);
            if (order) {
                order &= order - 1;
                stage_ik[pos] = ((unsigned long long)(base + (uint32_t)j) << 32) | __float_as_uint(key);
                stage_val[pos] = hj;
                ++pos;
            }
        }
    } else {
        over = true;
    }
    n_staged += tot;
}

struct PickShared {
    uint32_t scan[17];
    uint32_t bin, total;
    uint64_t rem_in;
    int ok;
};

// The bin of the 2048-bin histogram h that holds rank `rem`, counted from the largest bin
// down (1-based), and the rank inside that bin.  Called by all 256 threads of a workgroup
// (contains barriers); false when rem is 0 or exceeds the total.
__device__ __forceinline__ bool block_pick(const uint32_t *__restrict__ h, uint64_t rem, PickShared &ps,
                                           uint32_t &bin, uint64_t &rem_in, uint32_t &total) {
    constexpr int kPer = kBins / kWThreads;
    const int r0 = threadIdx.x * kPer;  // position r <-> bin kBins - 1 - r
    uint32_t v[kPer], sum = 0;
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        v[r] = h[kBins - 1 - (r0 + r)];
        sum += v[r];
    }
    uint32_t tot;
    const uint32_t before = block_scan_excl_u32(sum, ps.scan, &tot);
    if (threadIdx.x == 0) {
        ps.ok = 0;
        ps.total = tot;
        ps.bin = 0;
        ps.rem_in = 0;
    }
    __syncthreads();
    if (rem != 0 && rem <= tot) {
        uint64_t run = before;
#pragma unroll
        for (int r = 0; r < kPer; ++r) {
            if (v[r] && run < rem && rem <= run + v[r]) {
                ps.bin = (uint32_t)(kBins - 1 - (r0 + r));
                ps.rem_in = rem - run;
                ps.ok = 1;
            }
            run += v[r];
        }
    }
    __syncthreads();
    bin = ps.bin;
    rem_in = ps.rem_in;
    total = ps.total;
    return ps.ok != 0;
}

// Exact chain: the digits fixed by the first `passes` histograms (11, 11, 10 bits from
// the top) for rank k, and the rank left inside them.  `all` when k exceeds the number of
// candidates: every candidate is taken (prefix 0).  Called by all threads of a workgroup.
__device__ __forceinline__ void exact_prefix(const uint32_t *__restrict__ hist, uint64_t k, int passes,
                                             PickShared &ps, uint32_t &prefix, uint64_t &rem, bool &all) {
    prefix = 0;
    rem = k;
    all = false;
    for (int pass = 0; pass < passes; ++pass) {
        uint32_t bin, tot;
        uint64_t rem_in;
        if (!block_pick(hist + pass * kBins, rem, ps, bin, rem_in, tot)) {
            all = true;
            prefix = 0;
            return;
        }
        prefix |= bin << (pass == 0 ? 21 : (pass == 1 ? 10 : 0));
        rem = rem_in;
    }
}

// Fast chain, sample passes: histogram of the first (PASS 0) or, inside the first digit's
// bin, the second (PASS 1) 11-bit digit over every sample_stride-th wave-chunk.
template <typename TW, int PASS>
__global__ __launch_bounds__(kWThreads) void wsel_sample_kernel(WselArgs a, uint32_t *__restrict__ hist) {
    __shared__ uint32_t lh[kBins];
    __shared__ PickShared ps;
    for (int b = threadIdx.x; b < kBins; b += kWThreads) lh[b] = 0;
    uint32_t bin0 = 0;
    if (PASS == 1) {
        uint64_t r;
        uint32_t tot;
        if (!block_pick(hist + 3 * kBins, a.sample_rank, ps, bin0, r, tot)) return;
    }
    __syncthreads();
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t n_waves = (int64_t)gridDim.x * kWaves;
    // few workgroups (every one ends with a flush into the same global counters), several
    // wave-chunks per wavefront, the next one's loads issued before the current one is used
    struct Item {
        int64_t i, o0;
        bool live;
        float cent;
        Raw8<TW> raw;
    };
    auto load = [&](int64_t j, Item &it) {
        const int64_t q = j * a.sample_stride;
        it.i = q / a.wc_per_channel;
        it.o0 = (q % a.wc_per_channel) * kWaveChunk + lane * kWPerLane;
        // all loads at once: the few channels of O_act are fetched and then dropped
        it.live = channel_live(a, it.i);  // uniform over the wavefront
        fetch8(a, it.i, it.o0, it.raw);
        it.cent = a.centroids ? a.centroids[it.i * CMPQ_KMAX + (lane & 15)] : 0.f;
    };
    int64_t j = (int64_t)blockIdx.x * kWaves + wave;
    Item cur = {}, nxt = {};
    if (j < a.n_sample) load(j, cur);
    for (; j < a.n_sample; j += n_waves) {
        if (j + n_waves < a.n_sample) load(j + n_waves, nxt);
        if (cur.live) {
            uint32_t key[8];
            float wv[8];
            score_keys8<TW>(a, cur.raw, cur.cent, key, wv);
            const uint32_t valid = valid8(cur.o0, a.d_out);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (!((valid >> e) & 1u)) continue;
                if (PASS == 0) {
                    atomicAdd(&lh[key[e] >> 21], 1u);
                } else if ((key[e] >> 21) == bin0) {
                    atomicAdd(&lh[(key[e] >> 10) & 2047u], 1u);
                }
            }
        }
        cur = nxt;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kWThreads)
        if (lh[b]) atomicAdd(&hist[(3 + PASS) * kBins + b], lh[b]);
}

// Fast chain, the one pass over the data: stages every entry whose top 22 bits reach the
// guess read off the sample's histograms.
// NEAR (FP16 weights, residual score, no codes): candidates by the channel's intervals.
template <typename TW, bool NEAR>
__global__ __launch_bounds__(kWThreads) void wsel_stage_kernel(WselArgs a, WselState *st,
                                                                const uint32_t *__restrict__ hist) {
    __shared__ PickShared ps;
    uint32_t guess22 = 0;  // no usable sample: everything reaches it, the list overflows, the exact chain runs
    {
        uint32_t bin0, bin1, tot;
        uint64_t rem0, rem1;
        if (block_pick(hist + 3 * kBins, a.sample_rank, ps, bin0, rem0, tot) &&
            block_pick(hist + 4 * kBins, rem0, ps, bin1, rem1, tot))
            guess22 = (bin0 << 11) | bin1;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) st->guess22 = guess22;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t q0 = unit * a.wc_per_unit;
    const int64_t q1 = min(a.total_wc, q0 + a.wc_per_unit);
    uint32_t n_staged = 0;
    bool over = false;
    const uint32_t reach = guess22 << 10;  // (key >> 10) >= guess22 as one compare
    unsigned long long *stage_ik = a.stage_ik + unit * a.cap;
    uint16_t *stage_val = a.stage_val + unit * a.cap;
    if constexpr (std::is_same<TW, __half>::value) {
        // FP16 weights: the scores stay signed floats and are compared by magnitude (the order of
        // non-negative floats is that of their bit patterns, and "not below" keeps a NaN score a
        // candidate, as its bit pattern would be), the conversion of a weight is folded into the
        // subtraction, and only a candidate's key and value are formed
        const float reach_f = __uint_as_float(reach);
        if constexpr (NEAR) {
            // no codes: per channel the intervals of weights that stay below the guess, per
            // wave-chunk the weights outside them
            int64_t have = -1;
            int K = 0;
            SafeIntervals iv = {};
            for_each_raw_chunk<TW>(a, q0, q1, [&](int64_t i, int o0, const Raw8<TW> &raw, float cent) {
                if (i != have) {
                    have = i;
                    K = levels_in(cent);
                    iv = safe_intervals(cent, K, reach_f);
                }
                uint32_t cand = outside_intervals8(raw.w, iv);
                if (o0 - lane * kWPerLane + kWaveChunk > (int)a.d_out)  // the ragged end of a channel (uniform)
                    cand &= pairs_layout(valid8(o0, a.d_out));
                stage_chunk_nearest(cand, i, o0, a.d_out, raw.w, cent, K, iv, stage_ik, stage_val, a.cap, n_staged, over);
            });
        } else
        for_each_raw_chunk<TW>(a, q0, q1, [&](int64_t i, int o0, const Raw8<TW> &raw, float cent) {
            float d[8];
            signed_scores8(a, raw, cent, d);
            uint32_t cand = 0;  // bit j: entry j reaches the guess
#pragma unroll
            for (int j = 7; j >= 0; --j) cand = cand + cand + (!(fabsf(d[j]) < reach_f) ? 1u : 0u);
            cand &= valid8(o0, a.d_out);
            stage_chunk_half(cand, i, o0, a.d_out, d, raw.w, stage_ik, stage_val, a.cap, n_staged, over);
        });
    } else {
        for_each_wave_chunk<TW>(a, q0, q1, [&](int64_t i, int o0, const uint32_t (&key)[8], const float (&wv)[8], uint32_t valid) {
            // bit j of cand: entry j exists and reaches the guess
            uint32_t cand = 0;
#pragma unroll
            for (int j = 7; j >= 0; --j) cand = cand + cand + (key[j] >= reach ? 1u : 0u);
            cand &= valid;
            stage_chunk(cand, i, o0, a.d_out, key, wv, stage_ik, stage_val, a.cap, n_staged, over);
        });
    }
    if (lane == 0) {
        a.stage_cnt[unit] = over ? 0u : n_staged;
        if (over) st->fast_overflow = 1u;
    }
}

// Fast chain, passes over the list: the exact k-th key of the list by the same three
// digits as the exact chain (11 + 11 + 10 bits), each pass reading the digits the earlier
// ones fixed off their histograms.  The second pass also settles whether the list holds
// the answer at all: it does unless it overflowed or is shorter than k.
template <int PASS>
__global__ __launch_bounds__(kWThreads) void wsel_list_kernel(WselArgs a, WselState *st, int nunits,
                                                               uint32_t *__restrict__ hist, uint64_t k) {
    __shared__ uint32_t lh[kBins];
    __shared__ PickShared ps;
    for (int b = threadIdx.x; b < kBins; b += kWThreads) lh[b] = 0;
    const bool overflowed = st->fast_overflow != 0;
    uint32_t prefix = 0;
    if (PASS > 0) {
        uint64_t rem;
        bool all;
        exact_prefix(hist + 5 * kBins, k, PASS, ps, prefix, rem, all);
        const bool failed = overflowed || all;
        if (PASS == 1 && blockIdx.x == 0 && threadIdx.x == 0) st->fast_failed = failed ? 1u : 0u;
        if (failed) return;
    } else if (overflowed) {
        return;
    }
    __syncthreads();
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    for (int64_t unit = (int64_t)blockIdx.x * kWaves + wave; unit < nunits; unit += (int64_t)gridDim.x * kWaves) {
        const unsigned long long *ik = a.stage_ik + unit * a.cap;
        const uint32_t n = a.stage_cnt[unit];
#pragma unroll 4
        for (uint32_t e = lane; e < n; e += CMPQ_WAVE) {
            const uint32_t key = (uint32_t)ik[e];
            if (PASS == 0) {
                atomicAdd(&lh[key >> 21], 1u);
            } else if (PASS == 1) {
                if ((key >> 21) == (prefix >> 21)) atomicAdd(&lh[(key >> 10) & 2047u], 1u);
            } else {
                if ((key >> 10) == (prefix >> 10)) atomicAdd(&lh[key & 1023u], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kWThreads)
        if (lh[b]) atomicAdd(&hist[(5 + PASS) * kBins + b], lh[b]);
}

__global__ void wsel_init_kernel(WselState *st, uint32_t *hist, int32_t *idx_out,
                                 int64_t k_fill) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < kHists * kBins) hist[t] = 0;
    if (t == 0) {
        st->T = 0;
        st->need = 0;
        st->overflow = 0;
        st->fast_overflow = 0;
        st->fast_failed = 0;
        st->guess22 = 0;
    }
    for (int64_t j = t; j < k_fill; j += (int64_t)gridDim.x * blockDim.x) idx_out[j] = -1;
}

// PASS 0: digit = key >> 21 (11 bits), PASS 1: (key >> 10) & 2047, PASS 2: key & 1023.
// The last pass also stages the entries whose top 22 bits reach the prefix and leaves,
// per workgroup, how many of its keys lie above the 22-bit prefix and its own histogram
// of the last digit (what the full path needs to place its output without counting again).
template <typename TW, int PASS>
__global__ __launch_bounds__(kWThreads) void wsel_hist_kernel(WselArgs a, WselState *st, uint64_t k,
                                                               uint32_t *__restrict__ hist,
                                                               uint32_t *__restrict__ above,
                                                               uint32_t *__restrict__ local_last) {
    // the first digit is the same for most keys: its histogram is kept in 4 copies, chosen
    // by lane, so that fewer lanes collide on one counter
    constexpr int kCopies = PASS == 0 ? 4 : 1;
    __shared__ uint32_t lh[kCopies * kBins];
    __shared__ uint32_t red[kWaves];
    if (!st->fast_failed) return;  // the fast chain settled the answer
    for (int b = threadIdx.x; b < kCopies * kBins; b += kWThreads) lh[b] = 0;
    __shared__ PickShared ps;
    uint32_t prefix = 0;
    {
        uint64_t rem;
        bool all;
        exact_prefix(hist, k, PASS, ps, prefix, rem, all);  // the digits the passes before this one fixed
    }
    __syncthreads();
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    uint32_t *lh0 = lh + (lane & (kCopies - 1)) * kBins;
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t q0 = unit * a.wc_per_unit;
    const int64_t q1 = min(a.total_wc, q0 + a.wc_per_unit);
    uint32_t n_above = 0, n_staged = 0;
    bool over = false;
    unsigned long long *stage_ik = a.stage_ik + unit * a.cap;
    uint16_t *stage_val = a.stage_val + unit * a.cap;
    for_each_wave_chunk<TW>(a, q0, q1, [&](int64_t i, int o0, const uint32_t (&key)[8], const float (&wv)[8], uint32_t valid) {
        uint32_t cand = 0;  // bit j: entry j reaches the 22-bit prefix
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (!((valid >> j) & 1u)) continue;
            if (PASS == 0) {
                atomicAdd(&lh0[key[j] >> 21], 1u);
            } else if (PASS == 1) {
                if ((key[j] >> 21) == (prefix >> 21)) atomicAdd(&lh[(key[j] >> 10) & 2047u], 1u);
            } else {
                if ((key[j] >> 10) == (prefix >> 10)) atomicAdd(&lh[key[j] & 1023u], 1u);
                n_above += (key[j] >> 10) > (prefix >> 10);
                cand |= (uint32_t)((key[j] >> 10) >= (prefix >> 10)) << j;
            }
        }
        if (PASS == 2) stage_chunk(cand, i, o0, a.d_out, key, wv, stage_ik, stage_val, a.cap, n_staged, over);
    });
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kWThreads) {
        uint32_t n = lh[b];
#pragma unroll
        for (int r = 1; r < kCopies; ++r) n += lh[r * kBins + b];
        if (n) atomicAdd(&hist[PASS * kBins + b], n);
    }
    if (PASS == 2) {
        if (lane == 0) {
            a.stage_cnt[unit] = over ? 0u : n_staged;
            if (over) st->overflow = 1u;
        }
        for (int b = threadIdx.x; b < 1024; b += kWThreads) local_last[(int64_t)blockIdx.x * 1024 + b] = lh[b];
        n_above = wave_sum_u32(n_above);
        if (lane == 0) red[wave] = n_above;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t t = 0;
            for (int w = 0; w < kWaves; ++w) t += red[w];
            above[blockIdx.x] = t;
        }
    }
}

// Keys above the threshold and keys equal to it: per unit from the staging list, or, on
// the full path, per workgroup from the tables the last histogram pass left.
// First settles the threshold: read off the list's second histogram when the fast chain
// holds the answer, else off the three histograms of the exact chain.
__global__ __launch_bounds__(kWThreads) void wsel_count_kernel(WselState *st, WselArgs a, uint64_t k,
                                                                const uint32_t *__restrict__ hist,
                                                                const uint32_t *__restrict__ above,
                                                                const uint32_t *__restrict__ local_last,
                                                                uint32_t *__restrict__ cnt_gt,
                                                                uint32_t *__restrict__ cnt_eq) {
    __shared__ uint32_t red[kWaves];
    __shared__ PickShared ps;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const bool exact = st->fast_failed != 0;
    uint32_t T;
    uint64_t need;
    {
        bool all;  // the three digits of the list's histograms, or of the exact chain's
        exact_prefix(exact ? hist : hist + 5 * kBins, k, 3, ps, T, need, all);
        if (all) need = ~0ull;  // T = 0: every candidate counts
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->T = T;
        st->need = need;
    }
    if (!exact || !st->overflow) {
        const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
        const unsigned long long *ik = a.stage_ik + unit * a.cap;
        const uint32_t n = a.stage_cnt[unit];
        uint32_t gt = 0, eq = 0;
        for (uint32_t e = lane; e < n; e += CMPQ_WAVE) {
            const uint32_t key = (uint32_t)ik[e];
            gt += key > T;
            eq += key == T;
        }
        gt = wave_sum_u32(gt);
        eq = wave_sum_u32(eq);
        if (lane == 0) {
            cnt_gt[unit] = gt;
            cnt_eq[unit] = eq;
        }
        return;
    }
    const uint32_t digit = T & 1023u;
    const bool everything = need == ~0ull;  // more asked than there is: every candidate counts
    const uint32_t *h = local_last + (int64_t)blockIdx.x * 1024;
    uint32_t gt = 0;
    for (int b = threadIdx.x; b < 1024; b += kWThreads)
        if (everything ? b > 0 : (uint32_t)b > digit) gt += h[b];
    gt = wave_sum_u32(gt);
    if (lane == 0) red[wave] = gt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t g = above[blockIdx.x];
        for (int w = 0; w < kWaves; ++w) g += red[w];
        cnt_gt[blockIdx.x] = g;
        cnt_eq[blockIdx.x] = h[everything ? 0 : digit];
    }
}

// Exclusive prefix over units (or workgroups, on the full path) of (ties seen) and
// (entries written).  A thread takes kMaxUnits / 1024 consecutive entries.
__global__ __launch_bounds__(1024) void wsel_offsets_kernel(const WselState *st, int nunits, int nblocks,
                                                            const uint32_t *__restrict__ cnt_gt,
                                                            const uint32_t *__restrict__ cnt_eq,
                                                            uint64_t *__restrict__ tie_base,
                                                            uint64_t *__restrict__ out_base) {
    constexpr int kPer = kMaxUnits / 1024;
    __shared__ uint32_t scan[17];
    const uint64_t need = st->need;
    const int n = st->fast_failed && st->overflow ? nblocks : nunits;
    const int b0 = threadIdx.x * kPer;
    uint32_t e[kPer], g[kPer], e_sum = 0;
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        e[r] = b0 + r < n ? cnt_eq[b0 + r] : 0;
        g[r] = b0 + r < n ? cnt_gt[b0 + r] : 0;
        e_sum += e[r];
    }
    uint32_t e_total, w_total;
    uint64_t tb = block_scan_excl_u32(e_sum, scan, &e_total);
    // ties of an entry that are still within the first `need`
    uint32_t w[kPer], w_sum = 0;
    uint64_t tbs[kPer];
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        tbs[r] = tb;
        uint64_t take = 0;
        if (tb < need) take = (need - tb) < e[r] ? (need - tb) : e[r];
        w[r] = g[r] + (uint32_t)take;
        w_sum += w[r];
        tb += e[r];
    }
    uint64_t ob = block_scan_excl_u32(w_sum, scan, &w_total);
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        if (b0 + r < n) {
            tie_base[b0 + r] = tbs[r];
            out_base[b0 + r] = ob;
        }
        ob += w[r];
    }
}

__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Writes the answer from the staging list: a wavefront per unit, 64 staged entries a step.
__device__ __forceinline__ void emit_from_list(const WselArgs &a, const WselState *st,
                                               const uint64_t *__restrict__ tie_base,
                                               const uint64_t *__restrict__ out_base, int64_t k,
                                               int32_t *__restrict__ idx_out, uint16_t *__restrict__ val_out) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t unit = (int64_t)blockIdx.x * kWaves + wave;
    const uint32_t T = st->T;
    const uint64_t need = st->need;
    const unsigned long long *ik = a.stage_ik + unit * a.cap;
    const uint16_t *sv = a.stage_val + unit * a.cap;
    const uint32_t n = a.stage_cnt[unit];
    uint64_t ties = tie_base[unit], outp = out_base[unit];
    for (uint32_t e0 = 0; e0 < n; e0 += CMPQ_WAVE) {
        const uint32_t e = e0 + lane;
        const unsigned long long v = e < n ? ik[e] : 0ull;
        const uint32_t key = (uint32_t)v;
        const bool is_eq = e < n && key == T, is_gt = e < n && key > T;
        const unsigned long long eq_mask = __ballot(is_eq);
        const bool sel = is_gt || (is_eq && ties + lanes_below(eq_mask) < need);
        const unsigned long long sel_mask = __ballot(sel);
        const uint64_t pos = outp + lanes_below(sel_mask);
        if (sel && (int64_t)pos < k) {
            idx_out[pos] = (int32_t)(v >> 32);
            if (val_out) val_out[pos] = sv[e];
        }
        ties += __popcll(eq_mask);
        outp += __popcll(sel_mask);
    }
}

// Writes, in index order, the selected entries of the wave-chunks [q0, q1): keys above T, and
// of the keys equal to T those whose running tie count is still below `need`.  The whole
// workgroup takes 4 wave-chunks (2048 consecutive entries) a step; `ties` and `outp` are the
// tie count and the output position before q0, positions at or beyond out_end are dropped.
template <typename TW>
__device__ __forceinline__ void write_chunks(const WselArgs &a, uint32_t T, uint64_t need, uint64_t ties,
                                             uint64_t outp, int64_t q0, int64_t q1, int64_t out_end,
                                             int32_t *__restrict__ idx_out, uint16_t *__restrict__ val_out,
                                             uint32_t *scan) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    for (int64_t qb = q0; qb < q1; qb += kWaves) {
        const int64_t q = qb + wave;
        const int64_t i = q / a.wc_per_channel, c = q % a.wc_per_channel;
        const int64_t o0 = c * kWaveChunk + lane * kWPerLane;
        uint32_t key[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        float wv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        uint32_t valid = 0;
        if (q < q1 && channel_live(a, i)) {  // uniform over the wavefront
            Raw8<TW> raw;
            fetch8(a, i, o0, raw);
            const float cent = a.centroids ? a.centroids[i * CMPQ_KMAX + (lane & 15)] : 0.f;
            score_keys8<TW>(a, raw, cent, key, wv);
            valid = valid8(o0, a.d_out);
        }
        uint32_t n_eq = 0, n_gt = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool v = (valid >> j) & 1u;
            n_eq += v && key[j] == T;
            n_gt += v && key[j] > T;
        }
        // ties are taken in index order until `need` are in: the number of taken ties before
        // a position is min(ties before it, need), so one scan places everything
        uint32_t eq_excl, gt_excl, eq_total, gt_total;
        block_scan_excl_2xu32(n_eq, n_gt, scan, eq_excl, gt_excl, eq_total, gt_total);
        uint64_t my_tie = ties + eq_excl;
        const uint64_t taken_before = (my_tie < need ? my_tie : need) - (ties < need ? ties : need);
        uint64_t pos = outp + gt_excl + taken_before;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (!((valid >> j) & 1u)) continue;
            bool sel = key[j] > T;
            if (key[j] == T) {
                sel = my_tie < need;
                ++my_tie;
            }
            if (sel) {
                if ((int64_t)pos < out_end) {
                    idx_out[pos] = (int32_t)(i * a.d_out + o0 + j);
                    if (val_out) val_out[pos] = __half_as_ushort(__float2half_rn(wv[j]));
                }
                ++pos;
            }
        }
        const uint64_t ties_after = ties + eq_total;
        const uint32_t sel_total =
            gt_total + (uint32_t)((ties_after < need ? ties_after : need) - (ties < need ? ties : need));
        ties += eq_total;
        outp += sel_total;
    }
}

// Full path: one more pass over the data, a workgroup per run of 4 units.
template <typename TW>
__device__ __forceinline__ void write_full(const WselArgs &a, const WselState *st,
                                           const uint64_t *__restrict__ tie_base,
                                           const uint64_t *__restrict__ out_base, int64_t k,
                                           int32_t *__restrict__ idx_out, uint16_t *__restrict__ val_out,
                                           uint32_t *scan) {
    const int64_t q0 = (int64_t)blockIdx.x * kWaves * a.wc_per_unit;
    const int64_t q1 = min(a.total_wc, q0 + kWaves * a.wc_per_unit);
    write_chunks<TW>(a, st->T, st->need, tie_base[blockIdx.x], out_base[blockIdx.x], q0, q1, k, idx_out, val_out,
                     scan);
}

// The last kernel of a call: from the list, unless the exact chain ran and its list
// overflowed.
template <typename TW>
__global__ __launch_bounds__(kWThreads) void wsel_emit_kernel(WselArgs a, const WselState *st,
                                                               const uint64_t *__restrict__ tie_base,
                                                               const uint64_t *__restrict__ out_base,
                                                               int64_t k, int32_t *__restrict__ idx_out,
                                                               uint16_t *__restrict__ val_out) {
    __shared__ uint32_t scan[34];
    if (st->fast_failed && st->overflow)
        write_full<TW>(a, st, tie_base, out_base, k, idx_out, val_out, scan);
    else
        emit_from_list(a, st, tie_base, out_base, k, idx_out, val_out);
}

// ------------------------------------------------------------------ one channel at a time
//
// The variant of O_q with the same count in every channel: a workgroup per channel finds the
// channel's k-th largest key by the same three digits (11 + 11 + 10 bits, the keys formed
// again from the weights in every pass: a channel's row stays in cache) and writes the
// channel's k entries in index order at the place its rank among the quantized channels gives.

// rank[i] = number of channels before i with bits in 1..4.
__global__ __launch_bounds__(1024) void wsel_live_rank_kernel(const uint8_t *__restrict__ bits, int64_t d_in,
                                                              int32_t *__restrict__ rank) {
    __shared__ uint32_t scan[17];
    uint32_t run = 0;
    for (int64_t base = 0; base < d_in; base += blockDim.x) {
        const int64_t i = base + threadIdx.x;
        const uint32_t f = i < d_in && bits[i] >= 1 && bits[i] <= 4;
        uint32_t total;
        const uint32_t before = run + block_scan_excl_u32(f, scan, &total);
        if (i < d_in) rank[i] = (int32_t)before;
        run += total;
    }
}

template <typename TW>
__global__ __launch_bounds__(kWThreads) void wsel_channel_kernel(WselArgs a, const int32_t *__restrict__ live_rank,
                                                                  int64_t k, int32_t *__restrict__ idx_out,
                                                                  uint16_t *__restrict__ val_out) {
    __shared__ uint32_t lh[kBins];
    __shared__ PickShared ps;
    __shared__ uint32_t scan[34];
    const int64_t i = blockIdx.x;
    if (!channel_live(a, i)) return;  // uniform over the workgroup
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const float cent = a.centroids ? a.centroids[i * CMPQ_KMAX + (lane & 15)] : 0.f;
    uint32_t prefix = 0;
    uint64_t rem = (uint64_t)k;  // 1 <= k <= d_out: every pass finds its digit
    for (int pass = 0; pass < 3; ++pass) {
        for (int b = threadIdx.x; b < kBins; b += kWThreads) lh[b] = 0;
        __syncthreads();
        for (int64_t c = wave; c < a.wc_per_channel; c += kWaves) {
            const int64_t o0 = c * kWaveChunk + lane * kWPerLane;
            Raw8<TW> raw;
            fetch8(a, i, o0, raw);
            uint32_t key[8];
            float wv[8];
            score_keys8<TW>(a, raw, cent, key, wv);
            const uint32_t valid = valid8(o0, a.d_out);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (!((valid >> j) & 1u)) continue;
                if (pass == 0) {
                    atomicAdd(&lh[key[j] >> 21], 1u);
                } else if (pass == 1) {
                    if ((key[j] >> 21) == (prefix >> 21)) atomicAdd(&lh[(key[j] >> 10) & 2047u], 1u);
                } else {
                    if ((key[j] >> 10) == (prefix >> 10)) atomicAdd(&lh[key[j] & 1023u], 1u);
                }
            }
        }
        __syncthreads();
        uint32_t bin, tot;
        uint64_t rem_in;
        block_pick(lh, rem, ps, bin, rem_in, tot);
        prefix |= bin << (pass == 0 ? 21 : (pass == 1 ? 10 : 0));
        rem = rem_in;
        __syncthreads();
    }
    const int64_t out0 = (int64_t)live_rank[i] * k;
    write_chunks<TW>(a, prefix, rem, 0, (uint64_t)out0, i * a.wc_per_channel, (i + 1) * a.wc_per_channel, out0 + k,
                     idx_out, val_out, scan);
}

struct WselWs {
    WselState *st;
    uint32_t *hist, *cnt_gt, *cnt_eq, *above, *local_last, *stage_cnt;
    uint64_t *tie_base, *out_base;
    unsigned long long *stage_ik;
    uint16_t *stage_val;
    size_t bytes;
};

WselWs wsel_carve(void *ws, const WselPlan &p) {
    WsCarver carve(ws);
    WselWs w;
    w.st = carve.take<WselState>(1);
    w.hist = carve.take<uint32_t>(kHists * kBins);
    w.cnt_gt = carve.take<uint32_t>(kMaxUnits);
    w.cnt_eq = carve.take<uint32_t>(kMaxUnits);
    w.tie_base = carve.take<uint64_t>(kMaxUnits);
    w.out_base = carve.take<uint64_t>(kMaxUnits);
    w.above = carve.take<uint32_t>(kMaxBlocks);
    w.local_last = carve.take<uint32_t>((size_t)kMaxBlocks * 1024);
    w.stage_cnt = carve.take<uint32_t>(kMaxUnits);
    w.stage_ik = carve.take<unsigned long long>((size_t)p.nunits * p.cap);
    w.stage_val = carve.take<uint16_t>((size_t)p.nunits * p.cap);
    w.bytes = carve.need();
    return w;
}

template <typename TW>
int launch_weight_select(WselArgs a, const WselPlan &p, int64_t k, int32_t *idx_out,
                         uint16_t *val_out, void *ws, hipStream_t s) {
    const WselWs w = wsel_carve(ws, p);
    a.stage_ik = w.stage_ik;
    a.stage_val = w.stage_val;
    a.stage_cnt = w.stage_cnt;
    a.cap = p.cap;
    a.sample_stride = p.sample_stride;
    a.n_sample = p.n_sample;
    a.sample_rank = p.sample_rank;
    int64_t sample_blocks = cdiv(p.n_sample, kWaves);
    if (sample_blocks > 512) sample_blocks = 512;
    if (sample_blocks < 1) sample_blocks = 1;
    wsel_init_kernel<<<64, 256, 0, s>>>(w.st, w.hist, idx_out, k);
    // fast chain
    wsel_sample_kernel<TW, 0><<<(unsigned)sample_blocks, kWThreads, 0, s>>>(a, w.hist);
    wsel_sample_kernel<TW, 1><<<(unsigned)sample_blocks, kWThreads, 0, s>>>(a, w.hist);
    cmpq_timing_before(CMPQ_KERNEL_OUTLIER_STAGE, s);
    if (std::is_same<TW, __half>::value && a.score == CMPQ_SCORE_RESIDUAL && !a.codes)
        wsel_stage_kernel<TW, true><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, w.hist);
    else
        wsel_stage_kernel<TW, false><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, w.hist);
    cmpq_timing_after(CMPQ_KERNEL_OUTLIER_STAGE, s);
    const int list_blocks = p.nblocks < 256 ? p.nblocks : 256;  // few: each ends with a flush into shared counters
    wsel_list_kernel<0><<<list_blocks, kWThreads, 0, s>>>(a, w.st, p.nunits, w.hist, (uint64_t)k);
    wsel_list_kernel<1><<<list_blocks, kWThreads, 0, s>>>(a, w.st, p.nunits, w.hist, (uint64_t)k);
    wsel_list_kernel<2><<<list_blocks, kWThreads, 0, s>>>(a, w.st, p.nunits, w.hist, (uint64_t)k);
    // exact chain: these return at once unless the fast chain raised its flag
    wsel_hist_kernel<TW, 0><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, (uint64_t)k, w.hist, w.above, w.local_last);
    wsel_hist_kernel<TW, 1><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, (uint64_t)k, w.hist, w.above, w.local_last);
    wsel_hist_kernel<TW, 2><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, (uint64_t)k, w.hist, w.above, w.local_last);
    // threshold, placement and output, from whichever chain holds the answer
    wsel_count_kernel<<<p.nblocks, kWThreads, 0, s>>>(w.st, a, (uint64_t)k, w.hist, w.above, w.local_last, w.cnt_gt, w.cnt_eq);
    wsel_offsets_kernel<<<1, 1024, 0, s>>>(w.st, p.nunits, p.nblocks, w.cnt_gt, w.cnt_eq, w.tie_base, w.out_base);
    wsel_emit_kernel<TW><<<p.nblocks, kWThreads, 0, s>>>(a, w.st, w.tie_base, w.out_base, k, idx_out, val_out);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

size_t cmpq_ws_allocate_bits(int64_t) { return 256; }
size_t cmpq_ws_outlier_channels(int64_t) { return 256; }
size_t cmpq_ws_outlier_weights(int64_t d_in, int64_t d_out, int64_t k) {
    if (k < 0) k = 0;
    // the layer-wide selection's tables and lists; the per-channel one needs d_in ranks
    const size_t layer = wsel_carve(nullptr, wsel_plan(d_in, d_out, k)).bytes;
    const size_t channel = align_up((size_t)(d_in > 0 ? d_in : 1) * sizeof(int32_t), 256);
    return layer > channel ? layer : channel;
}

extern "C" int cmpq_allocate_bits(const float *sumsq, int64_t d_in, const uint8_t *chan_mask,
                                  int64_t n_protected, const int32_t *bit_set, int n_set,
                                  double avg_bits, uint8_t *bits, int64_t *counts_host, void *ws,
                                  size_t ws_bytes, void *stream) {
    (void)ws;
    (void)ws_bytes;
    if (!sumsq || !bits || !bit_set || d_in < 0 || n_protected < 0 || n_protected > d_in)
        return CMPQ_EINVAL;
    if (!chan_mask && n_protected != 0) return CMPQ_EINVAL;
    if (d_in >= (int64_t)1 << 31) return CMPQ_ESHAPE;
    if (n_set < 1 || n_set > 4) return CMPQ_EBUDGET;
    for (int j = 0; j < n_set; ++j) {
        if (bit_set[j] < 1 || bit_set[j] > 4) return CMPQ_EBUDGET;
        if (j && bit_set[j] != bit_set[j - 1] + 1) return CMPQ_EBUDGET;
    }
    const int lo = bit_set[0], hi = bit_set[n_set - 1];
    if (!(avg_bits >= lo - 1e-9 && avg_bits <= hi + 1e-9)) return CMPQ_EBUDGET;
    const int64_t d_eff = d_in - n_protected;
    // the integer budget
    int64_t k_hi, k_mid;
    int w_hi, w_mid, w_lo, all_mid;
    const double nearest = (double)(int64_t)(avg_bits + 0.5);
    const double gap = avg_bits - nearest;
    if ((gap < 0 ? -gap : gap) < 1e-9) {
        const int s = (int)nearest;
        int64_t m = 0;
        if (s - 1 >= lo && s + 1 <= hi && d_eff > 0) {
            const double x = 0.01 * (double)(d_eff - 1) - 1e-12;
            m = (int64_t)x;
            if ((double)m < x) ++m;  // ceil
            if (m < 0) m = 0;
            if (2 * m > d_eff) m = d_eff / 2;
        }
        k_hi = m;
        k_mid = d_eff - m;
        w_hi = s + 1;
        w_mid = s;
        w_lo = s - 1;
        all_mid = m == 0;
    } else {
        const int s = (int)avg_bits;  // floor, avg_bits > 0
        const int64_t T = (int64_t)(avg_bits * (double)d_eff + 1e-9);
        k_hi = T - (int64_t)s * d_eff;
        k_mid = d_eff;
        w_hi = s + 1;
        w_mid = s;
        w_lo = s;
        all_mid = 1;
    }
    if (counts_host) {
        for (int j = 0; j < n_set; ++j) counts_host[j] = 0;
        if (k_hi > 0) counts_host[w_hi - lo] += k_hi;
        if (k_mid - k_hi > 0) counts_host[w_mid - lo] += k_mid - k_hi;
        if (d_eff - k_mid > 0) counts_host[w_lo - lo] += d_eff - k_mid;
    }
    if (d_in == 0) return CMPQ_OK;
    allocate_bits_kernel<<<1, kSelThreads, 0, static_cast<hipStream_t>(stream)>>>(
        sumsq, d_in, chan_mask, (uint32_t)k_hi, (uint32_t)k_mid, all_mid, w_hi, w_mid, w_lo, bits);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

extern "C" int cmpq_extract_outliers(int mode, int score, int scope, const float *sumsq, const void *W,
                                     int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                                     const float *centroids, const uint8_t *codes,
                                     const uint8_t *bits, int64_t k, int32_t *idx_out,
                                     uint16_t *val_out, uint8_t *chan_mask_out, void *ws,
                                     size_t ws_bytes, void *stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d_in < 0 || k < 0) return CMPQ_EINVAL;
    if (mode == CMPQ_OUTLIER_CHANNELS) {
        if (!sumsq || (k > 0 && !idx_out)) return CMPQ_EINVAL;
        if (d_in >= (int64_t)1 << 31) return CMPQ_ESHAPE;
        if (k > d_in) return CMPQ_ECOUNT;
        if (d_in == 0) return CMPQ_OK;
        top_channels_kernel<<<1, kSelThreads, 0, s>>>(sumsq, d_in, (uint32_t)k, idx_out, chan_mask_out);
        CMPQ_LAUNCH_CHECK();
        return CMPQ_OK;
    }
    if (mode != CMPQ_OUTLIER_WEIGHTS) return CMPQ_EINVAL;
    if (score != CMPQ_SCORE_RESIDUAL && score != CMPQ_SCORE_MAGNITUDE) return CMPQ_EINVAL;
    if (scope != CMPQ_SCOPE_LAYER && scope != CMPQ_SCOPE_CHANNEL) return CMPQ_EINVAL;
    if (dtype != CMPQ_F16 && dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (d_out < 0 || !bits || (k > 0 && !idx_out)) return CMPQ_EINVAL;
    if (d_in > 0 && d_out > 0 && !W) return CMPQ_EINVAL;
    if (score == CMPQ_SCORE_RESIDUAL && d_in > 0 && d_out > 0 && !centroids) return CMPQ_EINVAL;
    if (ldw < d_out) return CMPQ_ESHAPE;
    if (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;  // linear index in int32
    if (scope == CMPQ_SCOPE_CHANNEL ? k > d_out : k > d_in * d_out) return CMPQ_ECOUNT;
    if (scope == CMPQ_SCOPE_CHANNEL && d_in > 0 && k > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;
    if (k == 0 || d_in == 0 || d_out == 0) return CMPQ_OK;
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_outlier_weights(d_in, d_out, k))
        return CMPQ_EWORKSPACE;
    const WselPlan p = wsel_plan(d_in, d_out, k);
    WselArgs a;
    a.W = W;
    a.centroids = centroids;
    a.codes = score == CMPQ_SCORE_RESIDUAL ? codes : nullptr;
    a.bits = bits;
    a.d_in = d_in;
    a.d_out = d_out;
    a.ldw = ldw;
    a.wc_per_channel = p.wc_per_channel;
    a.total_wc = p.total_wc;
    a.wc_per_unit = p.wc_per_unit;
    a.score = score;
    const int esz = dtype == CMPQ_F16 ? 2 : 4;
    a.vec_ok = reinterpret_cast<uintptr_t>(W) % 16 == 0 && (ldw * esz) % 16 == 0 &&
               (a.codes == nullptr || (reinterpret_cast<uintptr_t>(codes) % 8 == 0 && d_out % 8 == 0));
    if (scope == CMPQ_SCOPE_CHANNEL) {
        int32_t *live_rank = static_cast<int32_t *>(ws);
        wsel_live_rank_kernel<<<1, 1024, 0, s>>>(bits, d_in, live_rank);
        if (dtype == CMPQ_F16)
            wsel_channel_kernel<__half><<<(unsigned)d_in, kWThreads, 0, s>>>(a, live_rank, k, idx_out, val_out);
        else
            wsel_channel_kernel<float><<<(unsigned)d_in, kWThreads, 0, s>>>(a, live_rank, k, idx_out, val_out);
        CMPQ_LAUNCH_CHECK();
        return CMPQ_OK;
    }
    return dtype == CMPQ_F16 ? launch_weight_select<__half>(a, p, k, idx_out, val_out, ws, s)
                             : launch_weight_select<float>(a, p, k, idx_out, val_out, ws, s);
}
