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

constexpr int kWThreads = 256;
constexpr int kWPerThread = 8;
constexpr int kChunk = kWThreads * kWPerThread;  // elements of one channel handled per step
constexpr int kMaxBlocks = 2048;
constexpr int kBins = 2048;

struct WselState {
    uint32_t prefix;    // digits fixed so far (high bits of the threshold key)
    uint32_t T;         // final threshold key
    uint64_t rem;       // rank still to resolve inside the current prefix
    uint64_t need;      // ties (key == T) to take, in index order
    uint64_t total;     // number of candidate keys
};

struct WselArgs {
    const void *W;
    const float *centroids;
    const uint8_t *codes;
    const uint8_t *bits;
    int64_t d_in, d_out, ldw;
    int64_t chunks_per_channel, total_chunks, chunks_per_block;
    int score;
    int vec_ok;  // 16-byte loads of W and 8-byte loads of codes are aligned
};

// Keys of 8 consecutive entries of channel i starting at output o0 (o0 % 8 == 0).
// valid bit j set when o0+j < d_out.
template <typename TW>
__device__ __forceinline__ uint32_t load_keys8(const WselArgs &a, int64_t i, int64_t o0,
                                               const float *__restrict__ lut, uint32_t (&key)[8],
                                               float (&wv)[8]) {
    uint32_t valid = 0;
    const TW *wrow = static_cast<const TW *>(a.W) + i * a.ldw;
    const uint8_t *crow = a.codes ? a.codes + i * a.d_out : nullptr;
    uint8_t c[8];
    if (a.vec_ok && o0 + 8 <= a.d_out) {
        valid = 0xffu;
        if constexpr (sizeof(TW) == 2) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(wrow + o0);
            const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float2 t = __half22float2(h[j]);
                wv[2 * j] = t.x;
                wv[2 * j + 1] = t.y;
            }
        } else {
            const float4 r0 = *reinterpret_cast<const float4 *>(wrow + o0);
            const float4 r1 = *reinterpret_cast<const float4 *>(wrow + o0 + 4);
            wv[0] = r0.x, wv[1] = r0.y, wv[2] = r0.z, wv[3] = r0.w;
            wv[4] = r1.x, wv[5] = r1.y, wv[6] = r1.z, wv[7] = r1.w;
        }
        if (crow) {
            const uint2 cr = *reinterpret_cast<const uint2 *>(crow + o0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = (cr.x >> (8 * j)) & 0xff;
                c[4 + j] = (cr.y >> (8 * j)) & 0xff;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            wv[j] = 0.f;
            c[j] = 0;
            if (o0 + j < a.d_out) {
                valid |= 1u << j;
                wv[j] = load_as_f32<TW>(wrow, o0 + j);
                if (crow) c[j] = crow[o0 + j];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float s = a.score == CMPQ_SCORE_RESIDUAL ? fabsf(wv[j] - lut[c[j] & 15]) : fabsf(wv[j]);
        key[j] = __float_as_uint(s);
    }
    return valid;
}

__device__ __forceinline__ bool channel_live(const WselArgs &a, int64_t i) {
    const uint8_t b = a.bits[i];
    return b >= 1 && b <= 4;
}

__device__ __forceinline__ void stage_lut(const WselArgs &a, int64_t i, float *lut) {
    __syncthreads();
    if (threadIdx.x < CMPQ_KMAX)
        lut[threadIdx.x] = a.centroids ? a.centroids[i * CMPQ_KMAX + threadIdx.x] : 0.f;
    __syncthreads();
}

__global__ void wsel_init_kernel(WselState *st, uint32_t *hist, uint64_t k, int32_t *idx_out,
                                 int64_t k_fill) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < 3 * kBins) hist[t] = 0;
    if (t == 0) {
        st->prefix = 0;
        st->T = 0;
        st->rem = k;
        st->need = 0;
        st->total = 0;
    }
    for (int64_t j = t; j < k_fill; j += (int64_t)gridDim.x * blockDim.x) idx_out[j] = -1;
}

// PASS 0: digit = key >> 21 (11 bits), PASS 1: (key >> 10) & 2047, PASS 2: key & 1023.
// The last pass also leaves, per workgroup, how many of its keys lie above the 22-bit
// prefix and its own histogram of the last digit: once the threshold is known, the
// counts that ordered compaction needs follow from these without another pass.
template <typename TW, int PASS>
__global__ __launch_bounds__(kWThreads) void wsel_hist_kernel(WselArgs a, const WselState *st,
                                                               uint32_t *__restrict__ hist,
                                                               uint32_t *__restrict__ above,
                                                               uint32_t *__restrict__ local_last) {
    __shared__ uint32_t lh[kBins];
    __shared__ float lut[CMPQ_KMAX];
    __shared__ uint32_t red[kWThreads / CMPQ_WAVE];
    for (int b = threadIdx.x; b < kBins; b += kWThreads) lh[b] = 0;
    const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
    const int64_t q0 = (int64_t)blockIdx.x * a.chunks_per_block;
    const int64_t q1 = min(a.total_chunks, q0 + a.chunks_per_block);
    int64_t cur = -1;
    uint32_t n_above = 0;
    for (int64_t q = q0; q < q1; ++q) {
        const int64_t i = q / a.chunks_per_channel, c = q % a.chunks_per_channel;
        if (!channel_live(a, i)) continue;
        if (i != cur) {
            stage_lut(a, i, lut);
            cur = i;
        }
        uint32_t key[8];
        float wv[8];
        const uint32_t valid = load_keys8<TW>(a, i, c * kChunk + threadIdx.x * kWPerThread, lut, key, wv);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (!((valid >> j) & 1u)) continue;
            if (PASS == 0) {
                atomicAdd(&lh[key[j] >> 21], 1u);
            } else if (PASS == 1) {
                if ((key[j] >> 21) == (prefix >> 21)) atomicAdd(&lh[(key[j] >> 10) & 2047u], 1u);
            } else {
                if ((key[j] >> 10) == (prefix >> 10)) atomicAdd(&lh[key[j] & 1023u], 1u);
                n_above += (key[j] >> 10) > (prefix >> 10);
            }
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kWThreads)
        if (lh[b]) atomicAdd(&hist[PASS * kBins + b], lh[b]);
    if (PASS == 2) {
        for (int b = threadIdx.x; b < 1024; b += kWThreads) local_last[(int64_t)blockIdx.x * 1024 + b] = lh[b];
        n_above = wave_sum_u32(n_above);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = n_above;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t t = 0;
            for (int w = 0; w < kWThreads / CMPQ_WAVE; ++w) t += red[w];
            above[blockIdx.x] = t;
        }
    }
}

// One workgroup of 1024 threads, two bins each: find the digit holding rank `rem`.
template <int PASS>
__global__ __launch_bounds__(1024) void wsel_pick_kernel(WselState *st, const uint32_t *__restrict__ hist) {
    __shared__ uint32_t scan[17];
    const uint32_t *h = hist + PASS * kBins;
    // walk bins from the largest digit down: position r <-> bin 2047 - r
    const int r0 = 2 * threadIdx.x, r1 = r0 + 1;
    const uint32_t h0 = h[kBins - 1 - r0], h1 = h[kBins - 1 - r1];
    uint32_t total;
    const uint32_t before = block_scan_excl_u32(h0 + h1, scan, &total);
    const uint64_t rem = st->rem;
    __syncthreads();
    if (PASS == 0 && threadIdx.x == 0) st->total = total;
    if (rem == 0 || rem > total) {
        // nothing to take, or more asked than there is: take every candidate
        if (threadIdx.x == 0) {
            st->prefix = rem == 0 ? 0xffffffffu : 0u;
            st->rem = rem == 0 ? 0 : rem;  // stays out of range; later passes land here again
            if (PASS == 2) {
                st->T = rem == 0 ? 0xffffffffu : 0u;
                st->need = rem == 0 ? 0 : ~0ull;
            }
        }
        return;
    }
    const int shift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
    if (h0 && before < rem && rem <= (uint64_t)before + h0) {
        st->prefix |= (uint32_t)(kBins - 1 - r0) << shift;
        st->rem = rem - before;
        if (PASS == 2) {
            st->T = st->prefix;
            st->need = rem - before;
        }
    } else if (h1 && before + h0 < rem && rem <= (uint64_t)before + h0 + h1) {
        st->prefix |= (uint32_t)(kBins - 1 - r1) << shift;
        st->rem = rem - before - h0;
        if (PASS == 2) {
            st->T = st->prefix;
            st->need = rem - before - h0;
        }
    }
}

// Per workgroup of the passes: keys above the threshold and keys equal to it, from the
// tables the last histogram pass left.
__global__ __launch_bounds__(kWThreads) void wsel_count_kernel(const WselState *st,
                                                                const uint32_t *__restrict__ above,
                                                                const uint32_t *__restrict__ local_last,
                                                                uint32_t *__restrict__ cnt_gt,
                                                                uint32_t *__restrict__ cnt_eq) {
    __shared__ uint32_t red[kWThreads / CMPQ_WAVE];
    const uint32_t digit = st->T & 1023u;
    const bool everything = st->need == ~0ull;  // more asked than there is: every candidate counts
    const uint32_t *h = local_last + (int64_t)blockIdx.x * 1024;
    uint32_t gt = 0;
    for (int b = threadIdx.x; b < 1024; b += kWThreads)
        if (everything ? b > 0 : (uint32_t)b > digit) gt += h[b];
    gt = wave_sum_u32(gt);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = gt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t g = above[blockIdx.x];
        for (int w = 0; w < kWThreads / CMPQ_WAVE; ++w) g += red[w];
        cnt_gt[blockIdx.x] = g;
        cnt_eq[blockIdx.x] = h[everything ? 0 : digit];
    }
}

// Exclusive prefix over workgroups of (ties seen) and (entries written).
__global__ __launch_bounds__(1024) void wsel_offsets_kernel(const WselState *st, int nblocks,
                                                            const uint32_t *__restrict__ cnt_gt,
                                                            const uint32_t *__restrict__ cnt_eq,
                                                            uint64_t *__restrict__ tie_base,
                                                            uint64_t *__restrict__ out_base) {
    __shared__ uint32_t scan[17];
    const uint64_t need = st->need;
    uint64_t tie_run = 0, out_run = 0;
    for (int base = 0; base < nblocks; base += 1024) {
        const int b = base + threadIdx.x;
        const uint32_t e = b < nblocks ? cnt_eq[b] : 0, g = b < nblocks ? cnt_gt[b] : 0;
        uint32_t e_total, w_total;
        const uint64_t tb = tie_run + block_scan_excl_u32(e, scan, &e_total);
        // ties of this workgroup that are still within the first `need`
        uint64_t take = 0;
        if (tb < need) take = (need - tb) < e ? (need - tb) : e;
        const uint64_t ob = out_run + block_scan_excl_u32(g + (uint32_t)take, scan, &w_total);
        if (b < nblocks) {
            tie_base[b] = tb;
            out_base[b] = ob;
        }
        tie_run += e_total;
        out_run += w_total;
    }
}

template <typename TW>
__global__ __launch_bounds__(kWThreads) void wsel_write_kernel(
    WselArgs a, const WselState *st, const uint64_t *__restrict__ tie_base,
    const uint64_t *__restrict__ out_base, int64_t k, int32_t *__restrict__ idx_out,
    uint16_t *__restrict__ val_out) {
    __shared__ float lut[CMPQ_KMAX];
    __shared__ uint32_t scan[34];
    const uint32_t T = st->T;
    const uint64_t need = st->need;
    uint64_t ties = tie_base[blockIdx.x], outp = out_base[blockIdx.x];
    const int64_t q0 = (int64_t)blockIdx.x * a.chunks_per_block;
    const int64_t q1 = min(a.total_chunks, q0 + a.chunks_per_block);
    int64_t cur = -1;
    for (int64_t q = q0; q < q1; ++q) {
        const int64_t i = q / a.chunks_per_channel, c = q % a.chunks_per_channel;
        if (!channel_live(a, i)) continue;
        if (i != cur) {
            stage_lut(a, i, lut);
            cur = i;
        }
        uint32_t key[8];
        float wv[8];
        const int64_t o0 = c * kChunk + threadIdx.x * kWPerThread;
        const uint32_t valid = load_keys8<TW>(a, i, o0, lut, key, wv);
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
                if ((int64_t)pos < k) {
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

struct WselPlan {
    int64_t chunks_per_channel, total_chunks, chunks_per_block;
    int nblocks;
};

WselPlan wsel_plan(int64_t d_in, int64_t d_out) {
    WselPlan p;
    p.chunks_per_channel = cdiv(d_out, kChunk);
    p.total_chunks = p.chunks_per_channel * d_in;
    int64_t nb = p.total_chunks < kMaxBlocks ? p.total_chunks : kMaxBlocks;
    if (nb < 1) nb = 1;
    p.chunks_per_block = cdiv(p.total_chunks, nb);
    if (p.chunks_per_block < 1) p.chunks_per_block = 1;
    p.nblocks = (int)cdiv(p.total_chunks, p.chunks_per_block);
    if (p.nblocks < 1) p.nblocks = 1;
    return p;
}

template <typename TW>
int launch_weight_select(const WselArgs &a, const WselPlan &p, int64_t k, int32_t *idx_out,
                         uint16_t *val_out, void *ws, hipStream_t s) {
    WsCarver carve(ws);
    WselState *st = carve.take<WselState>(1);
    uint32_t *hist = carve.take<uint32_t>(3 * kBins);
    uint32_t *cnt_gt = carve.take<uint32_t>(kMaxBlocks);
    uint32_t *cnt_eq = carve.take<uint32_t>(kMaxBlocks);
    uint64_t *tie_base = carve.take<uint64_t>(kMaxBlocks);
    uint64_t *out_base = carve.take<uint64_t>(kMaxBlocks);
    uint32_t *above = carve.take<uint32_t>(kMaxBlocks);
    uint32_t *local_last = carve.take<uint32_t>((size_t)kMaxBlocks * 1024);
    wsel_init_kernel<<<64, 256, 0, s>>>(st, hist, (uint64_t)k, idx_out, k);
    wsel_hist_kernel<TW, 0><<<p.nblocks, kWThreads, 0, s>>>(a, st, hist, above, local_last);
    wsel_pick_kernel<0><<<1, 1024, 0, s>>>(st, hist);
    wsel_hist_kernel<TW, 1><<<p.nblocks, kWThreads, 0, s>>>(a, st, hist, above, local_last);
    wsel_pick_kernel<1><<<1, 1024, 0, s>>>(st, hist);
    wsel_hist_kernel<TW, 2><<<p.nblocks, kWThreads, 0, s>>>(a, st, hist, above, local_last);
    wsel_pick_kernel<2><<<1, 1024, 0, s>>>(st, hist);
    wsel_count_kernel<<<p.nblocks, kWThreads, 0, s>>>(st, above, local_last, cnt_gt, cnt_eq);
    wsel_offsets_kernel<<<1, 1024, 0, s>>>(st, p.nblocks, cnt_gt, cnt_eq, tie_base, out_base);
    wsel_write_kernel<TW><<<p.nblocks, kWThreads, 0, s>>>(a, st, tie_base, out_base, k, idx_out, val_out);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

size_t cmpq_ws_allocate_bits(int64_t) { return 256; }
size_t cmpq_ws_outlier_channels(int64_t) { return 256; }
size_t cmpq_ws_outlier_weights(int64_t, int64_t) {
    WsCarver carve(nullptr);
    carve.take<WselState>(1);
    carve.take<uint32_t>(3 * kBins);
    carve.take<uint32_t>(kMaxBlocks);
    carve.take<uint32_t>(kMaxBlocks);
    carve.take<uint64_t>(kMaxBlocks);
    carve.take<uint64_t>(kMaxBlocks);
    carve.take<uint32_t>(kMaxBlocks);
    carve.take<uint32_t>((size_t)kMaxBlocks * 1024);
    return carve.need();
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

extern "C" int cmpq_extract_outliers(int mode, int score, const float *sumsq, const void *W,
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
    if (dtype != CMPQ_F16 && dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (d_out < 0 || !bits || (k > 0 && !idx_out)) return CMPQ_EINVAL;
    if (d_in > 0 && d_out > 0 && !W) return CMPQ_EINVAL;
    if (score == CMPQ_SCORE_RESIDUAL && d_in > 0 && d_out > 0 && (!centroids || !codes)) return CMPQ_EINVAL;
    if (ldw < d_out) return CMPQ_ESHAPE;
    if (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;  // linear index in int32
    if (k > d_in * d_out) return CMPQ_ECOUNT;
    if (k == 0 || d_in == 0 || d_out == 0) return CMPQ_OK;
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_outlier_weights(d_in, d_out))
        return CMPQ_EWORKSPACE;
    const WselPlan p = wsel_plan(d_in, d_out);
    WselArgs a;
    a.W = W;
    a.centroids = centroids;
    a.codes = score == CMPQ_SCORE_RESIDUAL ? codes : nullptr;
    a.bits = bits;
    a.d_in = d_in;
    a.d_out = d_out;
    a.ldw = ldw;
    a.chunks_per_channel = p.chunks_per_channel;
    a.total_chunks = p.total_chunks;
    a.chunks_per_block = p.chunks_per_block;
    a.score = score;
    const int esz = dtype == CMPQ_F16 ? 2 : 4;
    a.vec_ok = reinterpret_cast<uintptr_t>(W) % 16 == 0 && (ldw * esz) % 16 == 0 &&
               (a.codes == nullptr || (reinterpret_cast<uintptr_t>(codes) % 8 == 0 && d_out % 8 == 0));
    return dtype == CMPQ_F16 ? launch_weight_select<__half>(a, p, k, idx_out, val_out, ws, s)
                             : launch_weight_select<float>(a, p, k, idx_out, val_out, ws, s);
}
