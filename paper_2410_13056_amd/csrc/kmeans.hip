// cmpq_kmeans_quantize: channel-wise non-uniform quantization (Sec. 3.2.1 of
// arXiv 2410.13056).  One workgroup owns one input channel W[i,:]: the d_out
// weights are staged once in LDS and stay there through the start-up (exact order
// statistics by radix select), every Lloyd round and the final coding, so HBM sees
// 2 bytes in and 1 byte out per weight.
//
// Assignment never computes distances.  The levels are ranked once per round
// (they need not be ascending: a level that lost all members keeps a stale value),
// and between neighbouring distinct levels lo < hi the largest fp32 value that still
// belongs to lo is derived exactly from the fp64 midpoint, with the tie rule "equal
// distance goes to the smaller level index" folded in.  A weight's cell is then the
// number of thresholds below it - K-1 compares, identical to the nearest level in
// exact arithmetic (Sec. 3 eq. Q(x)).
//
// Update: each lane adds its weights into private (cell, lane) slots of an fp64
// table in LDS, the table is reduced per cell in a fixed order, and the new level is
// the fp64 quotient rounded once to fp32.  For fp16 inputs with 0/1 weights these
// sums are exact, so the result does not depend on the lane layout.
#include "kmeans_args.h"

namespace {

constexpr int kT = 256;  // threads per workgroup
constexpr int kWavesPerBlock = kT / CMPQ_WAVE;

struct KmSmall {
    float cent[CMPQ_KMAX];   // levels, by level index
    float sorted[CMPQ_KMAX]; // levels, ascending
    float thr[CMPQ_KMAX];    // thr[p]: largest value of the cell at sorted position p
    int perm[CMPQ_KMAX];     // sorted position -> level index
    double tot_sum[CMPQ_KMAX];
    double tot_mass[CMPQ_KMAX];
    uint32_t q_rank[CMPQ_KMAX];
    uint32_t q_prefix[CMPQ_KMAX];
    int q_leader[CMPQ_KMAX];
    uint32_t scan[17];
    uint32_t M;
    int seg_lo, seg_hi;
    int nonfinite;
};

template <typename TW>
struct Elem;
template <>
struct Elem<__half> {
    static constexpr int kKeyBits = 16;
    __device__ static float to_f32(__half h) { return __half2float(h); }
    __device__ static uint32_t key(__half h) {
        uint32_t u = __half_as_ushort(h);
        return (u & 0x8000u) ? (~u & 0xffffu) : (u | 0x8000u);
    }
    __device__ static float from_key(uint32_t k) {
        uint32_t u = (k & 0x8000u) ? (k & 0x7fffu) : (~k & 0xffffu);
        return __half2float(__ushort_as_half((unsigned short)u));
    }
    __device__ static __half canon(__half h, int &bad) {
        const unsigned short u = __half_as_ushort(h);
        if ((u & 0x7c00u) == 0x7c00u) bad = 1;
        return u == 0x8000u ? __ushort_as_half((unsigned short)0) : h;
    }
};
template <>
struct Elem<float> {
    static constexpr int kKeyBits = 32;
    __device__ static float to_f32(float f) { return f; }
    __device__ static uint32_t key(float f) { return f32_ordered_key(f); }
    __device__ static float from_key(uint32_t k) { return f32_from_ordered_key(k); }
    __device__ static float canon(float f, int &bad) {
        if (!isfinite(f)) bad = 1;
        return f == 0.0f ? 0.0f : f;
    }
};

__device__ __forceinline__ float next_below(float t) {
    uint32_t u = __float_as_uint(t);
    if (t > 0.0f)
        u -= 1;
    else if (t == 0.0f)
        u = 0x80000001u;
    else
        u += 1;
    return __uint_as_float(u);
}

// Largest fp32 value that is nearer to `lo` than to `hi` (lo < hi), a value at equal
// distance going to the level with the smaller index.
__device__ __forceinline__ float cell_upper_edge(float lo, float hi, int owner_lo, int owner_hi) {
    const double mid = ((double)lo + (double)hi) * 0.5;
    float t = (float)mid;
    if ((double)t > mid) t = next_below(t);
    if ((double)t == mid && owner_hi < owner_lo) t = next_below(t);
    return t;
}

// Ranks the K levels and derives the K-1 cell edges.  Called by every thread.
__device__ void prepare_cells(KmSmall &sm, int K) {
    const int j = threadIdx.x;
    if (j < K) {
        const float c = sm.cent[j];
        int rank = 0;
        for (int l = 0; l < K; ++l) {
            const float cl = sm.cent[l];
            rank += (cl < c) || (cl == c && l < j);
        }
        sm.sorted[rank] = c;
        sm.perm[rank] = j;
    }
    __syncthreads();
    if (j < K - 1) {
        const float lo = sm.sorted[j];
        int q = j + 1;
        while (q < K && sm.sorted[q] == lo) ++q;
        float t = INFINITY;
        if (q < K && sm.sorted[q] > lo) {
            int g = j;
            while (g > 0 && sm.sorted[g - 1] == lo) --g;
            t = cell_upper_edge(lo, sm.sorted[q], sm.perm[g], sm.perm[q]);
        }
        sm.thr[j] = t;
    }
    __syncthreads();
}

template <int K>
__device__ __forceinline__ int cell_of(float x, const float (&thr)[K - 1 > 0 ? K - 1 : 1]) {
    int pos = 0;
#pragma unroll
    for (int p = 0; p < K - 1; ++p) pos += x > thr[p];
    return pos;
}

template <typename TW, bool WEIGHTED, int K>
__device__ void lloyd_rounds(const KmArgs &a, int64_t i, KmSmall &sm, const TW *xs,
                             const uint32_t *incl, double *sums, void *mass_raw) {
    using MassT = typename std::conditional<WEIGHTED, double, uint32_t>::type;
    MassT *mass = static_cast<MassT *>(mass_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d_out = (int)a.d_out;
    for (int round = 0; round <= a.iters; ++round) {
        prepare_cells(sm, K);
        float thr[K - 1 > 0 ? K - 1 : 1];
#pragma unroll
        for (int p = 0; p < K - 1; ++p) thr[p] = sm.thr[p];
        if (round == a.iters) {  // final coding
            uint8_t *crow = a.codes + i * a.d_out;
            for (int o = tid; o < d_out; o += kT)
                crow[o] = (uint8_t)sm.perm[cell_of<K>(Elem<TW>::to_f32(xs[o]), thr)];
            break;
        }
#pragma unroll
        for (int p = 0; p < K; ++p) {
            sums[p * kT + tid] = 0.0;
            mass[p * kT + tid] = (MassT)0;
        }
        for (int o = tid; o < d_out; o += kT) {
            const float x = Elem<TW>::to_f32(xs[o]);
            const int pos = cell_of<K>(x, thr);
            if ((incl[o >> 5] >> (o & 31)) & 1u) {
                if constexpr (WEIGHTED) {
                    const double m = (double)a.ew[i * a.d_out + o];
                    sums[pos * kT + tid] += m * (double)x;
                    mass[pos * kT + tid] += m;
                } else {
                    sums[pos * kT + tid] += (double)x;
                    mass[pos * kT + tid] += 1u;
                }
            }
        }
        __syncthreads();
        for (int p = wave; p < K; p += kWavesPerBlock) {
            double s = 0.0, m = 0.0;
#pragma unroll
            for (int r = 0; r < kWavesPerBlock; ++r) {
                s += sums[p * kT + r * 64 + lane];
                m += (double)mass[p * kT + r * 64 + lane];
            }
            s = wave_sum_f64(s);
            m = wave_sum_f64(m);
            if (lane == 0) {
                sm.tot_sum[p] = s;
                sm.tot_mass[p] = m;
            }
        }
        __syncthreads();
        if (tid < K && sm.tot_mass[tid] > 0.0)
            sm.cent[sm.perm[tid]] = (float)(sm.tot_sum[tid] / sm.tot_mass[tid]);
        __syncthreads();
    }
}

// Start-up: level j = order statistic floor((2j+1)*M/(2K)) of the M included values,
// found exactly by a most-significant-digit radix select run for all K ranks at once.
template <typename TW>
__device__ void quantile_start(KmSmall &sm, int K, int d_out, const TW *xs, const uint32_t *incl,
                               uint32_t *hist /* [K*256] */) {
    constexpr int kBits = Elem<TW>::kKeyBits;
    const int tid = threadIdx.x;
    const uint32_t M = sm.M;
    if (M == 0) {
        if (tid < K) sm.cent[tid] = 0.0f;
        __syncthreads();
        return;
    }
    if (tid < K) {
        sm.q_rank[tid] = (uint32_t)(((uint64_t)(2 * tid + 1) * M) / (uint64_t)(2 * K));
        sm.q_prefix[tid] = 0;
    }
    __syncthreads();
    for (int shift = kBits - 8; shift >= 0; shift -= 8) {
        if (tid < K) {  // ranks that share a prefix share a histogram: the first of them leads
            int lead = tid;
            for (int l = tid - 1; l >= 0; --l)
                if (sm.q_prefix[l] == sm.q_prefix[tid]) lead = l;
            sm.q_leader[tid] = lead;
        }
        for (int b = tid; b < K * 256; b += kT) hist[b] = 0;
        __syncthreads();
        for (int o = tid; o < d_out; o += kT) {
            if (!((incl[o >> 5] >> (o & 31)) & 1u)) continue;
            const uint32_t key = Elem<TW>::key(xs[o]);
            const uint32_t hi = shift + 8 >= kBits ? 0u : key >> (shift + 8);
            const uint32_t digit = (key >> shift) & 255u;
            for (int j = 0; j < K; ++j)
                if (sm.q_leader[j] == j && sm.q_prefix[j] == hi) atomicAdd(&hist[j * 256 + digit], 1u);
        }
        __syncthreads();
        if (tid < K) {
            const uint32_t *h = hist + sm.q_leader[tid] * 256;
            uint32_t rank = sm.q_rank[tid], cum = 0;
            int b = 0;
            for (; b < 255; ++b) {
                if (cum + h[b] > rank) break;
                cum += h[b];
            }
            sm.q_rank[tid] = rank - cum;
            sm.q_prefix[tid] = (sm.q_prefix[tid] << 8) | (uint32_t)b;
        }
        __syncthreads();
    }
    if (tid < K) sm.cent[tid] = Elem<TW>::from_key(sm.q_prefix[tid]);
    __syncthreads();
}

template <typename TW, bool WEIGHTED>
__device__ void kmeans_channel(const KmArgs &a, int64_t i, unsigned char *lds, KmSmall &sm) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int d_out = (int)a.d_out;
    const int b = a.bits[i];
    float *crow = a.centroids + i * CMPQ_KMAX;
    if (b < 1 || b > 4) {  // a channel of O_act: no levels, no codes
        if (tid < CMPQ_KMAX) crow[tid] = INFINITY;
        for (int o = tid; o < d_out; o += kT) a.codes[i * a.d_out + o] = 0;
        return;
    }
    const int K = 1 << b;
    // LDS carve-up (sizes mirrored by kmeans_lds_bytes on the host)
    size_t off = 0;
    TW *xs = reinterpret_cast<TW *>(lds);
    off += align_up_dev((size_t)d_out * sizeof(TW));
    uint32_t *incl = reinterpret_cast<uint32_t *>(lds + off);
    off += align_up_dev((size_t)((d_out + 63) / 64) * 8);
    double *sums = reinterpret_cast<double *>(lds + off);  // doubles as the start-up histograms
    off += (size_t)CMPQ_KMAX * kT * sizeof(double);
    void *mass = lds + off;

    if (tid == 0) sm.nonfinite = 0;
    __syncthreads();
    // stage the channel; one bit per entry says whether it takes part in the updates
    const TW *wrow = static_cast<const TW *>(a.W) + i * a.ldw;
    int bad = 0;
    for (int base = 0; base < d_out; base += kT) {
        const int o = base + tid;
        bool in = false;
        if (o < d_out) {
            xs[o] = Elem<TW>::canon(wrow[o], bad);
            in = true;
            if constexpr (WEIGHTED) in = a.ew[i * a.d_out + o] > 0.0f;
        }
        const unsigned long long m = __ballot(in);
        if (lane == 0 && base + (tid & ~63) < d_out) {
            incl[(o >> 5)] = (uint32_t)m;
            incl[(o >> 5) + 1] = (uint32_t)(m >> 32);
        }
    }
    if (bad) sm.nonfinite = 1;
    // entries removed before clustering: the slice of out_idx that falls in this channel
    if (tid == 0) {
        sm.seg_lo = a.seg ? a.seg[i] : 0;
        const int64_t lo = a.seg ? a.seg[i + 1] : 0;
        sm.seg_hi = (int)lo;
    }
    __syncthreads();
    for (int e = sm.seg_lo + tid; e < sm.seg_hi; e += kT) {
        const int o = (int)(a.out_idx[e] - i * a.d_out);
        atomicAnd(&incl[o >> 5], ~(1u << (o & 31)));
    }
    __syncthreads();
    uint32_t cnt = 0;
    for (int w = tid; w < (d_out + 31) / 32; w += kT) cnt += __popc(incl[w]);
    uint32_t total;
    block_scan_excl_u32(cnt, sm.scan, &total);
    if (tid == 0) sm.M = total;
    if (tid == 0 && sm.nonfinite && a.status) atomicOr(a.status, CMPQ_STATUS_NONFINITE);
    __syncthreads();

    if (a.start_given) {  // the caller's levels, in level order; -0 is taken as +0
        if (tid < K) {
            const float given = crow[tid];
            if (!isfinite(given) && a.status) atomicOr(a.status, CMPQ_STATUS_NONFINITE);
            sm.cent[tid] = given == 0.0f ? 0.0f : given;
        }
        __syncthreads();
    } else {
        quantile_start<TW>(sm, K, d_out, xs, incl, reinterpret_cast<uint32_t *>(sums));
    }

    switch (K) {
        case 2: lloyd_rounds<TW, WEIGHTED, 2>(a, i, sm, xs, incl, sums, mass); break;
        case 4: lloyd_rounds<TW, WEIGHTED, 4>(a, i, sm, xs, incl, sums, mass); break;
        case 8: lloyd_rounds<TW, WEIGHTED, 8>(a, i, sm, xs, incl, sums, mass); break;
        default: lloyd_rounds<TW, WEIGHTED, 16>(a, i, sm, xs, incl, sums, mass); break;
    }
    if (tid < CMPQ_KMAX) crow[tid] = tid < K ? sm.cent[tid] : INFINITY;
}

// Without a `deferred` list: workgroup i takes channel i.  With one: a small grid walks
// the list and takes the channels the first kernel left behind (usually none).
template <typename TW, bool WEIGHTED>
__global__ __launch_bounds__(kT) void kmeans_kernel(KmArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ KmSmall sm;
    if (!a.deferred) {
        kmeans_channel<TW, WEIGHTED>(a, blockIdx.x, lds, sm);
        return;
    }
    // usually nothing was left over: look at all flags of this workgroup's channels at once
    int any = 0;
    for (int64_t i = blockIdx.x + (int64_t)threadIdx.x * gridDim.x; i < a.d_in; i += (int64_t)kT * gridDim.x)
        any |= a.deferred[i];
    if (!__syncthreads_or(any)) return;
    for (int64_t i = blockIdx.x; i < a.d_in; i += gridDim.x) {
        if (!a.deferred[i]) continue;
        __syncthreads();  // LDS of the previous channel is no longer in use
        kmeans_channel<TW, WEIGHTED>(a, i, lds, sm);
    }
}

size_t kmeans_lds_bytes(int64_t d_out, size_t esz, bool weighted) {
    size_t b = align_up((size_t)d_out * esz, 16);
    b += align_up((size_t)cdiv(d_out, 64) * 8, 16);
    b += (size_t)CMPQ_KMAX * kT * sizeof(double);
    b += (size_t)CMPQ_KMAX * kT * (weighted ? sizeof(double) : sizeof(uint32_t));
    return b;
}

template <typename TW, bool WEIGHTED>
int launch_kmeans(const KmArgs &a, hipStream_t s) {
    const size_t lds = kmeans_lds_bytes(a.d_out, sizeof(TW), WEIGHTED);
    auto kern = kmeans_kernel<TW, WEIGHTED>;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return CMPQ_EHIP;
    }
    const int64_t grid = a.deferred ? (a.d_in < 256 ? a.d_in : 256) : a.d_in;
    kern<<<(unsigned)grid, kT, lds, s>>>(a);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

size_t cmpq_ws_pack_with_error(int64_t d_in);

static size_t ws_kmeans_base(int64_t d_in) {
    // one byte per channel (deferred flags) | d_in + 1 slice offsets of out_idx
    return align_up((size_t)(d_in > 0 ? d_in : 1), 256) + align_up((size_t)(d_in + 1) * sizeof(int32_t), 256);
}

size_t cmpq_ws_kmeans_arrangement(int64_t d_in, int64_t d_out) {
    return align_up((size_t)(d_in > 0 ? d_in : 0) * kmeans_hist_arrangement_stride(d_out), 256);
}

size_t cmpq_ws_kmeans(int64_t d_in, int64_t) {
    // ... | each channel's row in its width group | what cmpq_pack_with_error needs when the
    // stored format is asked for and the histogram kernel does not take the input
    return ws_kmeans_base(d_in) + align_up((size_t)(d_in > 0 ? d_in : 1) * sizeof(int32_t), 256) +
           cmpq_ws_pack_with_error(d_in);
}

extern "C" int cmpq_kmeans_quantize_job(const cmpq_kmeans_job *job, void *ws, size_t ws_bytes, void *stream) {
    if (!job) return CMPQ_EINVAL;
    const cmpq_kmeans_job &j = *job;
    const int64_t d_in = j.d_in, d_out = j.d_out;
    if (d_in < 0 || d_out < 0 || j.n_out < 0 || j.iters < 0) return CMPQ_EINVAL;
    if (j.dtype != CMPQ_F16 && j.dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (j.init != CMPQ_INIT_QUANTILE && j.init != CMPQ_INIT_GIVEN) return CMPQ_EINVAL;
    if (j.algorithm != CMPQ_KMEANS_HISTOGRAM && j.algorithm != CMPQ_KMEANS_DIRECT) return CMPQ_EINVAL;
    if (j.arrangement_use != CMPQ_ARRANGEMENT_NONE && j.arrangement_use != CMPQ_ARRANGEMENT_KEEP &&
        j.arrangement_use != CMPQ_ARRANGEMENT_REUSE)
        return CMPQ_EINVAL;
    if (!j.bits || !j.centroids || (j.n_out > 0 && !j.out_idx)) return CMPQ_EINVAL;
    const bool want_format = j.bit_set || j.n_set || j.counts_host || j.packed || j.chan_idx || j.lut || j.err_ch ||
                             j.err_total || j.sumsq;
    if (want_format && (!j.bit_set || !j.counts_host || !j.err_ch || !j.err_total)) return CMPQ_EINVAL;
    if (d_in > 0 && d_out > 0 && !j.W) return CMPQ_EINVAL;
    if (j.ldw < d_out) return CMPQ_ESHAPE;
    if (d_out > (j.dtype == CMPQ_F16 ? 32768 : 16384)) return CMPQ_ESHAPE;
    if (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;
    if (d_in >= ((int64_t)1 << 31)) return CMPQ_ESHAPE;
    if (d_in == 0)
        return want_format ? launch_error_totals(j.err_ch, j.sumsq, 0, j.err_total, static_cast<hipStream_t>(stream)) : CMPQ_OK;
    KmArgs a;
    a.W = j.W;
    a.d_in = d_in;
    a.d_out = d_out;
    a.ldw = j.ldw;
    a.bits = j.bits;
    a.out_idx = j.out_idx;
    a.n_out = j.n_out;
    a.ew = j.elem_weight;
    a.iters = j.iters;
    a.start_given = j.init == CMPQ_INIT_GIVEN;
    a.centroids = j.centroids;
    a.codes = j.codes;
    a.status = j.status;
    a.deferred = nullptr;
    a.seg = nullptr;
    a.fused = 0;
    a.row_of = nullptr;
    a.err_ch = nullptr;
    a.arr_keep = nullptr;
    a.arr_reuse = nullptr;
    a.arr_stride = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_kmeans(d_in, d_out))
        return CMPQ_EWORKSPACE;
    char *ws_row_of = static_cast<char *>(ws) + ws_kmeans_base(d_in);
    char *ws_tail = ws_row_of + align_up((size_t)d_in * sizeof(int32_t), 256);
    const bool hist_takes_it = kmeans_fast_eligible(a, j.dtype) && (j.algorithm != CMPQ_KMEANS_DIRECT || a.start_given);
    // levels alone (no codes, no stored format): only the histogram kernel leaves the coding pass out
    if (d_out > 0 && !j.codes && !want_format && !hist_takes_it) return CMPQ_EINVAL;
    if (j.arrangement_use != CMPQ_ARRANGEMENT_NONE) {
        // only the histogram kernel builds and reads arrangements; one is kept from all weights
        if (!j.arrangement || !hist_takes_it || reinterpret_cast<uintptr_t>(j.arrangement) % 16 != 0) return CMPQ_EINVAL;
        if (j.arrangement_use == CMPQ_ARRANGEMENT_KEEP && j.n_out > 0) return CMPQ_EINVAL;
        a.arr_stride = (int64_t)kmeans_hist_arrangement_stride(d_out);
        if (j.arrangement_use == CMPQ_ARRANGEMENT_KEEP) a.arr_keep = j.arrangement;
        else a.arr_reuse = j.arrangement;
    }
    if (want_format) {
        if (d_out > 1 << 20) return CMPQ_ESHAPE;
        if (const int rc = gather_pack_ptrs(d_in, d_out, j.bit_set, j.n_set, j.counts_host, j.packed, j.chan_idx, j.lut, a.pack))
            return rc;
        if (!hist_takes_it) {
            // the general kernels write dense codes; the stored format follows in a pass of its own
            if (d_out > 0 && !j.codes) return CMPQ_EINVAL;
            cmpq_kmeans_job plain = j;
            plain.bit_set = nullptr, plain.n_set = 0, plain.counts_host = nullptr, plain.packed = nullptr;
            plain.chan_idx = nullptr, plain.lut = nullptr, plain.sumsq = nullptr, plain.err_ch = nullptr;
            plain.err_total = nullptr;
            if (const int rc = cmpq_kmeans_quantize_job(&plain, ws, ws_bytes, stream)) return rc;
            return cmpq_pack_with_error(j.W, j.dtype, d_in, d_out, j.ldw, j.codes, j.bits, j.centroids, j.bit_set,
                                        j.n_set, j.counts_host, j.packed, j.chan_idx, j.lut, j.out_idx, j.n_out,
                                        j.sumsq, j.err_ch, j.err_total, ws_tail, cmpq_ws_pack_with_error(d_in), stream);
        }
        int32_t *row_of = reinterpret_cast<int32_t *>(ws_row_of);
        if (const int rc = launch_pack_index(j.bits, d_in, a.pack, row_of, s)) return rc;
        a.fused = 1;
        a.row_of = row_of;
        a.err_ch = j.err_ch;
    }
    if (j.n_out > 0) {
        int32_t *seg = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + align_up((size_t)d_in, 256));
        const int rc = launch_segment_offsets(j.out_idx, j.n_out, d_in, d_out, seg, s);
        if (rc != CMPQ_OK) return rc;
        a.seg = seg;
    }
    if (kmeans_fast_eligible(a, j.dtype)) {
        // the bucket kernel takes every channel itself
        // (so does a run from given levels, whichever implementation is named)
        if (hist_takes_it) {
            if (const int rc = launch_kmeans_hist(a, s)) return rc;
            return a.fused ? launch_error_totals(j.err_ch, j.sumsq, d_in, j.err_total, s) : CMPQ_OK;
        }
        a.deferred = static_cast<uint8_t *>(ws);
        const int rc = launch_kmeans_fast(a, s);
        if (rc != CMPQ_OK) return rc;
        return launch_kmeans<__half, false>(a, s);  // only the channels the first kernel deferred
    }
    if (j.dtype == CMPQ_F16)
        return j.elem_weight ? launch_kmeans<__half, true>(a, s) : launch_kmeans<__half, false>(a, s);
    return j.elem_weight ? launch_kmeans<float, true>(a, s) : launch_kmeans<float, false>(a, s);
}

extern "C" int cmpq_kmeans_quantize(const void *W, int dtype, int64_t d_in, int64_t d_out,
                                    int64_t ldw, const uint8_t *bits, const int32_t *out_idx,
                                    int64_t n_out, const float *elem_weight, int iters, int init,
                                    float *centroids, uint8_t *codes, void *ws, size_t ws_bytes,
                                    int32_t *status, void *stream) {
    cmpq_kmeans_job j = {};
    j.W = W;
    j.dtype = dtype;
    j.d_in = d_in;
    j.d_out = d_out;
    j.ldw = ldw;
    j.bits = bits;
    j.out_idx = out_idx;
    j.n_out = n_out;
    j.elem_weight = elem_weight;
    j.iters = iters;
    j.init = init;
    j.centroids = centroids;
    j.codes = codes;
    j.status = status;
    j.algorithm = CMPQ_KMEANS_HISTOGRAM;
    return cmpq_kmeans_quantize_job(&j, ws, ws_bytes, stream);
}
