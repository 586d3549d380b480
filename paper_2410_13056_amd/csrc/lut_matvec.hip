// The product with the deployed weight (Sec. 6 / Fig. 4 of arXiv 2410.13056): per width a
// table-driven product of the input with the packed codes of cmpq_pack, plus the rows of
// O_act and the entries of O_q.
//
//   Y[t,o] = sum_i X[t,i] * W_hat[i,o]
//
// The packed rows are input channels, so a row contributes X[t,i] * lut_i[code] to every
// output: the 2^b products X[t,i] * lut_i[c] are formed once per row and the rest is table
// look-ups and additions.  HBM bound: b/8 bytes per weight are read once per token.
//
//   * lut_matvec_kernel: one launch, two kinds of workgroup, each leaving one partial row
//     per token:
//       - a slab of 128 packed rows of one width times 2048 outputs (a lane 32 consecutive
//         outputs: exactly B words of a row; 32 rows per wavefront).  The per-row tables of
//         4 rows at a time sit in LDS (one entry per lane to fill); a code becomes the
//         address of its table entry with two instructions.  The 16 entries of a table lie
//         in 16 banks, so the look-ups of a wavefront never collide.
//         Width 2 looks two neighbouring codes up at once (pair tables).
//       - a slab of 32 rows of O_act (FP16 rows) times 2048 outputs.
//     The four wavefronts' sums are added in order.  A launch serves up to 8 products
//     (cmpq_lut_matvec_group): every layer owns a range of blockIdx.y.
//   * lut_matvec_finish_kernel: per output, the partial rows in order (packed slabs, O_act
//     slabs), then the column's O_q entries - every sum in a fixed order, so the result is
//     reproducible bit for bit.
//   * cmpq_outliers_by_column / cmpq_gather_channels prepare O_q and O_act for this once,
//     at quantization time.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / CMPQ_WAVE;
constexpr int kOutPerLane = 32;                        // 32 codes = B whole words
constexpr int kTileOut = CMPQ_WAVE * kOutPerLane;      // outputs per workgroup
constexpr int kMaxRowsPerWave = 32;                    // a workgroup's slab: 4 wavefronts x 8, 16 or 32 rows
constexpr int kGroup = 4;                              // rows whose tables are in LDS at once
constexpr int kMaxWidths = 4;

struct LmWidth {
    const uint32_t *packed;
    const int32_t *chan_idx;
    const uint16_t *lut;
    int64_t rows, words_per_row;
    int slab0;  // index of this width's first slab among all slabs
    int bits;
};

// One product of a launch, as the kernels see it.
struct LmArgs {
    LmWidth w[kMaxWidths];
    const __half *X;
    int64_t ldx, d_out;
    float *partial;                // [tokens][n_rows_total][d_out]
    const int32_t *act_idx;
    const __half *W_act;
    int64_t k_act, ld_act;
    int n_widths, rows_per_wave;
    int n_lut_slabs, n_act_slabs;  // a layer's blockIdx.y range: O_act slabs first, then the packed slabs
    int n_rows_total;              // partial rows per token: packed slabs, then O_act slabs
    int act_vec_ok;                // W_act rows may be read 16 bytes at a time
    int tiles;                     // tiles of 2048 outputs
    int y0;                        // first blockIdx.y of this layer
};

constexpr int kMaxLayers = CMPQ_MAX_GROUP;

struct LmGroup {
    LmArgs l[kMaxLayers];
    int n_layers;
};

constexpr int kRedStride = CMPQ_WAVE + 1;  // sums of output k of all lanes: 64 floats, padded by one
constexpr int kRedHalf = kOutPerLane / 2;  // the sums meet in LDS in two halves of 16 outputs per lane
constexpr int kRedFloats = kRedHalf * kRedStride;

// The four wavefronts' sums of a 2048-output tile, added in wavefront order, into a partial
// row.  Called once by every lane of the workgroup.  Lanes write with stride 1 and read with
// stride 65: no bank is hit twice by a half-wavefront either way.  Two halves, so that the
// LDS of a workgroup stays small enough for five workgroups per compute unit.
__device__ __forceinline__ void store_partial(const float (&acc)[kOutPerLane], float (*red)[kRedFloats],
                                              float *__restrict__ prow, int64_t d_out) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        __syncthreads();  // the sums reuse the LDS of the tables (and of the first half)
#pragma unroll
        for (int k = 0; k < kRedHalf; ++k) red[wave][k * kRedStride + lane] = acc[h * kRedHalf + k];
        __syncthreads();
        // lane l holds outputs 32 l .. 32 l + 31 of the tile; this half covers k = 16 h .. 16 h + 15
        for (int c = threadIdx.x; c < kTileOut / 2; c += kThreads) {
            const int l = c / kRedHalf, k = c % kRedHalf;
            const int64_t o = (int64_t)blockIdx.x * kTileOut + l * kOutPerLane + h * kRedHalf + k;
            if (o < d_out) {
                const int at = k * kRedStride + l;
                float t = red[0][at];
#pragma unroll
                for (int wv = 1; wv < kWaves; ++wv) t += red[wv][at];
                prow[o] = t;
            }
        }
    }
}

// Code k of a lane's 32 codes held in w[0..B-1] (one bit-field extract, two instructions
// where the code straddles two words).
template <int B>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&w)[B], int k) {
    const int bit = k * B, idx = bit >> 5, sh = bit & 31;
    if (sh + B <= 32) return __builtin_amdgcn_ubfe(w[idx], sh, B);
    return __builtin_amdgcn_alignbit(w[idx + 1 < B ? idx + 1 : idx], w[idx], sh) & ((1u << B) - 1u);
}

// (code << 2) + base in one instruction.  Written out because the compiler otherwise turns
// the extract-then-shift into shift-mask-add, one instruction more per weight.
__device__ __forceinline__ uint32_t entry_offset(uint32_t code, uint32_t base) {
    uint32_t r;
    asm("v_lshl_add_u32 %0, %1, 2, %2" : "=v"(r) : "v"(code), "v"(base));
    return r;
}

template <int B>
__device__ __forceinline__ void lut_slab(const LmArgs &a, const LmWidth &wd, int slab,
                                         float (*tbl_all)[2][kGroup * 16], float (*red)[kRedFloats]) {
    const __half *__restrict__ X = a.X;
    const int64_t ldx = a.ldx, d_out = a.d_out;
    const int rows_per_wave = a.rows_per_wave, n_rows_total = a.n_rows_total;
    float *__restrict__ partial = a.partial;
    constexpr int K = 1 << B;
    // per wavefront: two buffers of kGroup row tables (K floats each)
    float(*tbl)[2][kGroup * 16] = tbl_all;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t token = blockIdx.z;
    const __half *x = X + token * ldx;
    const int64_t word0 = (int64_t)blockIdx.x * (kTileOut / 32) * B + (int64_t)lane * B;
    const int64_t r0 = ((int64_t)slab * kWaves + wave) * rows_per_wave;
    const int64_t r1 = min(wd.rows, r0 + rows_per_wave);
    float acc[kOutPerLane];
#pragma unroll
    for (int k = 0; k < kOutPerLane; ++k) acc[k] = 0.f;

    // entry (row g, level c) of a group's tables is filled by lane g*K + c
    const int fill_g = lane / K, fill_c = lane % K;
    auto table_entry = [&](int64_t r) -> float {
        if (fill_g >= kGroup || r + fill_g >= r1) return 0.f;
        const int64_t row = r + fill_g;
        const float xi = __half2float(x[wd.chan_idx[row]]);
        return xi * __half2float(__ushort_as_half(wd.lut[row * K + fill_c]));
    };
    // a lane's B words of a row: one vector load when they all exist
    const bool full = word0 + B <= wd.words_per_row;
    auto load_words = [&](int64_t r, uint32_t (&w)[kGroup][B]) {
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const uint32_t *p = wd.packed + (r + g) * wd.words_per_row + word0;
            if (r + g < r1 && full) {
                typedef uint32_t WordsB __attribute__((ext_vector_type(B), aligned(4)));
                const WordsB v = __builtin_nontemporal_load(reinterpret_cast<const WordsB *>(p));  // dword-aligned vector load; a token reads the codes once
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = v[j];
            } else {
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = (r + g < r1 && word0 + j < wd.words_per_row) ? p[j] : 0u;
            }
        }
    };

    if (r0 < r1) {
        // The tables of a group are written one group ahead, into the buffer the look-ups of the
        // group before have just left, so that the write has a whole group of look-ups to land
        // in; the table entries themselves are fetched two groups ahead, the words one.
        uint32_t w[kGroup][B], wn[kGroup][B];
        const bool fills = kGroup * K >= CMPQ_WAVE || lane < kGroup * K;
        if (fills) tbl[wave][0][lane % (kGroup * K)] = table_entry(r0);
        float e = r0 + kGroup < r1 ? table_entry(r0 + kGroup) : 0.f, en = 0.f;
        load_words(r0, w);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int buf = 0;
        for (int64_t r = r0; r < r1; r += kGroup) {
            if (r + kGroup < r1) {
                if (fills) tbl[wave][buf ^ 1][lane % (kGroup * K)] = e;
                load_words(r + kGroup, wn);
            }
            if (r + 2 * kGroup < r1) en = table_entry(r + 2 * kGroup);
            // byte offset of this wavefront's current buffer; code * 4 is added to it with one
            // shift-and-add
            const char *base = reinterpret_cast<const char *>(&tbl[0][0][0]);
            const uint32_t wb = (uint32_t)((wave * 2 + buf) * (kGroup * 16 * 4));
#pragma unroll
            for (int g = 0; g < kGroup; ++g) {
                // rows past the end have all-zero tables: their look-ups add 0
#pragma unroll
                for (int k = 0; k < kOutPerLane; ++k)
                    acc[k] += *reinterpret_cast<const float *>(base + g * K * 4 + entry_offset(code_at<B>(w[g], k), wb));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            buf ^= 1;
            e = en;
#pragma unroll
            for (int g = 0; g < kGroup; ++g)
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = wn[g][j];
        }
    }
    store_partial(acc, red, partial + (token * n_rows_total + wd.slab0 + slab) * d_out, d_out);
}

// Field p of `bits` bits of a lane's words (two instructions where it straddles two words).
template <int B, int PB>
__device__ __forceinline__ uint32_t field_at(const uint32_t (&w)[B], int p) {
    const int bit = p * PB, idx = bit >> 5, sh = bit & 31;
    if (sh + PB <= 32) return __builtin_amdgcn_ubfe(w[idx], sh, PB);
    return __builtin_amdgcn_alignbit(w[idx + 1 < B ? idx + 1 : idx], w[idx], sh) & ((1u << PB) - 1u);
}

// Width 2: two neighbouring codes are looked up at once.  Per row two tables indexed by the
// pair (c0 | c1 << B): A[pair] = x * lut[c0] for the even output, B[pair] = x * lut[c1] for the
// odd one, read by one two-address LDS load.  One extract and one shift-and-add serve two
// weights, so a weight costs 2 instead of 3 vector instructions; the sums are the same
// products added in the same order.  A table of 16 entries lies in 16 banks: no conflicts.
// (Written for any width whose pair table fits a wavefront; with width 3 the 64-entry tables
// wrap around the LDS banks, the look-ups of a wavefront collide and the kernel is slower than
// with single look-ups, so width 3 does not use it.)  Same slab shape, prefetch and double
// buffering as lut_slab.
template <int B>
__device__ __forceinline__ void lut_slab_pairs(const LmArgs &a, const LmWidth &wd, int slab, float *smem,
                                               float (*red)[kRedFloats]) {
    constexpr int K = 1 << B, PB = 2 * B, KP = 1 << PB;   // levels, bits of a pair, entries of a pair table
    constexpr int kRowsPerFill = CMPQ_WAVE / KP < kGroup ? CMPQ_WAVE / KP : kGroup;  // rows one pass over the lanes fills
    constexpr int kFills = kGroup / kRowsPerFill;
    constexpr int kRowFloats = 2 * KP;                     // A then B
    constexpr int kBufFloats = kGroup * kRowFloats;
    static_assert(KP <= CMPQ_WAVE && kGroup % kRowsPerFill == 0, "pair tables are filled by whole wavefronts");
    const __half *__restrict__ X = a.X;
    const int64_t d_out = a.d_out;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t token = blockIdx.z;
    const __half *x = X + token * a.ldx;
    const int64_t word0 = (int64_t)blockIdx.x * (kTileOut / 32) * B + (int64_t)lane * B;
    const int64_t r0 = ((int64_t)slab * kWaves + wave) * a.rows_per_wave;
    const int64_t r1 = min(wd.rows, r0 + a.rows_per_wave);
    float acc[kOutPerLane];
#pragma unroll
    for (int k = 0; k < kOutPerLane; ++k) acc[k] = 0.f;

    // pass f over the lanes fills the tables of row f * kRowsPerFill + lane / KP, entry lane % KP
    const int fill_row = lane / KP, fill_e = lane % KP;
    auto table_entries = [&](int64_t r, float (&ea)[kFills], float (&eb)[kFills]) {
#pragma unroll
        for (int f = 0; f < kFills; ++f) {
            const int64_t row = r + f * kRowsPerFill + fill_row;
            ea[f] = 0.f;
            eb[f] = 0.f;
            if (fill_row < kRowsPerFill && row < r1) {
                const float xi = __half2float(x[wd.chan_idx[row]]);
                ea[f] = xi * __half2float(__ushort_as_half(wd.lut[row * K + (fill_e & (K - 1))]));
                eb[f] = xi * __half2float(__ushort_as_half(wd.lut[row * K + (fill_e >> B)]));
            }
        }
    };
    const bool full = word0 + B <= wd.words_per_row;
    auto load_words = [&](int64_t r, uint32_t (&w)[kGroup][B]) {
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const uint32_t *p = wd.packed + (r + g) * wd.words_per_row + word0;
            if (r + g < r1 && full) {
                typedef uint32_t WordsB __attribute__((ext_vector_type(B), aligned(4)));
                const WordsB v = __builtin_nontemporal_load(reinterpret_cast<const WordsB *>(p));
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = v[j];
            } else {
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = (r + g < r1 && word0 + j < wd.words_per_row) ? p[j] : 0u;
            }
        }
    };

    if (r0 < r1) {
        uint32_t w[kGroup][B], wn[kGroup][B];
        float ea[kFills], eb[kFills], ean[kFills], ebn[kFills];
        table_entries(r0, ea, eb);
        load_words(r0, w);
        int buf = 0;
        for (int64_t r = r0; r < r1; r += kGroup) {
            float *mine = smem + (wave * 2 + buf) * kBufFloats;
#pragma unroll
            for (int f = 0; f < kFills; ++f) {
                if (fill_row < kRowsPerFill) {
                    float *row_tbl = mine + (f * kRowsPerFill + fill_row) * kRowFloats;
                    row_tbl[fill_e] = ea[f];
                    row_tbl[KP + fill_e] = eb[f];
                }
            }
            if (r + kGroup < r1) {
                table_entries(r + kGroup, ean, ebn);
                load_words(r + kGroup, wn);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const char *base = reinterpret_cast<const char *>(smem);
            const uint32_t wb = (uint32_t)((wave * 2 + buf) * (kBufFloats * 4));
#pragma unroll
            for (int g = 0; g < kGroup; ++g) {
                // rows past the end have all-zero tables: their look-ups add 0
#pragma unroll
                for (int p = 0; p < kOutPerLane / 2; ++p) {
                    const char *at = base + g * (kRowFloats * 4) + entry_offset(field_at<B, PB>(w[g], p), wb);
                    acc[2 * p] += *reinterpret_cast<const float *>(at);
                    acc[2 * p + 1] += *reinterpret_cast<const float *>(at + KP * 4);
                }
            }
            __builtin_amdgcn_wave_barrier();
            buf ^= 1;
#pragma unroll
            for (int f = 0; f < kFills; ++f) {
                ea[f] = ean[f];
                eb[f] = ebn[f];
            }
#pragma unroll
            for (int g = 0; g < kGroup; ++g)
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = wn[g][j];
        }
    }
    store_partial(acc, red, a.partial + (token * a.n_rows_total + wd.slab0 + slab) * d_out, d_out);
}

// The variant that adds up in FP16 (the paper's product keeps FP16 throughout, Sec. 6): the
// products x * level are rounded to FP16, and a wavefront adds those of its run of at most 32
// rows of a slab in FP16, two outputs per packed addition; the run's sums are then widened
// to fp32 and take the same way as in lut_slab (added over wavefronts, slabs, O_act and O_q in
// fp32, in a fixed order).  Every width looks two neighbouring codes up at once: per row a
// table of 2^(2B) pairs (product of the even output's code, product of the odd one's), 4
// bytes an entry, built from the row's 2^B products with two LDS reads per entry (for width
// 4: four entries per lane and row from one 8-byte read, one 2-byte read and one 16-byte
// store).  A weight then costs half an extract, half a shift-and-add, half an LDS read and
// half a packed addition.  Tables of 64 and 256 entries wrap around the LDS banks, so their
// reads collide; with 4-byte entries that costs less than the instructions saved (with the
// 8-byte entries of fp32 pairs it did not).  Same slab shape, prefetch and double buffering
// as lut_slab.
constexpr int kHalfPairBytes = kGroup * 256 * 4;               // pair tables of a group of rows at width 4
constexpr int kHalfBufBytes = kHalfPairBytes + kGroup * 16 * 2;  // + the rows' own products
constexpr int kHalfLdsBytes = kWaves * 2 * kHalfBufBytes;

template <int B>
__device__ __forceinline__ void lut_slab_half(const LmArgs &a, const LmWidth &wd, int slab, unsigned char *smem,
                                              float (*red)[kRedFloats]) {
    constexpr int K = 1 << B, PB = 2 * B, KP = 1 << PB;
    const __half *__restrict__ X = a.X;
    const int64_t d_out = a.d_out;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t token = blockIdx.z;
    const __half *x = X + token * a.ldx;
    const int64_t word0 = (int64_t)blockIdx.x * (kTileOut / 32) * B + (int64_t)lane * B;
    const int64_t r0 = ((int64_t)slab * kWaves + wave) * a.rows_per_wave;
    const int64_t r1 = min(wd.rows, r0 + a.rows_per_wave);
    __half2 acc2[kOutPerLane / 2];
#pragma unroll
    for (int p = 0; p < kOutPerLane / 2; ++p) acc2[p] = __half2{__ushort_as_half(0), __ushort_as_half(0)};

    // product (row g, level c) of a group is formed by lane g * K + c
    const int fill_g = lane / K, fill_c = lane % K;
    auto product = [&](int64_t r) -> uint32_t {
        if (fill_g >= kGroup || r + fill_g >= r1) return 0u;  // rows past the end: tables of zeros
        const int64_t row = r + fill_g;
        const float xi = __half2float(x[wd.chan_idx[row]]);
        return __half_as_ushort(__float2half_rn(xi * __half2float(__ushort_as_half(wd.lut[row * K + fill_c]))));
    };
    const bool full = word0 + B <= wd.words_per_row;
    auto load_words = [&](int64_t r, uint32_t (&w)[kGroup][B]) {
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            const uint32_t *p = wd.packed + (r + g) * wd.words_per_row + word0;
            if (r + g < r1 && full) {
                typedef uint32_t WordsB __attribute__((ext_vector_type(B), aligned(4)));
                const WordsB v = __builtin_nontemporal_load(reinterpret_cast<const WordsB *>(p));
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = v[j];
            } else {
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = (r + g < r1 && word0 + j < wd.words_per_row) ? p[j] : 0u;
            }
        }
    };

    if (r0 < r1) {
        uint32_t w[kGroup][B], wn[kGroup][B];
        uint32_t e = product(r0), en = 0u;
        load_words(r0, w);
        int buf = 0;
        for (int64_t r = r0; r < r1; r += kGroup) {
            unsigned char *mine = smem + (wave * 2 + buf) * kHalfBufBytes;
            uint32_t *pair = reinterpret_cast<uint32_t *>(mine);
            uint16_t *own = reinterpret_cast<uint16_t *>(mine + kHalfPairBytes);  // [row of the group][level]
            if (kGroup * K >= CMPQ_WAVE || lane < kGroup * K) own[lane % (kGroup * K)] = (uint16_t)e;
            if (r + kGroup < r1) {
                en = product(r + kGroup);
                load_words(r + kGroup, wn);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if constexpr (B == 4) {
                // lane: odd output's code c1 = lane / 4, even output's codes 4 (lane % 4) .. + 3
                const int c1 = lane >> 2, c0 = (lane & 3) * 4;
#pragma unroll
                for (int g = 0; g < kGroup; ++g) {
                    const uint32_t hi = (uint32_t)own[g * K + c1] << 16;
                    const uint2 q = *reinterpret_cast<const uint2 *>(own + g * K + c0);
                    uint4 v;
                    v.x = (q.x & 0xffffu) | hi;
                    v.y = (q.x >> 16) | hi;
                    v.z = (q.y & 0xffffu) | hi;
                    v.w = (q.y >> 16) | hi;
                    *reinterpret_cast<uint4 *>(pair + g * KP + c1 * K + c0) = v;
                }
            } else {
#pragma unroll
                for (int t0 = 0; t0 < kGroup * KP; t0 += CMPQ_WAVE) {
                    const int t = t0 + lane;
                    if (kGroup * KP % CMPQ_WAVE == 0 || t < kGroup * KP) {
                        const int g = t / KP, ent = t % KP;
                        pair[t] = (uint32_t)own[g * K + (ent & (K - 1))] | ((uint32_t)own[g * K + (ent >> B)] << 16);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const char *base = reinterpret_cast<const char *>(smem);
            const uint32_t wb = (uint32_t)((wave * 2 + buf) * kHalfBufBytes);
#pragma unroll
            for (int g = 0; g < kGroup; ++g) {
#pragma unroll
                for (int p = 0; p < kOutPerLane / 2; ++p) {
                    const uint32_t v = *reinterpret_cast<const uint32_t *>(base + g * (KP * 4) + entry_offset(field_at<B, PB>(w[g], p), wb));
                    acc2[p] = __hadd2(acc2[p], __half2{__ushort_as_half((unsigned short)(v & 0xffffu)), __ushort_as_half((unsigned short)(v >> 16))});
                }
            }
            __builtin_amdgcn_wave_barrier();
            buf ^= 1;
            e = en;
#pragma unroll
            for (int g = 0; g < kGroup; ++g)
#pragma unroll
                for (int j = 0; j < B; ++j) w[g][j] = wn[g][j];
        }
    }
    float acc[kOutPerLane];
#pragma unroll
    for (int p = 0; p < kOutPerLane / 2; ++p) {
        acc[2 * p] = __low2float(acc2[p]);
        acc[2 * p + 1] = __high2float(acc2[p]);
    }
    store_partial(acc, red, a.partial + (token * a.n_rows_total + wd.slab0 + slab) * d_out, d_out);
}

// A slab of O_act: 8 rows of FP16 weights per wavefront times their inputs (few rows, so
// short slabs: the loop over rows is bound by latency).  A lane reads its 32 outputs of a
// row as four 16-byte pieces, two rows in flight; the rows' inputs are fetched up front,
// one per lane.
constexpr int kActRowsPerWave = 8;

__device__ __forceinline__ void act_slab(const LmArgs &a, int slab, float (*red)[kRedFloats]) {
    const __half *__restrict__ X = a.X;
    const int64_t ldx = a.ldx, d_out = a.d_out;
    float *__restrict__ partial = a.partial;
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t token = blockIdx.z;
    const __half *x = X + token * ldx;
    const int64_t o0 = (int64_t)blockIdx.x * kTileOut + (int64_t)lane * kOutPerLane;
    const int64_t r0 = ((int64_t)slab * kWaves + wave) * kActRowsPerWave;
    const int n = (int)max((int64_t)0, min(a.k_act - r0, (int64_t)kActRowsPerWave));
    float acc[kOutPerLane];
#pragma unroll
    for (int k = 0; k < kOutPerLane; ++k) acc[k] = 0.f;
    const float x_mine = lane < n ? __half2float(x[a.act_idx[r0 + lane]]) : 0.f;
    // every row's input in a scalar register (rows past the count: 0), read before lanes part ways
    float xs[kActRowsPerWave];
#pragma unroll
    for (int j = 0; j < kActRowsPerWave; ++j)
        xs[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x_mine), j));
    const bool vec = a.act_vec_ok && o0 + kOutPerLane <= d_out;
    if (vec) {
#pragma unroll
        for (int j = 0; j < kActRowsPerWave; j += 2) {
            if (j >= n) break;
            uint4 raw[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                // the second row of an odd count is read again from the first: its input is 0
                const int64_t r = r0 + (j + u < n ? j + u : j);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    raw[u][q] = reinterpret_cast<const uint4 *>(a.W_act + r * a.ld_act + o0)[q];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const float xi = xs[j + u];
                const __half2 *h = reinterpret_cast<const __half2 *>(raw[u]);
#pragma unroll
                for (int k = 0; k < kOutPerLane / 2; ++k) {
                    const float2 wv = __half22float2(h[k]);
                    acc[2 * k] = fmaf(xi, wv.x, acc[2 * k]);
                    acc[2 * k + 1] = fmaf(xi, wv.y, acc[2 * k + 1]);
                }
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < kActRowsPerWave; ++j) {
            if (j >= n) break;
            const float xi = xs[j];
            const __half *wrow = a.W_act + (r0 + j) * a.ld_act + o0;
#pragma unroll
            for (int k = 0; k < kOutPerLane; ++k)
                if (o0 + k < d_out) acc[k] = fmaf(xi, __half2float(wrow[k]), acc[k]);
        }
    }
    store_partial(acc, red, partial + (token * a.n_rows_total + a.n_lut_slabs + slab) * d_out, d_out);
}

// grid: (tiles of 2048 outputs of the widest layer; per layer its O_act slabs, then its packed
// slabs of all widths one after the other; tokens)
__global__ __launch_bounds__(kThreads) void lut_matvec_kernel(LmGroup g) {
    // the tables of the look-ups and, after them, the wavefronts' sums share one piece of LDS
    __shared__ float smem[kWaves * kRedFloats];
    float(*tbl)[2][kGroup * 16] = reinterpret_cast<float(*)[2][kGroup * 16]>(smem);
    float(*red)[kRedFloats] = reinterpret_cast<float(*)[kRedFloats]>(smem);
    static_assert(kWaves * 2 * kGroup * 2 * 16 <= kWaves * kRedFloats, "pair tables fit the shared piece");
    int l = 0;
    while (l + 1 < g.n_layers && (int)blockIdx.y >= g.l[l + 1].y0) ++l;
    const LmArgs &a = g.l[l];
    if ((int)blockIdx.x >= a.tiles) return;
    int y = (int)blockIdx.y - a.y0;
    if (y < a.n_act_slabs) {
        act_slab(a, y, red);
        return;
    }
    y -= a.n_act_slabs;
    int j = 0;
    while (j + 1 < a.n_widths && y >= a.w[j + 1].slab0) ++j;
    const LmWidth &wd = a.w[j];
    const int slab = y - wd.slab0;
    switch (wd.bits) {
        case 1: lut_slab<1>(a, wd, slab, tbl, red); break;
        case 2: lut_slab_pairs<2>(a, wd, slab, smem, red); break;
        case 3: lut_slab<3>(a, wd, slab, tbl, red); break;
        default: lut_slab<4>(a, wd, slab, tbl, red); break;
    }
}

// The same launch with the packed rows added up in FP16 (lut_slab_half); the O_act slabs are
// the fp32 ones.
__global__ __launch_bounds__(kThreads) void lut_matvec_half_kernel(LmGroup g) {
    __shared__ __align__(16) unsigned char smem[kHalfLdsBytes];
    static_assert(kHalfLdsBytes >= kWaves * kRedFloats * (int)sizeof(float), "the wavefronts' sums fit the shared piece");
    float(*red)[kRedFloats] = reinterpret_cast<float(*)[kRedFloats]>(smem);
    int l = 0;
    while (l + 1 < g.n_layers && (int)blockIdx.y >= g.l[l + 1].y0) ++l;
    const LmArgs &a = g.l[l];
    if ((int)blockIdx.x >= a.tiles) return;
    int y = (int)blockIdx.y - a.y0;
    if (y < a.n_act_slabs) {
        act_slab(a, y, red);
        return;
    }
    y -= a.n_act_slabs;
    int j = 0;
    while (j + 1 < a.n_widths && y >= a.w[j + 1].slab0) ++j;
    const LmWidth &wd = a.w[j];
    const int slab = y - wd.slab0;
    switch (wd.bits) {
        case 1: lut_slab_half<1>(a, wd, slab, smem, red); break;
        case 2: lut_slab_half<2>(a, wd, slab, smem, red); break;
        case 3: lut_slab_half<3>(a, wd, slab, smem, red); break;
        default: lut_slab_half<4>(a, wd, slab, smem, red); break;
    }
}

constexpr int kFinCols = 16;  // outputs per workgroup
constexpr int kFinRuns = kThreads / kFinCols;

// 16 consecutive outputs per workgroup of 256 lanes.
//   * O_q: 16 lanes per column; lane l takes the column's entries l, l+16, ... (8 in flight)
//     and adds them in that order.
//   * partial rows: cut into 16 runs of consecutive rows; lane (run, output) adds its run in
//     row order (4 loads in flight).
// Per output, the 16 run sums are added in run order, then the 16 O_q sums in lane order.
struct FinArgs {
    const __half *X;
    int64_t ldx, d_out;
    const float *partial;
    const int32_t *colptr, *row_idx;
    const float *delta;
    float *Y;
    int64_t ldy;
    int n_rows_total;
    int x0;  // first blockIdx.x of this layer
};

struct FinGroup {
    FinArgs l[kMaxLayers];
    int n_layers;
};

__global__ __launch_bounds__(kThreads) void lut_matvec_finish_kernel(FinGroup g) {
    int l = 0;
    while (l + 1 < g.n_layers && (int)blockIdx.x >= g.l[l + 1].x0) ++l;
    const FinArgs &a = g.l[l];
    const __half *__restrict__ X = a.X;
    const int64_t ldx = a.ldx, d_out = a.d_out, ldy = a.ldy;
    const float *__restrict__ partial = a.partial;
    const int n_rows_total = a.n_rows_total;
    const int32_t *__restrict__ colptr = a.colptr;
    const int32_t *__restrict__ row_idx = a.row_idx;
    const float *__restrict__ delta = a.delta;
    float *__restrict__ Y = a.Y;
    constexpr int U = 8;
    __shared__ float part[kFinRuns][kFinCols + 1];
    __shared__ float sp[kFinCols][kFinRuns + 1];
    const int hi = threadIdx.x / kFinCols, lo = threadIdx.x % kFinCols;
    const int64_t token = blockIdx.y;
    const int64_t o0 = (int64_t)((int)blockIdx.x - a.x0) * kFinCols;
    const __half *x = X + token * ldx;
    // O_q of column o0 + hi, entries lo, lo + 16, ...
    float t = 0.f;
    if (colptr && o0 + hi < d_out) {
        const int e1 = colptr[o0 + hi + 1];
        for (int e = colptr[o0 + hi] + lo; e < e1; e += 16 * U) {
            int32_t r[U];
            float d[U], xv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int ee = e + 16 * u;
                const bool ok = ee < e1;
                r[u] = ok ? row_idx[ee] : -1;
                d[u] = ok ? delta[ee] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) xv[u] = r[u] >= 0 ? __half2float(x[r[u]]) : 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) t = fmaf(xv[u], d[u], t);
        }
    }
    sp[hi][lo] = t;
    // partial rows of output o0 + lo, run hi
    float y = 0.f;
    if (o0 + lo < d_out) {
        const int per = (n_rows_total + kFinRuns - 1) / kFinRuns;
        const int r0 = hi * per, r1 = min(n_rows_total, r0 + per);
        const float *p = partial + token * n_rows_total * d_out + o0 + lo;
        int r = r0;
        for (; r + 4 <= r1; r += 4) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = p[(int64_t)(r + u) * d_out];
#pragma unroll
            for (int u = 0; u < 4; ++u) y += v[u];
        }
        for (; r < r1; ++r) y += p[(int64_t)r * d_out];
    }
    part[hi][lo] = y;
    __syncthreads();
    if (threadIdx.x < kFinCols && o0 + threadIdx.x < d_out) {
        float dense = 0.f, sparse = 0.f;
#pragma unroll
        for (int q = 0; q < kFinRuns; ++q) dense += part[q][threadIdx.x];
#pragma unroll
        for (int q = 0; q < 16; ++q) sparse += sp[threadIdx.x][q];
        Y[token * ldy + o0 + threadIdx.x] = dense + sparse;
    }
}

template <typename TW>
__global__ __launch_bounds__(kThreads) void gather_channels_kernel(const TW *__restrict__ W, int64_t d_out,
                                                                    int64_t ldw,
                                                                    const int32_t *__restrict__ act_idx,
                                                                    uint16_t *__restrict__ W_act,
                                                                    int64_t ld_act) {
    const int64_t j = blockIdx.y;
    const int64_t i = act_idx[j];
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < d_out; o += (int64_t)gridDim.x * kThreads)
        W_act[j * ld_act + o] = __half_as_ushort(__float2half_rn(load_as_f32<TW>(W, i * ldw + o)));
}

// ---- O_q by output column

__global__ void obc_zero_kernel(int32_t *cnt, int64_t n) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (int64_t)gridDim.x * blockDim.x)
        cnt[t] = 0;
}

__global__ void obc_count_kernel(const int32_t *__restrict__ out_idx, int64_t n_out, int64_t d_out,
                                 int32_t *__restrict__ cnt) {
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_out; e += (int64_t)gridDim.x * blockDim.x)
        atomicAdd(&cnt[out_idx[e] % d_out], 1);
}

// One workgroup: exclusive prefix of the column counts -> colptr and the scatter cursors.
__global__ __launch_bounds__(1024) void obc_scan_kernel(const int32_t *__restrict__ cnt, int64_t d_out,
                                                        int32_t *__restrict__ colptr,
                                                        int32_t *__restrict__ cursor) {
    __shared__ uint32_t scan[17];
    uint32_t run = 0;
    for (int64_t base = 0; base < d_out; base += 1024) {
        const int64_t o = base + threadIdx.x;
        const uint32_t c = o < d_out ? (uint32_t)cnt[o] : 0u;
        uint32_t total;
        const uint32_t before = run + block_scan_excl_u32(c, scan, &total);
        if (o < d_out) {
            colptr[o] = (int32_t)before;
            cursor[o] = (int32_t)before;
        }
        run += total;
    }
    if (threadIdx.x == 0) colptr[d_out] = (int32_t)run;
}

__global__ void obc_scatter_kernel(const int32_t *__restrict__ out_idx, const uint16_t *__restrict__ out_val,
                                   int64_t n_out, int64_t d_out, const float *__restrict__ centroids,
                                   const uint8_t *__restrict__ codes, int32_t *__restrict__ cursor,
                                   int32_t *__restrict__ row_idx, float *__restrict__ delta) {
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_out; e += (int64_t)gridDim.x * blockDim.x) {
        const int32_t lin = out_idx[e];
        const int32_t i = lin / (int32_t)d_out, o = lin % (int32_t)d_out;
        const float level = __half2float(__float2half_rn(centroids[(int64_t)i * CMPQ_KMAX + (codes[lin] & 15)]));
        const int32_t pos = atomicAdd(&cursor[o], 1);
        row_idx[pos] = i;
        delta[pos] = __half2float(__ushort_as_half(out_val[e])) - level;
    }
}

// The scatter leaves a column's entries in any order.  Channels are distinct inside a
// column, so ordering by channel gives one well-defined result.  A wavefront per column:
// an entry's final place is the number of entries of the column with a smaller channel
// (every lane walks the whole column; columns hold a few hundred entries).  A column longer
// than kRankLimit is ordered by one lane with a shell sort instead.
constexpr int kRankLimit = 2048;

__global__ __launch_bounds__(kThreads) void obc_order_kernel(const int32_t *__restrict__ colptr, int64_t d_out,
                                                              const int32_t *__restrict__ tmp_row,
                                                              const float *__restrict__ tmp_delta,
                                                              int32_t *__restrict__ row_idx,
                                                              float *__restrict__ delta) {
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = wave_index();
    const int64_t o = (int64_t)blockIdx.x * kWaves + wave;
    if (o >= d_out) return;
    const int b = colptr[o], n = colptr[o + 1] - b;
    if (n <= kRankLimit) {
        for (int e = lane; e < n; e += CMPQ_WAVE) {
            const int32_t mine = tmp_row[b + e];
            int rank = 0;
            for (int f = 0; f < n; ++f) rank += tmp_row[b + f] < mine;
            row_idx[b + rank] = mine;
            delta[b + rank] = tmp_delta[b + e];
        }
        return;
    }
    for (int e = lane; e < n; e += CMPQ_WAVE) {
        row_idx[b + e] = tmp_row[b + e];
        delta[b + e] = tmp_delta[b + e];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane != 0) return;
    int32_t *r = row_idx + b;
    float *d = delta + b;
    int gap = 1;
    while (gap < n / 3) gap = 3 * gap + 1;
    for (; gap >= 1; gap /= 3) {
        for (int i = gap; i < n; ++i) {
            const int32_t kr = r[i];
            const float kd = d[i];
            int j = i;
            while (j >= gap && r[j - gap] > kr) {
                r[j] = r[j - gap];
                d[j] = d[j - gap];
                j -= gap;
            }
            r[j] = kr;
            d[j] = kd;
        }
    }
}

int64_t total_slabs(const int64_t *counts, int n_set, int rows_per_wave) {
    int64_t s = 0;
    for (int j = 0; j < n_set; ++j) s += cdiv(counts[j] > 0 ? counts[j] : 0, (int64_t)kWaves * rows_per_wave);
    return s;
}

}  // namespace

// counts | cursors | channel and delta of every entry in scatter order
size_t cmpq_ws_outliers_by_column(int64_t d_out, int64_t n_out) {
    return align_up((size_t)(d_out + 1) * sizeof(int32_t), 256) * 2 + align_up((size_t)n_out * 4, 256) * 2;
}

// Upper bound without the per-width counts: every width and O_act may end with a partly
// filled slab.
size_t cmpq_ws_lut_matvec(int64_t d_in, int64_t d_out, int64_t m) {
    const int64_t slabs = cdiv(d_in, (int64_t)kWaves * 8) + kMaxWidths + 2;  // the smallest slabs
    return align_up((size_t)m * (size_t)slabs * (size_t)d_out * sizeof(float), 256);
}

extern "C" int cmpq_gather_channels(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                                    const int32_t *act_idx, int64_t k_act, uint16_t *W_act,
                                    int64_t ld_act, void *stream) {
    if (d_in < 0 || d_out < 0 || k_act < 0 || k_act > d_in) return CMPQ_EINVAL;
    if (dtype != CMPQ_F16 && dtype != CMPQ_F32) return CMPQ_EINVAL;
    if (k_act == 0 || d_out == 0) return CMPQ_OK;
    if (!W || !act_idx || !W_act) return CMPQ_EINVAL;
    if (ldw < d_out || ld_act < d_out || k_act > 65535) return CMPQ_ESHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t gx = cdiv(d_out, kThreads);
    if (gx > 64) gx = 64;
    const dim3 grid((unsigned)gx, (unsigned)k_act);
    if (dtype == CMPQ_F16)
        gather_channels_kernel<__half><<<grid, kThreads, 0, s>>>(static_cast<const __half *>(W), d_out, ldw, act_idx, W_act, ld_act);
    else
        gather_channels_kernel<float><<<grid, kThreads, 0, s>>>(static_cast<const float *>(W), d_out, ldw, act_idx, W_act, ld_act);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

extern "C" int cmpq_outliers_by_column(const int32_t *out_idx, const uint16_t *out_val, int64_t n_out,
                                       int64_t d_in, int64_t d_out, const float *centroids,
                                       const uint8_t *codes, int32_t *colptr, int32_t *row_idx,
                                       float *delta, void *ws, size_t ws_bytes, void *stream) {
    if (n_out < 0 || d_in < 0 || d_out < 0 || !colptr) return CMPQ_EINVAL;
    if (n_out > 0 && (!out_idx || !out_val || !centroids || !codes || !row_idx || !delta)) return CMPQ_EINVAL;
    if (d_out >= (1 << 20)) return CMPQ_ESHAPE;
    if (d_in > 0 && d_out > ((int64_t)1 << 31) / d_in) return CMPQ_ESHAPE;
    if (n_out > d_in * d_out) return CMPQ_ECOUNT;
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < cmpq_ws_outliers_by_column(d_out, n_out))
        return CMPQ_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *cnt = static_cast<int32_t *>(ws);
    const size_t col_bytes = align_up((size_t)(d_out + 1) * sizeof(int32_t), 256);
    int32_t *cursor = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + col_bytes);
    int32_t *tmp_row = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + 2 * col_bytes);
    float *tmp_delta = reinterpret_cast<float *>(static_cast<char *>(ws) + 2 * col_bytes + align_up((size_t)n_out * 4, 256));
    obc_zero_kernel<<<64, 256, 0, s>>>(cnt, d_out + 1);
    if (n_out > 0) {
        int64_t g = cdiv(n_out, 256);
        if (g > 2048) g = 2048;
        obc_count_kernel<<<(unsigned)g, 256, 0, s>>>(out_idx, n_out, d_out, cnt);
    }
    obc_scan_kernel<<<1, 1024, 0, s>>>(cnt, d_out, colptr, cursor);
    if (n_out > 0 && d_out > 0) {
        int64_t g = cdiv(n_out, 256);
        if (g > 2048) g = 2048;
        obc_scatter_kernel<<<(unsigned)g, 256, 0, s>>>(out_idx, out_val, n_out, d_out, centroids, codes, cursor, tmp_row, tmp_delta);
        obc_order_kernel<<<(unsigned)cdiv(d_out, kWaves), kThreads, 0, s>>>(colptr, d_out, tmp_row, tmp_delta, row_idx, delta);
    }
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

namespace {

// Host-side checks of one layer of a product (the rules of cmpq_lut_matvec).
int check_layer(const cmpq_deployed_layer &L, int64_t m) {
    if (L.d_in < 0 || L.d_out < 0 || L.k_act < 0 || L.n_set < 0 || L.n_set > kMaxWidths) return CMPQ_EINVAL;
    if (L.n_set > 0 && (!L.bit_set || !L.counts_host || !L.packed || !L.chan_idx || !L.lut)) return CMPQ_EINVAL;
    int64_t rows_total = L.k_act;
    for (int j = 0; j < L.n_set; ++j) {
        if (L.bit_set[j] < 1 || L.bit_set[j] > 4 || L.counts_host[j] < 0) return CMPQ_EINVAL;
        if (L.counts_host[j] > 0 && (!L.packed[j] || !L.chan_idx[j] || !L.lut[j])) return CMPQ_EINVAL;
        rows_total += L.counts_host[j];
    }
    if (rows_total > L.d_in) return CMPQ_EINVAL;
    if (m == 0 || L.d_out == 0) return CMPQ_OK;
    if (!L.Y || (L.d_in > 0 && !L.X)) return CMPQ_EINVAL;
    if (L.k_act > 0 && (!L.act_idx || !L.W_act)) return CMPQ_EINVAL;
    if (L.colptr && (!L.row_idx || !L.delta)) return CMPQ_EINVAL;
    if (L.ldx < L.d_in || L.ldy < L.d_out || (L.k_act > 0 && L.ld_act < L.d_out)) return CMPQ_ESHAPE;
    if (L.d_out >= (1 << 20)) return CMPQ_ESHAPE;
    return CMPQ_OK;
}

int launch_group(const cmpq_deployed_layer *layers, int n_layers, int64_t m, void *ws, size_t ws_bytes,
                 void *stream, bool half_sums = false) {
    if (n_layers < 0 || n_layers > kMaxLayers || m < 0 || (n_layers > 0 && !layers)) return CMPQ_EINVAL;
    for (int i = 0; i < n_layers; ++i) {
        const int rc = check_layer(layers[i], m);
        if (rc != CMPQ_OK) return rc;
    }
    if (m > 65535) return CMPQ_ESHAPE;
    if (m == 0) return CMPQ_OK;
    // the longest products first: their workgroups are dispatched first
    int order[kMaxLayers], n_live = 0;
    for (int i = 0; i < n_layers; ++i)
        if (layers[i].d_out > 0) order[n_live++] = i;
    for (int i = 1; i < n_live; ++i)
        for (int j = i; j > 0; --j) {
            const cmpq_deployed_layer &p = layers[order[j - 1]], &q = layers[order[j]];
            if (p.d_in * p.d_out >= q.d_in * q.d_out) break;
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    if (n_live == 0) return CMPQ_OK;
    LmGroup g;
    FinGroup f;
    g.n_layers = f.n_layers = n_live;
    size_t ws_used = 0;
    int64_t y_total = 0, x_total = 0, max_tiles = 0;
    for (int s = 0; s < n_live; ++s) {
        const cmpq_deployed_layer &L = layers[order[s]];
        LmArgs &a = g.l[s];
        // rows per wavefront: the largest of 32, 16, 8 that still gives two workgroups per compute unit
        const int64_t tiles = cdiv(L.d_out, kTileOut);
        int rpw = kMaxRowsPerWave;
        while (rpw > 8 && tiles * total_slabs(L.counts_host, L.n_set, rpw) * m < 512) rpw /= 2;
        const int64_t n_lut = total_slabs(L.counts_host, L.n_set, rpw);
        const int64_t n_act = cdiv(L.k_act, (int64_t)kWaves * kActRowsPerWave);
        const int64_t n_rows = n_lut + n_act;
        a.n_widths = 0;
        a.rows_per_wave = rpw;
        a.n_lut_slabs = (int)n_lut;
        a.n_act_slabs = (int)n_act;
        a.n_rows_total = (int)n_rows;
        a.tiles = (int)tiles;
        a.y0 = (int)y_total;
        a.X = static_cast<const __half *>(L.X);
        a.ldx = L.ldx;
        a.d_out = L.d_out;
        a.partial = reinterpret_cast<float *>(static_cast<char *>(ws) + ws_used);
        a.act_idx = L.act_idx;
        a.W_act = reinterpret_cast<const __half *>(L.W_act);
        a.k_act = L.k_act;
        a.ld_act = L.ld_act;
        a.act_vec_ok = reinterpret_cast<uintptr_t>(L.W_act) % 16 == 0 && L.ld_act % 8 == 0;
        int slab0 = 0;
        for (int j = 0; j < L.n_set; ++j) {
            if (L.counts_host[j] == 0) continue;
            LmWidth &wd = a.w[a.n_widths++];
            wd.packed = L.packed[j];
            wd.chan_idx = L.chan_idx[j];
            wd.lut = L.lut[j];
            wd.rows = L.counts_host[j];
            wd.words_per_row = cdiv(L.d_out * L.bit_set[j], 32);
            wd.slab0 = slab0;
            wd.bits = L.bit_set[j];
            slab0 += (int)cdiv(wd.rows, (int64_t)kWaves * rpw);
        }
        for (int j = a.n_widths; j < kMaxWidths; ++j) a.w[j] = LmWidth{nullptr, nullptr, nullptr, 0, 0, 0, 0};
        FinArgs &fa = f.l[s];
        fa.X = a.X;
        fa.ldx = L.ldx;
        fa.d_out = L.d_out;
        fa.partial = a.partial;
        fa.colptr = L.colptr;
        fa.row_idx = L.row_idx;
        fa.delta = L.delta;
        fa.Y = L.Y;
        fa.ldy = L.ldy;
        fa.n_rows_total = (int)n_rows;
        fa.x0 = (int)x_total;
        ws_used += align_up((size_t)m * (size_t)n_rows * (size_t)L.d_out * sizeof(float), 256);
        y_total += n_rows;
        x_total += cdiv(L.d_out, kFinCols);
        if (tiles > max_tiles) max_tiles = tiles;
    }
    for (int s = n_live; s < kMaxLayers; ++s) {
        g.l[s] = g.l[0];
        f.l[s] = f.l[0];
    }
    if (y_total > 65535 || x_total > 0x7fffffff) return CMPQ_ESHAPE;
    if (ws_used > 0 && (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < ws_used))
        return CMPQ_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (y_total > 0) {
        const dim3 grid((unsigned)max_tiles, (unsigned)y_total, (unsigned)m);
        if (half_sums) lut_matvec_half_kernel<<<grid, kThreads, 0, st>>>(g);
        else lut_matvec_kernel<<<grid, kThreads, 0, st>>>(g);
    }
    const dim3 fgrid((unsigned)x_total, (unsigned)m);
    lut_matvec_finish_kernel<<<fgrid, kThreads, 0, st>>>(f);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

extern "C" int cmpq_lut_matvec_group(const cmpq_deployed_layer *layers, int n_layers, int64_t m, void *ws,
                                     size_t ws_bytes, void *stream) {
    return launch_group(layers, n_layers, m, ws, ws_bytes, stream);
}

extern "C" int cmpq_lut_matvec_group_fp16acc(const cmpq_deployed_layer *layers, int n_layers, int64_t m, void *ws,
                                             size_t ws_bytes, void *stream) {
    return launch_group(layers, n_layers, m, ws, ws_bytes, stream, true);
}

extern "C" int cmpq_lut_matvec(const void *X, int64_t m, int64_t d_in, int64_t ldx, int64_t d_out,
                               const int32_t *bit_set, int n_set, const int64_t *counts_host,
                               const uint32_t *const *packed, const int32_t *const *chan_idx,
                               const uint16_t *const *lut, const int32_t *act_idx,
                               const uint16_t *W_act, int64_t k_act, int64_t ld_act,
                               const int32_t *colptr, const int32_t *row_idx, const float *delta,
                               float *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream) {
    cmpq_deployed_layer L;
    L.X = X;
    L.d_in = d_in;
    L.ldx = ldx;
    L.d_out = d_out;
    L.bit_set = bit_set;
    L.n_set = n_set;
    L.counts_host = counts_host;
    L.packed = packed;
    L.chan_idx = chan_idx;
    L.lut = lut;
    L.act_idx = act_idx;
    L.W_act = W_act;
    L.k_act = k_act;
    L.ld_act = ld_act;
    L.colptr = colptr;
    L.row_idx = row_idx;
    L.delta = delta;
    L.Y = Y;
    L.ldy = ldy;
    if (m < 0) return CMPQ_EINVAL;
    return launch_group(&L, 1, m, ws, ws_bytes, stream);
}
