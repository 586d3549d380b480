// cmpq_act_stats: per-channel sum of squares of the calibration activations
// (Sec. 3.2.1 of arXiv 2410.13056: the L2 norm of each channel of X, kept squared).
//
// HBM bound: every element of X is read once.  Each lane streams 16-byte
// pieces of a row (8 halves or 4 floats), a wave covers 1 KiB of one row, the
// four waves of a workgroup take consecutive rows, and the grid tiles X into
// (column block) x (row split) so that a few thousand workgroups are in flight.
// Squares are accumulated in fp64 (x*x is exact there for both input types), so
// the result does not depend on how rows are split beyond the last fp64 bit.
// Row splits leave fp64 partials in the workspace; a second kernel adds them in
// split order, which makes the whole reduction reproducible.
#include <mutex>

#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / CMPQ_WAVE;

template <typename T>
struct Vec;
template <>
struct Vec<__half> {
    static constexpr int N = 8;
    __device__ static void load(const __half *p, float (&f)[8]) {
        typedef uint32_t U4 __attribute__((ext_vector_type(4)));
        const U4 nt = __builtin_nontemporal_load(reinterpret_cast<const U4 *>(p));  // X is read once
        const uint4 raw = make_uint4(nt.x, nt.y, nt.z, nt.w);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float2 t = __half22float2(h[j]);
            f[2 * j] = t.x;
            f[2 * j + 1] = t.y;
        }
    }
};
template <>
struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float *p, float (&f)[4]) {
        const float4 raw = *reinterpret_cast<const float4 *>(p);
        f[0] = raw.x;
        f[1] = raw.y;
        f[2] = raw.z;
        f[3] = raw.w;
    }
};

// One element into the running value of its column: x^2 (l2, App. Tab. 13's default), |x|
// (l1) or the largest |x| (l-infinity).
template <int NORM>
__device__ __forceinline__ double fold(double s, float x) {
    const double d = (double)x;
    if (NORM == CMPQ_NORM_L2) return fma(d, d, s);
    if (NORM == CMPQ_NORM_L1) return s + fabs(d);
    // fmax drops a NaN operand; a channel that holds one must come out non-finite like under
    // the other norms, so that the status flag is raised for it
    return (d != d || s != s) ? s + d : fmax(s, fabs(d));
}
template <int NORM>
__device__ __forceinline__ double combine(double a, double b) {
    if (NORM != CMPQ_NORM_LINF) return a + b;
    return (a != a || b != b) ? a + b : fmax(a, b);  // a NaN partial stays
}

// partial[split * d_in + col] = the statistic over the rows of this split of column col
template <typename T, int NORM>
__global__ __launch_bounds__(kThreads) void act_stats_vec_kernel(const T *__restrict__ X, int64_t n,
                                                                  int64_t d_in, int64_t ldx,
                                                                  int64_t rows_per_split,
                                                                  double *__restrict__ partial) {
    constexpr int V = Vec<T>::N;
    constexpr int kCols = CMPQ_WAVE * V;  // columns per workgroup
    __shared__ double red[kWaves][kCols];
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = threadIdx.x / CMPQ_WAVE;
    const int64_t col0 = (int64_t)blockIdx.x * kCols + (int64_t)lane * V;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_split;
    const int64_t r_end = min(n, r_begin + rows_per_split);
    double s[V];
#pragma unroll
    for (int v = 0; v < V; ++v) s[v] = 0.0;
    if (col0 < d_in) {
        const T *p = X + col0;
        int64_t r = r_begin + wave;
        // eight rows in flight per wave
        for (; r + 7 * kWaves < r_end; r += 8 * kWaves) {
            float f[8][V];
#pragma unroll
            for (int u = 0; u < 8; ++u) Vec<T>::load(p + (r + u * kWaves) * ldx, f[u]);
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int v = 0; v < V; ++v) s[v] = fold<NORM>(s[v], f[u][v]);
        }
        for (; r < r_end; r += kWaves) {
            float f[V];
            Vec<T>::load(p + r * ldx, f);
#pragma unroll
            for (int v = 0; v < V; ++v) s[v] = fold<NORM>(s[v], f[v]);
        }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) red[wave][lane * V + v] = s[v];
    __syncthreads();
    for (int c = threadIdx.x; c < kCols; c += kThreads) {
        const int64_t col = (int64_t)blockIdx.x * kCols + c;
        if (col < d_in) {
            double t = red[0][c];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) t = combine<NORM>(t, red[w][c]);
            partial[(int64_t)blockIdx.y * d_in + col] = t;
        }
    }
}

// Any alignment: one thread per column, threads of a wave read neighbouring columns.
template <typename T, int NORM>
__global__ __launch_bounds__(kThreads) void act_stats_any_kernel(const T *__restrict__ X, int64_t n,
                                                                  int64_t d_in, int64_t ldx,
                                                                  int64_t rows_per_split,
                                                                  double *__restrict__ partial) {
    const int64_t col = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (col >= d_in) return;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_split;
    const int64_t r_end = min(n, r_begin + rows_per_split);
    double s = 0.0;
    for (int64_t r = r_begin; r < r_end; ++r) s = fold<NORM>(s, load_as_f32<T>(X, r * ldx + col));
    partial[(int64_t)blockIdx.y * d_in + col] = s;
}

// 64 columns per workgroup; the four wavefronts each add a quarter of the row splits
// (in split order), then the quarters are added in order: a fixed summation tree.
template <int NORM>
__global__ __launch_bounds__(kThreads) void act_stats_finish_kernel(
    const double *__restrict__ partial, int splits, int64_t d_in, double *__restrict__ acc,
    float *__restrict__ sumsq, int accumulate, int32_t *__restrict__ status) {
    __shared__ double red[kWaves][CMPQ_WAVE];
    const int lane = threadIdx.x & (CMPQ_WAVE - 1), wave = threadIdx.x / CMPQ_WAVE;
    const int64_t col = (int64_t)blockIdx.x * CMPQ_WAVE + lane;
    const int per = (splits + kWaves - 1) / kWaves;
    const int s0 = wave * per, s1 = min(splits, s0 + per);
    double t = 0.0;
    if (col < d_in)
        for (int sidx = s0; sidx < s1; ++sidx) t = combine<NORM>(t, partial[(int64_t)sidx * d_in + col]);
    red[wave][lane] = t;
    __syncthreads();
    if (wave == 0 && col < d_in) {
        double r = accumulate ? acc[col] : 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) r = combine<NORM>(r, red[w][lane]);
        acc[col] = r;
        if (sumsq) sumsq[col] = (float)r;
        if (status && !isfinite(r)) atomicOr(status, CMPQ_STATUS_NONFINITE);
    }
}

int64_t pick_splits(int64_t n, int64_t col_blocks) {
    if (n <= 0) return 0;
    int64_t want = cdiv(2048, col_blocks);       // ~8 workgroups per compute unit
    int64_t cap = cdiv(n, 16 * kWaves);           // at least 16 rows per wave
    int64_t s = want < cap ? want : cap;
    return s < 1 ? 1 : s;
}

size_t ws_act_stats_impl(int64_t d_in, int64_t n) {
    // the widest column block gives the fewest column blocks, hence the most row splits
    int64_t col_blocks = cdiv(d_in, 512) > 0 ? cdiv(d_in, 512) : 1;
    int64_t s = pick_splits(n, col_blocks);
    return align_up((size_t)(s > 0 ? s : 1) * (size_t)(d_in > 0 ? d_in : 1) * sizeof(double), 256);
}

template <int NORM>
int launch_act_stats(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx, double *acc,
                     float *stat, int accumulate, void *ws, size_t ws_bytes, int32_t *status,
                     hipStream_t st) {
    const int vec = dtype == CMPQ_F16 ? 8 : 4;
    const bool aligned = n > 0 && d_in % vec == 0 && ldx % vec == 0 &&
                         reinterpret_cast<uintptr_t>(X) % 16 == 0;
    const int64_t col_blocks = aligned ? cdiv(d_in, CMPQ_WAVE * vec) : cdiv(d_in, kThreads);
    const int64_t splits = pick_splits(n, col_blocks);
    double *partial = static_cast<double *>(ws);
    if (splits > 0) {
        if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 ||
            ws_bytes < (size_t)splits * d_in * sizeof(double))
            return CMPQ_EWORKSPACE;
        if (splits > 65535) return CMPQ_ESHAPE;
        const int64_t rps = cdiv(n, splits);
        dim3 grid((unsigned)col_blocks, (unsigned)splits);
        if (aligned) {
            cmpq_timing_before(CMPQ_KERNEL_ACT_STATS, st);
            if (dtype == CMPQ_F16)
                act_stats_vec_kernel<__half, NORM><<<grid, kThreads, 0, st>>>(
                    static_cast<const __half *>(X), n, d_in, ldx, rps, partial);
            else
                act_stats_vec_kernel<float, NORM><<<grid, kThreads, 0, st>>>(
                    static_cast<const float *>(X), n, d_in, ldx, rps, partial);
            cmpq_timing_after(CMPQ_KERNEL_ACT_STATS, st);
        } else {
            if (dtype == CMPQ_F16)
                act_stats_any_kernel<__half, NORM><<<grid, kThreads, 0, st>>>(
                    static_cast<const __half *>(X), n, d_in, ldx, rps, partial);
            else
                act_stats_any_kernel<float, NORM><<<grid, kThreads, 0, st>>>(
                    static_cast<const float *>(X), n, d_in, ldx, rps, partial);
        }
        CMPQ_LAUNCH_CHECK();
    }
    act_stats_finish_kernel<NORM><<<(unsigned)cdiv(d_in, CMPQ_WAVE), kThreads, 0, st>>>(
        partial, (int)splits, d_in, acc, stat, accumulate, status);
    CMPQ_LAUNCH_CHECK();
    return CMPQ_OK;
}

}  // namespace

size_t cmpq_ws_act_stats(int64_t d_in, int64_t n) { return ws_act_stats_impl(d_in, n); }

extern "C" int cmpq_act_stats_norm(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx,
                                   int norm, double *acc, float *stat, int accumulate, void *ws,
                                   size_t ws_bytes, int32_t *status, void *stream) {
    if (!acc || n < 0 || d_in < 0 || (dtype != CMPQ_F16 && dtype != CMPQ_F32)) return CMPQ_EINVAL;
    if (norm != CMPQ_NORM_L2 && norm != CMPQ_NORM_L1 && norm != CMPQ_NORM_LINF) return CMPQ_EINVAL;
    if (n > 0 && !X) return CMPQ_EINVAL;
    if (ldx < d_in) return CMPQ_ESHAPE;
    if (d_in == 0) return CMPQ_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (norm) {
        case CMPQ_NORM_L1: return launch_act_stats<CMPQ_NORM_L1>(X, dtype, n, d_in, ldx, acc, stat, accumulate, ws, ws_bytes, status, st);
        case CMPQ_NORM_LINF: return launch_act_stats<CMPQ_NORM_LINF>(X, dtype, n, d_in, ldx, acc, stat, accumulate, ws, ws_bytes, status, st);
        default: return launch_act_stats<CMPQ_NORM_L2>(X, dtype, n, d_in, ldx, acc, stat, accumulate, ws, ws_bytes, status, st);
    }
}

// ---- the same call for callers that cannot allocate ---------------------------------------
//
// The row-split partials live in a file-scope device array instead of a caller workspace.
// Every GPU holds its own copy of the array at its own address; the address is looked up once
// per device and only that pointer is handed to kernels.

constexpr int64_t kStaticMaxDin = 262144;
// row splits x d_in never exceeds 2048 x 512 + d_in (see pick_splits: about 2048 workgroups
// of 512 columns each, rounded up by at most one split)
constexpr size_t kStaticDoubles = (size_t)2048 * 512 + (size_t)kStaticMaxDin;
static __device__ __align__(256) double scratch[kStaticDoubles];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices];  // per device: where that GPU keeps `scratch`

// Device address of `scratch` on the current device; null if the runtime cannot name it.
double *scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        double *p = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int cmpq_act_stats_static(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx,
                                     double *acc, float *sumsq, int accumulate, int32_t *status,
                                     void *stream) {
    if (!acc || n < 0 || d_in < 0 || (dtype != CMPQ_F16 && dtype != CMPQ_F32)) return CMPQ_EINVAL;
    if (n > 0 && !X) return CMPQ_EINVAL;
    if (ldx < d_in) return CMPQ_ESHAPE;
    if (d_in > kStaticMaxDin) return CMPQ_ESHAPE;  // beyond what the fixed scratch array is sized for
    if (d_in == 0) return CMPQ_OK;
    if (ws_act_stats_impl(d_in, n) > sizeof(double) * kStaticDoubles) return CMPQ_ESHAPE;
    double *ptr = scratch_on_current_device();
    if (!ptr) return CMPQ_EHIP;
    return launch_act_stats<CMPQ_NORM_L2>(X, dtype, n, d_in, ldx, acc, sumsq, accumulate, ptr,
                                          sizeof(double) * kStaticDoubles, status,
                                          static_cast<hipStream_t>(stream));
}

extern "C" int cmpq_act_stats(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx,
                              double *acc, float *sumsq, int accumulate, void *ws, size_t ws_bytes,
                              int32_t *status, void *stream) {
    return cmpq_act_stats_norm(X, dtype, n, d_in, ldx, CMPQ_NORM_L2, acc, sumsq, accumulate, ws, ws_bytes,
                               status, stream);
}
