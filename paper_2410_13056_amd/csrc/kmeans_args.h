// Argument block shared by the two k-means kernels of libcmpq.
#pragma once
#include "common.h"

struct KmArgs {
    const void *W;
    int64_t d_in, d_out, ldw;
    const uint8_t *bits;
    const int32_t *out_idx;
    int64_t n_out;
    const float *ew;
    int iters;
    int start_given;  // the rounds start from the levels found in `centroids` (CMPQ_INIT_GIVEN)
    float *centroids;
    uint8_t *codes;
    int32_t *status;
    // One byte per channel in the workspace.  The fixed-point kernel raises it for a
    // channel it cannot hold (a magnitude of 128 or more, or a non-finite value); the
    // general kernel, launched after it, then handles exactly those channels.
    uint8_t *deferred;
    // seg[i]..seg[i+1]: the slice of out_idx inside channel i (null when n_out is 0).
    const int32_t *seg;
    // Stored format and error written by the coding pass of the bucket kernel (Sec. 5.1;
    // App. B.3) instead of by a pass of their own: where the rows go, the row of each channel
    // inside its width group, and the per-channel squared error.  Unused unless `fused`.
    int fused;
    PackPtrs pack;
    const int32_t *row_of;
    double *err_ch;
    // The bucket kernel's per-channel arrangement (bucket table and place array built from all
    // weights of a channel): written for a later run (arr_keep) or taken from an earlier one
    // instead of building it again (arr_reuse).  arr_stride bytes per channel.
    void *arr_keep;
    const void *arr_reuse;
    int64_t arr_stride;
};

// Histogram k-means (kmeans_hist.hip) and fixed-point brute-force k-means
// (kmeans_fast.hip), both for fp16 weights with unit importance.
int launch_kmeans_hist(const KmArgs &a, hipStream_t s);  // honours a.fused, a.arr_keep, a.arr_reuse
// Bytes per channel of the arrangement for channels of d_out weights (0: the kernel does not take them).
size_t kmeans_hist_arrangement_stride(int64_t d_out);
int launch_kmeans_fast(const KmArgs &a, hipStream_t s);
bool kmeans_fast_eligible(const KmArgs &a, int dtype);
