// The drafting step of the outer loop of speculative decoding (Alg. 3, "sample X_1 .. X_gamma from M_s")
// for a model whose conditional distributions are handed over as rows of logits: one token per row
// from softmax(logits / T), Y = min{x : C_x > u * C_total} with C the running sum in vocabulary order
// (the same convention as the draw of the correction token).  Not a hot path: a drafter produces its
// tokens as it runs; this exists so that the outer loop on toy models stays on the device.
#pragma once

#include "common.hpp"

namespace sv {

// One workgroup per row; thread t owns the contiguous range [t * len, (t + 1) * len) of the row, so that
// per-thread sums, scanned over the threads, are the running sum in vocabulary order.
template <typename T>
__global__ void sample_rows_kernel(const T *logits, int V, float k, const float *uniforms, int32_t *tokens)
{
    __shared__ double part[kThreads];
    __shared__ float red[kThreads];
    __shared__ int winner;
    __shared__ double total_all;
    const int nt = blockDim.x, t = threadIdx.x;
    const T *row = logits + (size_t)blockIdx.x * V;
    const int len = (V + nt - 1) / nt;
    const int lo = t * len < V ? t * len : V, hi = lo + len < V ? lo + len : V;

    float m = -INFINITY;
    for (int x = lo; x < hi; ++x) m = fmaxf(m, (float)logit_as_double(row + x));
    red[t] = m;
    __syncthreads();
    for (int s = nt / 2; s > 0; s >>= 1) {
        if (t < s) red[t] = fmaxf(red[t], red[t + s]);
        __syncthreads();
    }
    const float shift = red[0] * k;

    double mine = 0.0;
    for (int x = lo; x < hi; ++x) mine += (double)fast_exp2(__builtin_fmaf((float)logit_as_double(row + x), k, -shift));
    part[t] = mine;
    if (t == 0) winner = -1;
    __syncthreads();
    // running sum over the threads, in order (thread 0 walks the at most 256 partial sums)
    if (t == 0) {
        double c = 0.0;
        for (int i = 0; i < nt; ++i) { const double s = part[i]; part[i] = c; c += s; }
        total_all = c;
    }
    __syncthreads();
    const double total = total_all;
    const double target = (double)uniforms[blockIdx.x] * total;
    const double below = part[t];
    // the thread whose range holds the target walks it; the last such claim in thread order wins when
    // rounding makes neighbours both claim (it cannot: ranges are disjoint half-open intervals)
    if (mine > 0.0 && below <= target && target < below + mine) {
        double c = below;
        int y = -1, last_positive = -1;
        for (int x = lo; x < hi; ++x) {
            const float e = fast_exp2(__builtin_fmaf((float)logit_as_double(row + x), k, -shift));
            c += (double)e;
            if (e > 0.f) last_positive = x;
            if (c > target) { y = x; break; }
        }
        winner = y >= 0 ? y : last_positive;
    }
    __syncthreads();
    if (winner < 0 && t == 0) {
        // rounding pushed the target to the total: the last token of positive weight
        int y = 0;
        for (int x = V - 1; x >= 0; --x)
            if (fast_exp2(__builtin_fmaf((float)logit_as_double(row + x), k, -shift)) > 0.f) { y = x; break; }
        winner = y;
    }
    __syncthreads();
    if (t == 0) tokens[blockIdx.x] = winner;
}

}  // namespace sv
