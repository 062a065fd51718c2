// Error-norm telemetry and the copy probe.
#pragma once
#include "common.hpp"

namespace liec {

// ---------------------------------------------------------------------------------------------
// Telemetry: sum of squares of a vector in fp64 (the paper tracks the l2 norm of the error variable,
// Lemma 1 and the figure on the effect of immediate compensation).  Block partials in a fixed order;
// k_sumsq_final adds them on one block.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_sumsq(const float* __restrict__ v, uint64_t n, double* __restrict__ partial) {
    __shared__ double lds_w[4];
    double acc = 0.0;
    for (uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x; j < n; j += (uint64_t)gridDim.x * kBlock) {
        const double t = (double)v[j];
        acc += t * t;
    }
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// take_root: write the norm itself (the correctly rounded square root of the sum) instead of the sum.
__global__ __launch_bounds__(kBlock) void k_sumsq_final(const double* __restrict__ partial, uint32_t nparts,
                                                         double* __restrict__ out, bool take_root) {
    __shared__ double lds_w[4];
    double acc = 0.0;
    for (uint32_t q = threadIdx.x; q < nparts; q += kBlock) acc += partial[q];
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) *out = take_root ? __dsqrt_rn(s) : s;
}

// Plain device copy (128 bits per thread, streaming hints), used to measure the achievable
// read+write bandwidth next to the step's kernels and to calibrate byte counters.
__global__ __launch_bounds__(kBlock) void k_copy16(const v4f* __restrict__ src, v4f* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

}  // namespace liec
