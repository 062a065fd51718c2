// The averaging iteration of Algorithm 1.
#pragma once
#include "common.hpp"

namespace liec {

// ---------------------------------------------------------------------------------------------
// Averaging iteration of Algorithm 1: gradients and models travel uncompressed, so
//   v_j = e_j + (1/N) sum_i g_ij ; p = v ; e_j <- v_j - v_j ; x_ij <- (1/N) sum_i x_ij - lr * (v_j + (g_ij - g_ij)).
// Both sums run in worker order in fp32.  One block owns 1024 columns of every row.  grid = column tiles.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_sync(const float* __restrict__ grads, float* __restrict__ x,
                                                  float* __restrict__ e_inout, int N, uint32_t d, float inv_n,
                                                  float neg_lr) {
    const uint32_t j = blockIdx.x * kColTile + threadIdx.x * 4;
    if (j >= d) return;
    float4 ag = make_float4(0.f, 0.f, 0.f, 0.f), ax = make_float4(0.f, 0.f, 0.f, 0.f);
    int i = 0;
    for (; i + 4 <= N; i += 4) {
        float4 g[4], xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            g[u] = ld4<VEC, true>(grads + (size_t)(i + u) * d, j, d);
            xv[u] = ld4<VEC, true>(x + (size_t)(i + u) * d, j, d);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ag.x = __fadd_rn(ag.x, g[u].x); ag.y = __fadd_rn(ag.y, g[u].y);
            ag.z = __fadd_rn(ag.z, g[u].z); ag.w = __fadd_rn(ag.w, g[u].w);
            ax.x = __fadd_rn(ax.x, xv[u].x); ax.y = __fadd_rn(ax.y, xv[u].y);
            ax.z = __fadd_rn(ax.z, xv[u].z); ax.w = __fadd_rn(ax.w, xv[u].w);
        }
    }
    for (; i < N; ++i) {
        const float4 g = ld4<VEC, true>(grads + (size_t)i * d, j, d);
        const float4 xv = ld4<VEC, true>(x + (size_t)i * d, j, d);
        ag.x = __fadd_rn(ag.x, g.x); ag.y = __fadd_rn(ag.y, g.y);
        ag.z = __fadd_rn(ag.z, g.z); ag.w = __fadd_rn(ag.w, g.w);
        ax.x = __fadd_rn(ax.x, xv.x); ax.y = __fadd_rn(ax.y, xv.y);
        ax.z = __fadd_rn(ax.z, xv.z); ax.w = __fadd_rn(ax.w, xv.w);
    }
    const float4 e = ld4<VEC>(e_inout, j, d);
    float4 v, en, o;
    v.x = __fmaf_rn(ag.x, inv_n, e.x); v.y = __fmaf_rn(ag.y, inv_n, e.y);
    v.z = __fmaf_rn(ag.z, inv_n, e.z); v.w = __fmaf_rn(ag.w, inv_n, e.w);
    en.x = __fsub_rn(v.x, v.x); en.y = __fsub_rn(v.y, v.y);
    en.z = __fsub_rn(v.z, v.z); en.w = __fsub_rn(v.w, v.w);
    st4<VEC>(e_inout, j, d, en);
    // the cached local error g - p^i is g - g = +0 for every finite gradient
    o.x = __fmaf_rn(neg_lr, __fadd_rn(v.x, 0.f), __fmul_rn(ax.x, inv_n));
    o.y = __fmaf_rn(neg_lr, __fadd_rn(v.y, 0.f), __fmul_rn(ax.y, inv_n));
    o.z = __fmaf_rn(neg_lr, __fadd_rn(v.z, 0.f), __fmul_rn(ax.z, inv_n));
    o.w = __fmaf_rn(neg_lr, __fadd_rn(v.w, 0.f), __fmul_rn(ax.w, inv_n));
    for (i = 0; i < N; ++i) st4<VEC, true>(x + (size_t)i * d, j, d, o);
}

}  // namespace liec
