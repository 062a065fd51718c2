// The averaging iteration of Algorithm 1.
#pragma once
#include "common.hpp"

namespace liec {

// ---------------------------------------------------------------------------------------------
// Averaging iteration of Algorithm 1: gradients and models travel uncompressed, so
//   v_j = e_j + (1/N) sum_i g_ij ; p = v ; e_j <- v_j - v_j ; x_ij <- (1/N) sum_i x_ij - lr * (v_j + (g_ij - g_ij)).
// Both sums run in worker order in fp32.  Two kernels: k_sync_reduce reads (one block owns 1024 columns of
// every row: it must, the sums are sequential in the worker index) and writes the new model, which is the same
// for every worker, to row 0 of x only; k_sync_spread copies row 0 to the other N - 1 rows and writes e, one
// block per (1024 columns, row) in the update kernel's panel order (e takes the place of row 0).  A kernel that
// only reads runs at 6.8 TB/s in this shape and one that only writes at 6.3 TB/s, where the fused form (every
// thread reading 2 N tiles, then writing N) reached 4.8 TB/s; every byte the reading kernel writes costs it like
// five read ones, so it writes as little as it can (4 d bytes).
// e <- v - v is +0 for every finite v; k_sync_spread forms it as o - o from the new model o = fma(-lr, v, mean x),
// which is +0 for exactly the same inputs (and NaN where v is not finite, as v - v is).
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_sync_reduce(const float* __restrict__ grads, float* __restrict__ x,
                                                         const float* __restrict__ e_in, int N,
                                                         uint32_t d, float inv_n, float neg_lr) {
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
    const float4 e = ld4<VEC>(e_in, j, d);
    float4 v, o;
    v.x = __fmaf_rn(ag.x, inv_n, e.x); v.y = __fmaf_rn(ag.y, inv_n, e.y);
    v.z = __fmaf_rn(ag.z, inv_n, e.z); v.w = __fmaf_rn(ag.w, inv_n, e.w);
    // the cached local error g - p^i is g - g = +0 for every finite gradient
    o.x = __fmaf_rn(neg_lr, __fadd_rn(v.x, 0.f), __fmul_rn(ax.x, inv_n));
    o.y = __fmaf_rn(neg_lr, __fadd_rn(v.y, 0.f), __fmul_rn(ax.y, inv_n));
    o.z = __fmaf_rn(neg_lr, __fadd_rn(v.z, 0.f), __fmul_rn(ax.z, inv_n));
    o.w = __fmaf_rn(neg_lr, __fadd_rn(v.w, 0.f), __fmul_rn(ax.w, inv_n));
    st4<VEC, true>(x, j, d, o);                        // row 0 (this thread has read all it needs of its columns); a streaming
                                                       // store measured 3 % faster for the kernel than a plain one
}

// grid = number of panels * panel * N, as the update kernel's.  Row index 0 stands for e, 1 .. N - 1 for those rows of x.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_sync_spread(float* __restrict__ x, float* __restrict__ e_out, int N,
                                                         uint32_t panel, uint32_t ncol_tiles, uint32_t d) {
    const uint32_t per_panel = panel * (uint32_t)N;
    const uint32_t pn = blockIdx.x / per_panel, r = blockIdx.x % per_panel;
    const uint32_t i = r / panel, tile = pn * panel + r % panel;
    if (tile >= ncol_tiles) return;
    const uint32_t j = tile * kColTile + threadIdx.x * 4;
    if (j >= d) return;
    const float4 o = ld4<VEC>(x, j, d);                // row 0: the new model of every worker
    if (i == 0) {
        float4 en;
        en.x = __fsub_rn(o.x, o.x); en.y = __fsub_rn(o.y, o.y);
        en.z = __fsub_rn(o.z, o.z); en.w = __fsub_rn(o.w, o.w);
        st4<VEC>(e_out, j, d, en);
    } else {
        st4<VEC, true>(x + (size_t)i * d, j, d, o);
    }
}

}  // namespace liec
