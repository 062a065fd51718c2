// Scaled sign (Definition 4) and its blockwise form (Definition 5): L1 norms in fp64 and sign bits.
#pragma once
#include "common.hpp"

namespace liec {

// ---------------------------------------------------------------------------------------------
// Scaled sign, worker side (Definition 4): per-row partial sums of |g| in fp64 and the sign bits
// of the row.  Bit layout ("lane-major"): wave tile t of row i owns 64 half-words
// bits[(i*nwt + t)*64 + l]; bit 4u + q of half-word l is (g[1024t + 256u + 4l + q] < 0), i.e. every
// lane keeps the 16 bits of the 16 columns it owns, and a wave reads or writes 128 contiguous bytes.
// grid = (blocks per row, rows); waves stride over the row's wave tiles.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_l1_bits(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                     uint32_t nwt, double* __restrict__ partial,
                                                     uint16_t* __restrict__ bits) {
    __shared__ double lds_w[4];
    const uint32_t row = blockIdx.y;
    const float* __restrict__ g = src + (size_t)row * row_stride;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    double acc = 0.0;
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        float4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = ld4<VEC, true>(g, t * kWaveTile + u * kChunk + lane * 4, d);
        uint32_t m = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc += (double)fabsf(a[u].x);
            acc += (double)fabsf(a[u].y);
            acc += (double)fabsf(a[u].z);
            acc += (double)fabsf(a[u].w);
            m |= (a[u].x < 0.f ? 1u : 0u) << (4 * u);
            m |= (a[u].y < 0.f ? 1u : 0u) << (4 * u + 1);
            m |= (a[u].z < 0.f ? 1u : 0u) << (4 * u + 2);
            m |= (a[u].w < 0.f ? 1u : 0u) << (4 * u + 3);
        }
        // streaming hint on the bits store: 3.5 % faster than a plain store (the store still costs this
        // pass a fifth of its time: without it the kernel reads at 6.8 TB/s)
        __builtin_nontemporal_store((uint16_t)m, &bits[((size_t)row * nwt + t) * 64 + lane]);
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // let the small store land before the next loads (~2 % faster)
#endif
    }
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) partial[(size_t)row * gridDim.x + blockIdx.x] = s;
}

// Finishes the L1 norm of each row from its block partials (fixed order) and sets the scale.
// grid = rows, desc points at the first row's descriptor.
__global__ __launch_bounds__(kBlock) void k_l1_final(const double* __restrict__ partial, uint32_t nparts,
                                                      uint32_t d, RowDesc* __restrict__ desc) {
    __shared__ double lds_w[4];
    const uint32_t row = blockIdx.x;
    const double* __restrict__ p = partial + (size_t)row * nparts;
    // four independent running sums per thread (fixed assignment, fixed combination order) keep
    // four loads in flight
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    uint32_t q = threadIdx.x;
    for (; q + 3 * kBlock < nparts; q += 4 * kBlock) {
        a0 += p[q];
        a1 += p[q + kBlock];
        a2 += p[q + 2 * kBlock];
        a3 += p[q + 3 * kBlock];
    }
    for (; q < nparts; q += kBlock) a0 += p[q];
    const double acc = (a0 + a1) + (a2 + a3);
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) {
        desc[row].l1 = s;
        desc[row].scale = (float)(s / (double)d);
        desc[row].nonfinite = (s - s == 0.0) ? 0u : 1u;   // s - s is NaN for NaN and Inf
    }
}

// ---------------------------------------------------------------------------------------------
// Blockwise scaled sign (Definition 5): Definition 4 on each of B consecutive column blocks
// [off[b], off[b+1]) with its own length.  Sign bits are the same as for Definition 4; only the
// scale depends on the column's block.
// ---------------------------------------------------------------------------------------------
struct BlockTable {
    const uint32_t* tile_blk;   // [ceil(d/1024)] block of the tile's first column; bit 31: the tile spans a boundary
    const uint32_t* off;        // [B + 1] block offsets, off[0] = 0, off[B] = d
    const float* scales;        // [(N + 1) * B] scale of block b of row r at r*B + b (row N: the server's v)
    uint32_t B;
};

__device__ __forceinline__ uint32_t block_of(const BlockTable& bt, uint32_t first, uint32_t j) {
    uint32_t b = first;
    while (b + 1 < bt.B && j >= bt.off[b + 1]) ++b;
    return b;
}

// One unit of the blockwise L1 pass: the part [lo, hi) of one compression block that falls into the
// 4096-column tile `tile`.  Items are ordered by block, then by tile.
struct L1Item {
    uint32_t tile, lo, hi, write_bits;
};

// grid = (items, rows).  Partial sum of |src| over the item's columns (fp64) and, for the item that
// owns the tile's bits, the sign bits of the whole tile.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_l1_items(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                      uint32_t nwt, uint32_t row0, const L1Item* __restrict__ items,
                                                      double* __restrict__ partial, uint16_t* __restrict__ bits) {
    __shared__ double lds_w[4];
    const L1Item it = items[blockIdx.x];
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t t = it.tile * 4 + wave;
    double acc = 0.0;
    if (t < nwt) {
        float4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = ld4<VEC, true>(g, t * kWaveTile + u * kChunk + lane * 4, d);
        uint32_t m = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            if (j >= it.lo && j < it.hi) acc += (double)fabsf(a[u].x);
            if (j + 1 >= it.lo && j + 1 < it.hi) acc += (double)fabsf(a[u].y);
            if (j + 2 >= it.lo && j + 2 < it.hi) acc += (double)fabsf(a[u].z);
            if (j + 3 >= it.lo && j + 3 < it.hi) acc += (double)fabsf(a[u].w);
            m |= (a[u].x < 0.f ? 1u : 0u) << (4 * u);
            m |= (a[u].y < 0.f ? 1u : 0u) << (4 * u + 1);
            m |= (a[u].z < 0.f ? 1u : 0u) << (4 * u + 2);
            m |= (a[u].w < 0.f ? 1u : 0u) << (4 * u + 3);
        }
        if (bits && it.write_bits) bits[((size_t)blockIdx.y * nwt + t) * 64 + lane] = (uint16_t)m;
    }
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) partial[(size_t)(row0 + blockIdx.y) * gridDim.x + blockIdx.x] = s;
}

// grid = (B, rows).  Adds up the item partials of block b in a fixed order and sets its scale.
__global__ __launch_bounds__(kBlock) void k_l1_items_final(const double* __restrict__ partial, uint32_t nitems,
                                                            const uint32_t* __restrict__ item_start,
                                                            const uint32_t* __restrict__ off, uint32_t B, uint32_t row0,
                                                            float* __restrict__ scales, double* __restrict__ l1s) {
    __shared__ double lds_w[4];
    const uint32_t b = blockIdx.x, row = row0 + blockIdx.y;
    const double* __restrict__ p = partial + (size_t)row * nitems;
    const uint32_t q0 = item_start[b], q1 = item_start[b + 1];
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    uint32_t q = q0 + threadIdx.x;
    for (; q + 3 * kBlock < q1; q += 4 * kBlock) {
        a0 += p[q];
        a1 += p[q + kBlock];
        a2 += p[q + 2 * kBlock];
        a3 += p[q + 3 * kBlock];
    }
    for (; q < q1; q += kBlock) a0 += p[q];
    const double s = block_sum_f64((a0 + a1) + (a2 + a3), lds_w);
    if (threadIdx.x == 0) {
        l1s[(size_t)row * B + b] = s;
        scales[(size_t)row * B + b] = (float)(s / (double)(off[b + 1] - off[b]));
    }
}

}  // namespace liec
