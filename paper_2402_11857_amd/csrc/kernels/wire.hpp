// Wire forms of the compressed messages.
#pragma once
#include "common.hpp"
#include "sign.hpp"

namespace liec {

// ---------------------------------------------------------------------------------------------
// Wire form of a (blockwise) scaled-sign message: one bit per element, bit j % 8 of byte j / 8 set
// when the element is negative.  k_pack_sign turns one row of the lane-major bitmap into that
// form (one thread per output byte); k_unpack_sign expands wire bits and scale(s) into the dense
// message p_j = -s or +s (one 128-bit store per 4 columns).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_pack_sign(const uint16_t* __restrict__ row_bits, uint32_t nbytes,
                                                       uint8_t* __restrict__ out) {
    const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbytes) return;
    const uint32_t col = b * 8, t = col / kWaveTile, o = col % kWaveTile, u = o / kChunk, lane = (o % kChunk) / 4;
    const uint32_t m0 = row_bits[(size_t)t * 64 + lane], m1 = row_bits[(size_t)t * 64 + lane + 1];
    out[b] = (uint8_t)(((m0 >> (4 * u)) & 0xfu) | (((m1 >> (4 * u)) & 0xfu) << 4));
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_unpack_sign(const uint8_t* __restrict__ bytes, uint32_t d,
                                                         const float* __restrict__ scales, float scale0,
                                                         BlockTable bt, float* __restrict__ p) {
    const uint32_t nq = (d + 3) / 4;                            // groups of 4 columns = half a wire byte
    for (uint32_t q = blockIdx.x * kBlock + threadIdx.x; q < nq; q += gridDim.x * kBlock) {
        const uint32_t j0 = q * 4;
        const uint32_t m = (uint32_t)bytes[q >> 1] >> (4 * (q & 1u));
        float v[4];
        if (bt.B) {
            const uint32_t tb = bt.tile_blk[j0 / kColTile], first = tb & 0x7fffffffu;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t j = j0 + c < d ? j0 + c : d - 1;
                const float s = scales[(tb >> 31) ? block_of(bt, first, j) : first];
                v[c] = ((m >> c) & 1u) ? -s : s;
            }
        } else {
            const float s = scale0;                             // Definition 4: one scale, passed by value
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = ((m >> c) & 1u) ? -s : s;
        }
        st4<VEC>(p, j0, d, make_float4(v[0], v[1], v[2], v[3]));
    }
}

// ---------------------------------------------------------------------------------------------
// Wire form of a top-k message: the kept entries of one row as (index, value) pairs in increasing
// index order.  Three kernels: kept entries per wave tile, exclusive scan of those counts, ordered
// emission.  Inside a wave tile the order is chunk, then lane, then component.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__device__ __forceinline__ void kept_ballots(const float* __restrict__ g, uint32_t t, uint32_t lane, uint32_t d,
                                             uint32_t tau, uint32_t cut, const uint16_t* __restrict__ kept_row,
                                             float4 (&a)[4], uint64_t (&kb)[4][4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] = ld4<VEC>(g, t * kWaveTile + u * kChunk + lane * 4, d);
    if (kept_row) {                                 // random-k: the kept set is a bitmap (wave-uniform branch)
        const uint32_t m = kept_row[(size_t)t * 64 + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) kb[u][q] = __ballot((m >> (4 * u + q)) & 1u);
        return;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
        const float av[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t key = key_of(av[q]);
            kb[u][q] = __ballot(j + q < d && (key > tau || (key == tau && j + q <= cut)));
        }
    }
}

// grid = blocks over the wave tiles of the row.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_topk_count(const float* __restrict__ g, uint32_t d, uint32_t nwt,
                                                        const RowDesc* __restrict__ rd,
                                                        const uint16_t* __restrict__ kept_row,
                                                        uint32_t* __restrict__ tile_cnt) {
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t tau = rd->tau, cut = rd->cutoff;
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        float4 a[4];
        uint64_t kb[4][4];
        kept_ballots<VEC>(g, t, lane, d, tau, cut, kept_row, a, kb);
        uint32_t n = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) n += __popcll(kb[u][q]);
        if (lane == 0) tile_cnt[t] = n;
    }
}

// One block of 1024 threads: exclusive scan of n counts in place; *total receives the sum.  The block walks
// the array 4096 counts at a time (4 consecutive ones per thread, so the accesses coalesce).
__global__ __launch_bounds__(1024) void k_scan_u32(uint32_t* __restrict__ v, uint32_t n, uint32_t* __restrict__ total) {
    __shared__ uint32_t wsum[16];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < n; base += 4096) {          // uniform trip count
        const uint32_t i = base + tid * 4;
        uint32_t a[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = i + q < n ? v[i + q] : 0u;
        const uint32_t s = a[0] + a[1] + a[2] + a[3];
        uint32_t incl = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += up;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = carry, all = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < (int)wave) before += wsum[w];
            all += wsum[w];
        }
        uint32_t run = before + incl - s;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i + q < n) v[i + q] = run;
            run += a[q];
        }
        carry += all;
        __syncthreads();
    }
    if (tid == 0) *total = carry;
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_topk_emit(const float* __restrict__ g, uint32_t d, uint32_t nwt,
                                                       const RowDesc* __restrict__ rd,
                                                       const uint16_t* __restrict__ kept_row,
                                                       const uint32_t* __restrict__ tile_off, uint32_t k,
                                                       uint32_t* __restrict__ idx_out, float* __restrict__ val_out) {
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t tau = rd->tau, cut = rd->cutoff;
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        float4 a[4];
        uint64_t kb[4][4];
        kept_ballots<VEC>(g, t, lane, d, tau, cut, kept_row, a, kb);
        uint32_t base = tile_off[t];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            const float av[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
            // entries of lower lanes come first, then this lane's lower components
            uint32_t pos = base + lanes_below(kb[u][0]) + lanes_below(kb[u][1]) + lanes_below(kb[u][2]) +
                           lanes_below(kb[u][3]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if ((kb[u][q] >> lane) & 1) {
                    if (pos < k) {
                        idx_out[pos] = j + q;
                        val_out[pos] = av[q];
                    }
                    ++pos;
                }
            }
            base += __popcll(kb[u][0]) + __popcll(kb[u][1]) + __popcll(kb[u][2]) + __popcll(kb[u][3]);
        }
    }
}

// Dense vector from (index, value) pairs: the caller zero-fills p first.
__global__ __launch_bounds__(kBlock) void k_scatter_pairs(const uint32_t* __restrict__ idx, const float* __restrict__ val,
                                                           uint32_t k, uint32_t d, float* __restrict__ p) {
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r < k && idx[r] < d) p[idx[r]] = val[r];
}

__global__ __launch_bounds__(kBlock) void k_fill_f32(float* __restrict__ p, uint32_t n, float v) {
    for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < n; j += gridDim.x * kBlock) p[j] = v;
}

}  // namespace liec
