// Server compensation, server compression, error update and the workers' update (Algorithm 1).
#pragma once
#include "common.hpp"
#include "sign.hpp"

namespace liec {

// acc[u].{x,y,z,w} += (bit 4u + q of m) ? -s : s  -- one scaled-sign message, 16 columns of a lane.
__device__ __forceinline__ float signed_scale(uint32_t m, int b, float s) {
    // bit b of m moved to the sign position and merged over +s (s >= 0)
    return __uint_as_float(((m << (31 - b)) & 0x80000000u) | __float_as_uint(s));
}
__device__ __forceinline__ void add_signed(float4 (&acc)[4], uint32_t m, float s) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        acc[u].x = __fadd_rn(acc[u].x, signed_scale(m, 4 * u + 0, s));
        acc[u].y = __fadd_rn(acc[u].y, signed_scale(m, 4 * u + 1, s));
        acc[u].z = __fadd_rn(acc[u].z, signed_scale(m, 4 * u + 2, s));
        acc[u].w = __fadd_rn(acc[u].w, signed_scale(m, 4 * u + 3, s));
    }
}

// ---------------------------------------------------------------------------------------------
// Worker message element p^i_j rebuilt from g_ij and the row's descriptor.
// ---------------------------------------------------------------------------------------------
template <int WC>
__device__ __forceinline__ float message_of(float g, uint32_t j, float scale, uint32_t tau, uint32_t cutoff,
                                            uint32_t keep) {
    if (WC == kSign || WC == kBlockSign) return g < 0.f ? -scale : scale;
    if (WC == kRandk) return keep ? g : 0.f;
    if (WC == kTopk) {
        const uint32_t key = key_of(g);
        return (key > tau || (key == tau && j <= cutoff)) ? g : 0.f;
    }
    return g;
}

// ---------------------------------------------------------------------------------------------
// Server compensation (Algorithm 1): v_j = e_j + (1/N) sum_i p^i_j, messages added in worker
// order; v goes to its own buffer.  With SRV_L1 the kernel also emits per-block partial sums of
// |v| (fp64) for the server's scaled-sign operator.  grid = blocks; waves stride over wave tiles.
//   WC == kSign / kBlockSign  read the packed sign bits instead of the gradients (blockwise: the scale
//                   comes from the column's block);
//   WC == kTopk     reads each row's group bitmap (one bit per 4 columns, or `coarse`: per 64-byte line) and
//                   fetches only the flagged groups, testing their gradients against (tau, cut-off); per-lane
//                   sums live in LDS;
//   WC == kRandk    reads each row's kept bitmap and fetches only the groups of 4 gradients that hold a
//                   kept column;
//   WC == kIdentity reads the gradients.
// With `vbits` the kernel also leaves the sign bits of v (lane-major half-words like the workers' sign
// bits) for the update kernel of a scaled-sign server.
// ---------------------------------------------------------------------------------------------
template <int WC, bool SRV_L1, bool VEC, bool BATCH = false>
__global__ __launch_bounds__(kBlock) void k_aggregate(const float* __restrict__ grads, const uint16_t* __restrict__ bits,
                                                       const uint64_t* __restrict__ gbits,
                                                       int N, uint32_t d, uint32_t nwt, float inv_n,
                                                       const RowDesc* __restrict__ desc, const float* __restrict__ e_in,
                                                       float* __restrict__ v_out, double* __restrict__ srv_partial,
                                                       BlockTable bt, bool coarse, uint16_t* __restrict__ vbits) {
    __shared__ double lds_w[4];
    __shared__ float accs[((WC == kTopk && !BATCH) || WC == kRandk) ? 16 * kBlock : 1];
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    double l1 = 0.0;
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        const uint32_t j0 = t * kWaveTile + lane * 4;
        float4 acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (WC == kSign) {
            const uint16_t* __restrict__ bw = bits + (size_t)t * 64 + lane;
            const size_t brow = (size_t)nwt * 64;
            int i = 0;
            for (; i + 8 <= N; i += 8) {                       // 8 rows of bits in flight
                uint32_t m[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) m[r] = bw[(size_t)(i + r) * brow];
#pragma unroll
                for (int r = 0; r < 8; ++r) add_signed(acc, m[r], desc[i + r].scale);
            }
            for (; i < N; ++i) add_signed(acc, bw[(size_t)i * brow], desc[i].scale);
        } else if (WC == kBlockSign) {
            const uint16_t* __restrict__ bw = bits + (size_t)t * 64 + lane;
            const size_t brow = (size_t)nwt * 64;
            const uint32_t tb = bt.tile_blk[t], first = tb & 0x7fffffffu;
            if (!(tb >> 31)) {                                  // the whole wave tile lies in one block
                int i = 0;
                for (; i + 8 <= N; i += 8) {
                    uint32_t m[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) m[r] = bw[(size_t)(i + r) * brow];
#pragma unroll
                    for (int r = 0; r < 8; ++r) add_signed(acc, m[r], bt.scales[(size_t)(i + r) * bt.B + first]);
                }
                for (; i < N; ++i) add_signed(acc, bw[(size_t)i * brow], bt.scales[(size_t)i * bt.B + first]);
            } else {
                uint32_t bidx[16];
#pragma unroll
                for (int b = 0; b < 16; ++b) {
                    const uint32_t j = j0 + (b >> 2) * kChunk + (b & 3);
                    bidx[b] = block_of(bt, first, j < d ? j : d - 1);
                }
                for (int i = 0; i < N; ++i) {
                    const uint32_t m = bw[(size_t)i * brow];
                    const float* __restrict__ sc = bt.scales + (size_t)i * bt.B;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        acc[u].x = __fadd_rn(acc[u].x, signed_scale(m, 4 * u + 0, sc[bidx[4 * u + 0]]));
                        acc[u].y = __fadd_rn(acc[u].y, signed_scale(m, 4 * u + 1, sc[bidx[4 * u + 1]]));
                        acc[u].z = __fadd_rn(acc[u].z, signed_scale(m, 4 * u + 2, sc[bidx[4 * u + 2]]));
                        acc[u].w = __fadd_rn(acc[u].w, signed_scale(m, 4 * u + 3, sc[bidx[4 * u + 3]]));
                    }
                }
            }
        } else if (WC == kTopk && BATCH) {
            // Short rows: the kernel is bound by the latency of its dependent loads (group word, then gather, row
            // after row), not by bytes.  So the group words of 8 rows are requested together, then, chunk by
            // chunk, the flagged groups of those 8 rows, and only then are they added, in worker order.
            const uint64_t* __restrict__ gw = gbits + (coarse ? (size_t)t : (size_t)t * 4);
            const size_t grow = coarse ? (size_t)nwt : (size_t)nwt * 4;
            const uint32_t four = lane >> 2;
            for (int i0 = 0; i0 < N; i0 += 8) {
                uint32_t mask[8], tau[8], cut[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int i = i0 + r;
                    mask[r] = 0;
                    tau[r] = 0;
                    cut[r] = 0;
                    if (i < N) {                                // uniform
                        tau[r] = desc[i].tau;
                        cut[r] = desc[i].cutoff;
                        if (desc[i].dense) {
                            mask[r] = 0xfu;
                        } else if (coarse) {
                            mask[r] = (uint32_t)(gw[(size_t)i * grow] >> (4 * four)) & 0xfu;
                        } else {
                            const uint64_t* __restrict__ w = gw + (size_t)i * grow;
                            mask[r] = (uint32_t)((w[0] >> lane) & 1) | (uint32_t)((w[1] >> lane) & 1) << 1 |
                                      (uint32_t)((w[2] >> lane) & 1) << 2 | (uint32_t)((w[3] >> lane) & 1) << 3;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t j = j0 + u * kChunk;
                    float4 gq[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        gq[r] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if ((mask[r] >> u) & 1u) gq[r] = ld4<VEC>(grads + (size_t)(i0 + r) * d, j, d);
                    }
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        if ((mask[r] >> u) & 1u) {
                            const float gv[4] = {gq[r].x, gq[r].y, gq[r].z, gq[r].w};
                            float* av[4] = {&acc[u].x, &acc[u].y, &acc[u].z, &acc[u].w};
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const uint32_t key = key_of(gv[q]);
                                if (j + q < d && (key > tau[r] || (key == tau[r] && j + q <= cut[r])))
                                    *av[q] = __fadd_rn(*av[q], gv[q]);
                            }
                        }
                    }
                }
            }
        } else if (WC == kTopk) {
            float* my = accs + threadIdx.x;                    // slot b of this lane: my[b * kBlock]
#pragma unroll
            for (int b = 0; b < 16; ++b) my[b * kBlock] = 0.f;
            // the tile's group word(s) of row 0: one (coarse: bit 4m + u for 64-byte line m of chunk u) or four (a bit per lane)
            const uint64_t* __restrict__ gw = gbits + (coarse ? (size_t)t : (size_t)t * 4);
            const size_t grow = coarse ? (size_t)nwt : (size_t)nwt * 4;
            const uint32_t four = lane >> 2;                   // my 64-byte line inside a chunk
            for (int i = 0; i < N; ++i) {
                const float* __restrict__ gi = grads + (size_t)i * d;
                const uint32_t tau = desc[i].tau, cut = desc[i].cutoff;
                uint32_t mask = 0xfu;                          // bit u: my line of chunk u holds a candidate
                if (!desc[i].dense && coarse) {
                    mask = (uint32_t)(gw[(size_t)i * grow] >> (4 * four)) & 0xfu;   // bit 4 * line + chunk
                } else if (!desc[i].dense) {
                    const uint64_t* __restrict__ w = gw + (size_t)i * grow;
                    mask = (uint32_t)((w[0] >> lane) & 1) | (uint32_t)((w[1] >> lane) & 1) << 1 |
                           (uint32_t)((w[2] >> lane) & 1) << 2 | (uint32_t)((w[3] >> lane) & 1) << 3;
                }
                while (mask) {
                    const int u = __builtin_ctz(mask);
                    mask &= mask - 1;
                    const uint32_t j = j0 + u * kChunk;
                    const float4 g = ld4<VEC>(gi, j, d);
                    const float gv[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t key = key_of(gv[q]);
                        if (j + q < d && (key > tau || (key == tau && j + q <= cut))) {
                            float* slot = my + (4 * u + q) * kBlock;
                            *slot = __fadd_rn(*slot, gv[q]);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc[u] = make_float4(my[(4 * u) * kBlock], my[(4 * u + 1) * kBlock], my[(4 * u + 2) * kBlock],
                                     my[(4 * u + 3) * kBlock]);
        } else if (WC == kRandk) {
            // the kept bitmap of each row (one half-word per lane and wave tile) names the columns to fetch
            float* my = accs + threadIdx.x;
#pragma unroll
            for (int b = 0; b < 16; ++b) my[b * kBlock] = 0.f;
            const uint16_t* __restrict__ bw = bits + (size_t)t * 64 + lane;
            const size_t brow = (size_t)nwt * 64;
            for (int i = 0; i < N; ++i) {
                const float* __restrict__ gi = grads + (size_t)i * d;
                uint32_t m = bw[(size_t)i * brow];
                while (m) {
                    const int u = __builtin_ctz(m) >> 2;
                    const uint32_t nib = (m >> (4 * u)) & 0xfu;
                    m &= ~(0xfu << (4 * u));
                    const float4 g = ld4<VEC>(gi, j0 + u * kChunk, d);
                    const float gv[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if ((nib >> q) & 1) {
                            float* slot = my + (4 * u + q) * kBlock;
                            *slot = __fadd_rn(*slot, gv[q]);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc[u] = make_float4(my[(4 * u) * kBlock], my[(4 * u + 1) * kBlock], my[(4 * u + 2) * kBlock],
                                     my[(4 * u + 3) * kBlock]);
        } else {
            for (int i = 0; i < N; ++i) {
                const float* __restrict__ gi = grads + (size_t)i * d;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float4 g = ld4<VEC, true>(gi, j0 + u * kChunk, d);
                    acc[u].x = __fadd_rn(acc[u].x, g.x);
                    acc[u].y = __fadd_rn(acc[u].y, g.y);
                    acc[u].z = __fadd_rn(acc[u].z, g.z);
                    acc[u].w = __fadd_rn(acc[u].w, g.w);
                }
            }
        }
        uint32_t vm = 0;                                        // sign bits of my 16 values of v
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = j0 + u * kChunk;
            const float4 e = ld4<VEC>(e_in, j, d);
            float4 v;
            v.x = __fmaf_rn(acc[u].x, inv_n, e.x);
            v.y = __fmaf_rn(acc[u].y, inv_n, e.y);
            v.z = __fmaf_rn(acc[u].z, inv_n, e.z);
            v.w = __fmaf_rn(acc[u].w, inv_n, e.w);
            vm |= ((v.x < 0.f ? 1u : 0u) | (v.y < 0.f ? 2u : 0u) | (v.z < 0.f ? 4u : 0u) | (v.w < 0.f ? 8u : 0u)) << (4 * u);
            // with the gathering operators a streaming store of v measured 10 % faster, with the others slower
            if (WC == kTopk || WC == kRandk) st4<VEC, true>(v_out, j, d, v);
            else st4<VEC>(v_out, j, d, v);
            if (SRV_L1) {
                if (j < d) l1 += (double)fabsf(v.x);
                if (j + 1 < d) l1 += (double)fabsf(v.y);
                if (j + 2 < d) l1 += (double)fabsf(v.z);
                if (j + 3 < d) l1 += (double)fabsf(v.w);
            }
        }
        // a scaled-sign server's message is these bits and one scale: the update kernel reads them instead of v
        if (vbits) vbits[(size_t)t * 64 + lane] = (uint16_t)vm;
    }
    if (SRV_L1) {
        const double s = block_sum_f64(l1, lds_w);
        if (threadIdx.x == 0) srv_partial[blockIdx.x] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// Server compression + error update + broadcast + local immediate compensation (Algorithm 1):
//   p_j = C_s(v)_j ; e_j <- v_j - p_j ; x_ij <- x_ij - lr * (p_j + (g_ij - p^i_j)).
// One block = 1024 columns of one row.  Blocks are ordered panel by panel (a panel is `panel`
// consecutive column tiles), inside a panel row by row, so every row is walked in long contiguous
// runs while the panel's slice of v stays in cache for the N rows that reuse it; the row-0 block of
// a tile also writes e.  grid = number of panels * panel * N.
// ---------------------------------------------------------------------------------------------
template <int WC, int SC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_update(const float* __restrict__ grads, float* __restrict__ x,
                                                    const float* __restrict__ v_in, float* __restrict__ e_out, int N,
                                                    uint32_t panel, uint32_t ncol_tiles, uint32_t d, float neg_lr,
                                                    const RowDesc* __restrict__ desc, BlockTable bt,
                                                    const uint16_t* __restrict__ kbits, const uint16_t* __restrict__ vbits,
                                                    const uint64_t* __restrict__ sgbits) {
    const uint32_t per_panel = panel * (uint32_t)N;
    const uint32_t pn = blockIdx.x / per_panel, r = blockIdx.x % per_panel;
    const uint32_t i = r / panel, tile = pn * panel + r % panel;
    if (tile >= ncol_tiles) return;
    const uint32_t j = tile * kColTile + threadIdx.x * 4;
    if (j >= d) return;
    const float* __restrict__ gi = grads + (size_t)i * d;
    float* __restrict__ xi = x + (size_t)i * d;
    const uint32_t lane = threadIdx.x & 63, chunk = threadIdx.x >> 6;   // this thread is lane `lane` of chunk `chunk` of wave tile `tile`
    uint32_t tb = 0;
    if (WC == kBlockSign || SC == kBlockSign) tb = bt.tile_blk[tile];   // issued ahead of the streams
    // random-k: the 4 kept bits of this thread's columns; row N of the bitmap is the server's draw
    uint32_t wkeep = 0, skeep = 0;
    if (WC == kRandk) wkeep = (kbits[((size_t)i * ncol_tiles + tile) * 64 + lane] >> (4 * chunk)) & 0xfu;
    if (SC == kRandk) skeep = (kbits[((size_t)N * ncol_tiles + tile) * 64 + lane] >> (4 * chunk)) & 0xfu;
    const RowDesc* __restrict__ sd = desc + N;
    // What the server's message needs of v.  The row-0 block of a tile reads v in full (it writes e).  The other
    // rows' blocks take what the server side left behind instead of re-reading 4 d bytes of v per row: the sign
    // bits of v (scaled sign, either form), the candidate bit of these 4 columns (top-k: v is read only where
    // a candidate sits, unless the row's bitmap is not valid), the kept bits (random-k).
    uint32_t sbits = 0;
    bool need_v = true;
    if (i != 0) {
        if (SC == kSign || SC == kBlockSign) {
            sbits = ((uint32_t)vbits[(size_t)tile * 64 + lane] >> (4 * chunk)) & 0xfu;
            need_v = false;
        } else if (SC == kTopk) {
            need_v = sd->dense || ((sgbits[(size_t)tile * 4 + chunk] >> lane) & 1u);
        } else if (SC == kRandk) {
            need_v = skeep != 0;
        }
    }
    const float4 g = ld4<VEC, true>(gi, j, d);
#if defined(__HIP_DEVICE_COMPILE__)
    // One stream at a time per wave: waiting for the gradients before asking for the model measured
    // 2-4 % faster than having both 128-bit loads in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    const float4 xv = ld4<VEC, true>(xi, j, d);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (need_v) v = ld4<VEC>(v_in, j, d);
    const uint32_t stau = sd->tau, scut = sd->cutoff;
    float sw[4], ss[4];                                    // worker / server scale of each of the 4 columns
    if (WC == kBlockSign || SC == kBlockSign) {
        const uint32_t first = tb & 0x7fffffffu;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t b = (tb >> 31) ? block_of(bt, first, j + c < d ? j + c : d - 1) : first;
            sw[c] = WC == kBlockSign ? bt.scales[(size_t)i * bt.B + b] : desc[i].scale;
            ss[c] = SC == kBlockSign ? bt.scales[(size_t)N * bt.B + b] : sd->scale;
        }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            sw[c] = desc[i].scale;
            ss[c] = sd->scale;
        }
    }
    float4 p;
    if ((SC == kSign || SC == kBlockSign) && i != 0) {
        p.x = (sbits & 1u) ? -ss[0] : ss[0];
        p.y = (sbits & 2u) ? -ss[1] : ss[1];
        p.z = (sbits & 4u) ? -ss[2] : ss[2];
        p.w = (sbits & 8u) ? -ss[3] : ss[3];
    } else {                                               // for columns whose v was not read p is +0, as v is
        p.x = message_of<SC>(v.x, j, ss[0], stau, scut, skeep & 1u);
        p.y = message_of<SC>(v.y, j + 1, ss[1], stau, scut, skeep & 2u);
        p.z = message_of<SC>(v.z, j + 2, ss[2], stau, scut, skeep & 4u);
        p.w = message_of<SC>(v.w, j + 3, ss[3], stau, scut, skeep & 8u);
    }
    if (i == 0) {
        float4 en;
        en.x = __fsub_rn(v.x, p.x);
        en.y = __fsub_rn(v.y, p.y);
        en.z = __fsub_rn(v.z, p.z);
        en.w = __fsub_rn(v.w, p.w);
        st4<VEC>(e_out, j, d, en);
    }
    const uint32_t tau = desc[i].tau, cut = desc[i].cutoff;
    float4 o;
    o.x = __fmaf_rn(neg_lr, __fadd_rn(p.x, __fsub_rn(g.x, message_of<WC>(g.x, j, sw[0], tau, cut, wkeep & 1u))), xv.x);
    o.y = __fmaf_rn(neg_lr, __fadd_rn(p.y, __fsub_rn(g.y, message_of<WC>(g.y, j + 1, sw[1], tau, cut, wkeep & 2u))), xv.y);
    o.z = __fmaf_rn(neg_lr, __fadd_rn(p.z, __fsub_rn(g.z, message_of<WC>(g.z, j + 2, sw[2], tau, cut, wkeep & 4u))), xv.z);
    o.w = __fmaf_rn(neg_lr, __fadd_rn(p.w, __fsub_rn(g.w, message_of<WC>(g.w, j + 3, sw[3], tau, cut, wkeep & 8u))), xv.w);
    st4<VEC, true>(xi, j, d, o);
}

}  // namespace liec
