// Device kernels of the LIEC-SGD compressed step for gfx950 (CDNA4, wave64).
//
// Element ownership is the same in every kernel: a block of 256 threads walks
// "tiles" of 1024 consecutive columns; inside a tile, wave w owns the 256-column
// "chunk" 4*tile + w and lane l owns columns 4l..4l+3 of that chunk (one 128-bit
// access per lane, 1 KiB contiguous per wave).  All fp32 arithmetic that reaches
// the outputs is written as single IEEE operations (__fadd_rn / __fsub_rn /
// __fmaf_rn) so that the result does not depend on compiler contraction.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace liec {

constexpr int kBlock = 256;             // threads per block (4 waves)
constexpr int kTile = kBlock * 4;       // columns per block iteration
constexpr int kChunk = 256;             // columns per wave iteration
constexpr int kHistBins = 4096;         // widest radix digit (12 bits)

enum Comp : int { kIdentity = 0, kSign = 1, kTopk = 2 };

// One per worker row, plus one (index N) for the server's vector v.
struct RowDesc {
    double l1;             // scaled sign: sum |v_j| (fp64)
    float scale;           // scaled sign: fp32(l1 / d)
    uint32_t tau;          // top-k: key prefix while the digits are being resolved, then the k-th key
    uint32_t rank;         // top-k: rank still to be located inside the current prefix (1-based);
                           //        after the last digit: how many entries with key == tau are kept
    uint32_t ties;         // top-k: how many entries have key == tau
    uint32_t cutoff;       // top-k: largest kept index among entries with key == tau
    uint32_t nonfinite;    // a NaN/Inf reached the L1 sum or a key
};

// Radix digits of the 31-bit magnitude key, most significant first.
__host__ __device__ constexpr int digit_shift(int pass) { return pass == 0 ? 19 : (pass == 1 ? 9 : 0); }
__host__ __device__ constexpr int digit_bits(int pass) { return pass == 0 ? 12 : (pass == 1 ? 10 : 9); }

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// 4 consecutive floats starting at column j of a row of length d; zero beyond d.
template <bool VEC>
__device__ __forceinline__ float4 ld4(const float* __restrict__ row, uint32_t j, uint32_t d) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (VEC) {
        if (j < d) r = *reinterpret_cast<const float4*>(row + j);
    } else {
        if (j < d) r.x = row[j];
        if (j + 1 < d) r.y = row[j + 1];
        if (j + 2 < d) r.z = row[j + 2];
        if (j + 3 < d) r.w = row[j + 3];
    }
    return r;
}

template <bool VEC>
__device__ __forceinline__ void st4(float* __restrict__ row, uint32_t j, uint32_t d, float4 v) {
    if (VEC) {
        if (j < d) *reinterpret_cast<float4*>(row + j) = v;
    } else {
        if (j < d) row[j] = v.x;
        if (j + 1 < d) row[j + 1] = v.y;
        if (j + 2 < d) row[j + 2] = v.z;
        if (j + 3 < d) row[j + 3] = v.w;
    }
}

// Sum over the block in a fixed order (lanes by halving, then waves 0..3).
// The result is valid on thread 0 only.
__device__ __forceinline__ double block_sum_f64(double v, double* lds4) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds4[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) r = ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
    return r;
}

// ---------------------------------------------------------------------------------------------
// Scaled sign, worker side (Definition 4): per-row partial sums of |g| in fp64 and, optionally,
// the sign bits of the row.  Bit layout: for chunk c of row i, four 64-bit words
// bits[(i*nchunks + c)*4 + q], q = 0..3; bit l of word q is (g[256c + 4l + q] < 0).
// grid = (blocks per row, rows); block b of a row handles tiles b*tpb .. (b+1)*tpb - 1.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_l1_bits(const float* __restrict__ src, size_t row_stride,
                                                     uint32_t d, uint32_t ntiles, uint32_t tpb,
                                                     double* __restrict__ partial,
                                                     uint64_t* __restrict__ bits, uint32_t nchunks) {
    __shared__ double lds4[4];
    const uint32_t row = blockIdx.y;
    const float* __restrict__ g = src + (size_t)row * row_stride;
    const uint32_t t0 = blockIdx.x * tpb;
    const uint32_t t1 = min(t0 + tpb, ntiles);
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    double acc = 0.0;
#pragma unroll 4
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t j = t * kTile + threadIdx.x * 4;
        const float4 a = ld4<VEC>(g, j, d);
        acc += (double)fabsf(a.x);
        acc += (double)fabsf(a.y);
        acc += (double)fabsf(a.z);
        acc += (double)fabsf(a.w);
        if (bits) {
            const uint64_t b0 = __ballot(a.x < 0.f), b1 = __ballot(a.y < 0.f);
            const uint64_t b2 = __ballot(a.z < 0.f), b3 = __ballot(a.w < 0.f);
            const uint32_t chunk = t * 4 + wave;
            if (lane < 4 && chunk < nchunks) {
                const uint64_t w = lane == 0 ? b0 : (lane == 1 ? b1 : (lane == 2 ? b2 : b3));
                bits[((size_t)row * nchunks + chunk) * 4 + lane] = w;
            }
        }
    }
    const double s = block_sum_f64(acc, lds4);
    if (threadIdx.x == 0) partial[(size_t)row * gridDim.x + blockIdx.x] = s;
}

// Finishes the L1 norm of each row from its block partials (fixed order) and sets the scale.
// grid = rows, desc points at the first row's descriptor.
__global__ __launch_bounds__(kBlock) void k_l1_final(const double* __restrict__ partial, uint32_t nparts,
                                                      uint32_t d, RowDesc* __restrict__ desc) {
    __shared__ double lds4[4];
    const uint32_t row = blockIdx.x;
    const double* __restrict__ p = partial + (size_t)row * nparts;
    double acc = 0.0;
    for (uint32_t q = threadIdx.x; q < nparts; q += kBlock) acc += p[q];
    const double s = block_sum_f64(acc, lds4);
    if (threadIdx.x == 0) {
        desc[row].l1 = s;
        desc[row].scale = (float)(s / (double)d);
        desc[row].nonfinite = (s - s == 0.0) ? 0u : 1u;   // false for NaN and Inf
    }
}

// ---------------------------------------------------------------------------------------------
// Top-k (Definition 2) threshold search: radix select on the 31-bit magnitude key.
// k_hist counts, per row, the current digit of every key whose higher digits equal the prefix
// found so far; k_pick walks the counts from the top to the bin holding the wanted rank.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_hist(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                  uint32_t ntiles, uint32_t tpb, const RowDesc* __restrict__ desc,
                                                  int pass, uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[kHistBins];
    const uint32_t row = blockIdx.y;
    const float* __restrict__ g = src + (size_t)row * row_stride;
    const int shift = digit_shift(pass), nbins = 1 << digit_bits(pass);
    const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);   // bits above this digit
    const uint32_t prefix = pass == 0 ? 0u : desc[row].tau;
    for (int b = threadIdx.x; b < nbins; b += kBlock) h[b] = 0;
    __syncthreads();
    const uint32_t t0 = blockIdx.x * tpb;
    const uint32_t t1 = min(t0 + tpb, ntiles);
#pragma unroll 2
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t j = t * kTile + threadIdx.x * 4;
        const float4 a = ld4<VEC>(g, j, d);
        const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = key_of(av[c]);
            const bool match = (j + c < d) && (((key ^ prefix) >> hi_shift) == 0);
            if (match) atomicAdd(&h[(key >> shift) & (nbins - 1)], 1u);
        }
    }
    __syncthreads();
    uint32_t* __restrict__ out = hist + (size_t)row * kHistBins;
    for (int b = threadIdx.x; b < nbins; b += kBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// grid = rows.  Finds the bin of the current digit that holds the entry of rank `rank`
// (counting from the largest key), extends the prefix, and clears the histogram for reuse.
template <int PASS>
__global__ __launch_bounds__(kBlock) void k_pick(RowDesc* __restrict__ desc, uint32_t* __restrict__ hist, uint32_t k) {
    constexpr int nbins = 1 << digit_bits(PASS);
    constexpr int per = nbins / kBlock;                 // 16, 4 or 2 bins per thread
    __shared__ uint32_t part[kBlock];
    __shared__ uint32_t above_of[kBlock];               // count in the bins above the thread's range
    const uint32_t row = blockIdx.x;
    uint32_t* __restrict__ h = hist + (size_t)row * kHistBins;
    const uint32_t rank = PASS == 0 ? k : desc[row].rank;
    uint32_t local[per];
    uint32_t sum = 0;
    bool bad = false;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        local[q] = h[threadIdx.x * per + q];
        sum += local[q];
        // keys at or above 0x7f800000 are Inf/NaN: the top 8 of the 12 first-digit bits all ones
        if (PASS == 0) bad |= (local[q] != 0) && ((threadIdx.x * per + q) >= 0xff0);
        h[threadIdx.x * per + q] = 0;
    }
    part[threadIdx.x] = sum;
    const int any_bad = __syncthreads_or(bad ? 1 : 0);
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int t = kBlock - 1; t >= 0; --t) {
            above_of[t] = run;
            run += part[t];
        }
    }
    __syncthreads();
    const uint32_t above = above_of[threadIdx.x];
    if (above < rank && rank <= above + sum) {           // true for exactly one thread
        uint32_t run = above, bin = threadIdx.x * per, ties = local[0];
        bool done = false;
#pragma unroll
        for (int q = per - 1; q >= 0; --q) {
            if (!done && run + local[q] >= rank) {
                bin = threadIdx.x * per + q;
                ties = local[q];
                done = true;
            }
            if (!done) run += local[q];
        }
        RowDesc r = desc[row];
        if (PASS == 0) {
            r.tau = 0;
            r.nonfinite = any_bad ? 1u : 0u;
        }
        r.tau |= bin << digit_shift(PASS);
        r.rank = rank - run;
        r.ties = ties;
        desc[row] = r;
    }
}

// Ties at the threshold are admitted by increasing index.  k_tie_count counts, per block span of
// a row, the entries whose key equals tau; k_tie_pick then locates the rank-th of them.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_tie_count(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                       uint32_t ntiles, uint32_t tpb,
                                                       const RowDesc* __restrict__ desc, uint32_t* __restrict__ cnt) {
    __shared__ uint32_t wsum[4];
    const uint32_t row = blockIdx.y;
    const float* __restrict__ g = src + (size_t)row * row_stride;
    const uint32_t tau = desc[row].tau;
    const uint32_t t0 = blockIdx.x * tpb;
    const uint32_t t1 = min(t0 + tpb, ntiles);
    uint32_t c = 0;
#pragma unroll 4
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t j = t * kTile + threadIdx.x * 4;
        const float4 a = ld4<VEC>(g, j, d);
        c += (j < d && key_of(a.x) == tau) + (j + 1 < d && key_of(a.y) == tau) +
             (j + 2 < d && key_of(a.z) == tau) + (j + 3 < d && key_of(a.w) == tau);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) cnt[(size_t)row * gridDim.x + blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// grid = rows.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_tie_pick(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                      uint32_t ntiles, uint32_t tpb, uint32_t nblk,
                                                      RowDesc* __restrict__ desc, const uint32_t* __restrict__ cnt) {
    __shared__ uint32_t s_blk, s_rank;
    __shared__ uint32_t scan[kBlock];
    __shared__ uint32_t s_found;
    const uint32_t row = blockIdx.x;
    const float* __restrict__ g = src + (size_t)row * row_stride;
    const uint32_t tau = desc[row].tau;
    if (threadIdx.x == 0) {
        uint32_t want = desc[row].rank, run = 0, b = 0;
        for (; b + 1 < nblk; ++b) {
            const uint32_t c = cnt[(size_t)row * nblk + b];
            if (run + c >= want) break;
            run += c;
        }
        s_blk = b;
        s_rank = want - run;
        s_found = 0xffffffffu;
    }
    __syncthreads();
    const uint32_t t0 = s_blk * tpb;
    const uint32_t t1 = min(t0 + tpb, ntiles);
    uint32_t want = s_rank;
    for (uint32_t t = t0; t < t1; ++t) {           // uniform trip count and exit for the whole block
        const uint32_t j = t * kTile + threadIdx.x * 4;
        const float4 a = ld4<VEC>(g, j, d);
        const bool m0 = j < d && key_of(a.x) == tau, m1 = j + 1 < d && key_of(a.y) == tau;
        const bool m2 = j + 2 < d && key_of(a.z) == tau, m3 = j + 3 < d && key_of(a.w) == tau;
        const uint32_t mine = m0 + m1 + m2 + m3;
        scan[threadIdx.x] = mine;
        __syncthreads();
        if (threadIdx.x == 0) {                    // exclusive scan of 256 small counts
            uint32_t run = 0;
            for (int q = 0; q < kBlock; ++q) {
                const uint32_t c = scan[q];
                scan[q] = run;
                run += c;
            }
            s_rank = run;                          // total in this tile
        }
        __syncthreads();
        const uint32_t before = scan[threadIdx.x], total = s_rank;
        if (want <= total) {
            if (before < want && want <= before + mine) {
                uint32_t need = want - before;     // 1-based among this thread's matches
                uint32_t idx = j;
                if (m0 && --need == 0) idx = j;
                else if (m1 && --need == 0) idx = j + 1;
                else if (m2 && --need == 0) idx = j + 2;
                else idx = j + 3;
                s_found = idx;
            }
            break;                                 // `want` and `total` are block-uniform
        }
        want -= total;
        __syncthreads();
    }
    __syncthreads();
    if (threadIdx.x == 0) desc[row].cutoff = s_found;
}

// ---------------------------------------------------------------------------------------------
// Worker message element p^i_j rebuilt from g_ij and the row's descriptor.
// ---------------------------------------------------------------------------------------------
template <int WC>
__device__ __forceinline__ float message_of(float g, uint32_t j, float scale, uint32_t tau, uint32_t cutoff) {
    if (WC == kSign) return g < 0.f ? -scale : scale;
    if (WC == kTopk) {
        const uint32_t key = key_of(g);
        return (key > tau || (key == tau && j <= cutoff)) ? g : 0.f;
    }
    return g;
}

// ---------------------------------------------------------------------------------------------
// Server compensation (Algorithm 1): v_j = e_j + (1/N) sum_i p^i_j, messages added in worker
// order.  v overwrites e in place.  With SRV_L1 the kernel also emits per-block partial sums of
// |v| (fp64) for the server's scaled-sign operator.  grid = blocks, each handling tpb tiles.
// FROM_BITS (scaled-sign workers only) reads the packed sign bits instead of the gradients.
// ---------------------------------------------------------------------------------------------
template <int WC, bool FROM_BITS, bool SRV_L1, bool VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate(const float* __restrict__ grads, const uint64_t* __restrict__ bits,
                                                       uint32_t nchunks, int N, uint32_t d, uint32_t ntiles,
                                                       uint32_t tpb, float inv_n, const RowDesc* __restrict__ desc,
                                                       float* __restrict__ e_inout, double* __restrict__ srv_partial) {
    __shared__ double lds4[4];
    const uint32_t t0 = blockIdx.x * tpb;
    const uint32_t t1 = min(t0 + tpb, ntiles);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    double l1 = 0.0;
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t j = t * kTile + threadIdx.x * 4;
        const float4 e = ld4<VEC>(e_inout, j, d);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (FROM_BITS) {
            const uint32_t chunk = t * 4 + wave;               // wave-uniform
            if (chunk < nchunks) {
#pragma unroll 4
                for (int i = 0; i < N; ++i) {
                    const uint64_t* __restrict__ w = bits + ((size_t)i * nchunks + chunk) * 4;
                    const float s = desc[i].scale;
                    acc.x = __fadd_rn(acc.x, ((w[0] >> lane) & 1) ? -s : s);
                    acc.y = __fadd_rn(acc.y, ((w[1] >> lane) & 1) ? -s : s);
                    acc.z = __fadd_rn(acc.z, ((w[2] >> lane) & 1) ? -s : s);
                    acc.w = __fadd_rn(acc.w, ((w[3] >> lane) & 1) ? -s : s);
                }
            }
        } else {
#pragma unroll 4
            for (int i = 0; i < N; ++i) {
                const float4 g = ld4<VEC>(grads + (size_t)i * d, j, d);
                const float s = desc[i].scale;
                const uint32_t tau = desc[i].tau, cut = desc[i].cutoff;
                acc.x = __fadd_rn(acc.x, message_of<WC>(g.x, j, s, tau, cut));
                acc.y = __fadd_rn(acc.y, message_of<WC>(g.y, j + 1, s, tau, cut));
                acc.z = __fadd_rn(acc.z, message_of<WC>(g.z, j + 2, s, tau, cut));
                acc.w = __fadd_rn(acc.w, message_of<WC>(g.w, j + 3, s, tau, cut));
            }
        }
        float4 v;
        v.x = __fmaf_rn(acc.x, inv_n, e.x);
        v.y = __fmaf_rn(acc.y, inv_n, e.y);
        v.z = __fmaf_rn(acc.z, inv_n, e.z);
        v.w = __fmaf_rn(acc.w, inv_n, e.w);
        st4<VEC>(e_inout, j, d, v);
        if (SRV_L1) {
            if (j < d) l1 += (double)fabsf(v.x);
            if (j + 1 < d) l1 += (double)fabsf(v.y);
            if (j + 2 < d) l1 += (double)fabsf(v.z);
            if (j + 3 < d) l1 += (double)fabsf(v.w);
        }
    }
    if (SRV_L1) {
        const double s = block_sum_f64(l1, lds4);
        if (threadIdx.x == 0) srv_partial[blockIdx.x] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// Server compression + error update + broadcast + local immediate compensation (Algorithm 1):
//   p_j = C_s(v)_j ; e_j <- v_j - p_j ; x_ij <- x_ij - lr * (p_j + (g_ij - p^i_j)).
// v is read from (and e written to) the same buffer.  grid = tiles; a block owns 1024 columns
// of every row.
// ---------------------------------------------------------------------------------------------
template <int WC, int SC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_update(const float* __restrict__ grads, float* __restrict__ x,
                                                    float* __restrict__ e_inout, int N, uint32_t d, float neg_lr,
                                                    const RowDesc* __restrict__ desc) {
    const uint32_t j = blockIdx.x * kTile + threadIdx.x * 4;
    if (j >= d) return;
    const float4 v = ld4<VEC>(e_inout, j, d);
    const RowDesc* __restrict__ sd = desc + N;
    const float ss = sd->scale;
    const uint32_t stau = sd->tau, scut = sd->cutoff;
    float4 p;
    p.x = message_of<SC>(v.x, j, ss, stau, scut);
    p.y = message_of<SC>(v.y, j + 1, ss, stau, scut);
    p.z = message_of<SC>(v.z, j + 2, ss, stau, scut);
    p.w = message_of<SC>(v.w, j + 3, ss, stau, scut);
    float4 en;
    en.x = __fsub_rn(v.x, p.x);
    en.y = __fsub_rn(v.y, p.y);
    en.z = __fsub_rn(v.z, p.z);
    en.w = __fsub_rn(v.w, p.w);
    st4<VEC>(e_inout, j, d, en);
#pragma unroll 4
    for (int i = 0; i < N; ++i) {
        const float* __restrict__ gi = grads + (size_t)i * d;
        float* __restrict__ xi = x + (size_t)i * d;
        const float4 g = ld4<VEC>(gi, j, d);
        const float4 xv = ld4<VEC>(xi, j, d);
        const float s = desc[i].scale;
        const uint32_t tau = desc[i].tau, cut = desc[i].cutoff;
        float4 o;
        o.x = __fmaf_rn(neg_lr, __fadd_rn(p.x, __fsub_rn(g.x, message_of<WC>(g.x, j, s, tau, cut))), xv.x);
        o.y = __fmaf_rn(neg_lr, __fadd_rn(p.y, __fsub_rn(g.y, message_of<WC>(g.y, j + 1, s, tau, cut))), xv.y);
        o.z = __fmaf_rn(neg_lr, __fadd_rn(p.z, __fsub_rn(g.z, message_of<WC>(g.z, j + 2, s, tau, cut))), xv.z);
        o.w = __fmaf_rn(neg_lr, __fadd_rn(p.w, __fsub_rn(g.w, message_of<WC>(g.w, j + 3, s, tau, cut))), xv.w);
        st4<VEC>(xi, j, d, o);
    }
}

// Plain device copy (128-bit), used to measure the achievable streaming bandwidth next to the
// step's kernels and to calibrate byte counters.
__global__ __launch_bounds__(kBlock) void k_copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ void k_fill_u32(uint32_t* __restrict__ p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

}  // namespace liec
