// Device kernels of the LIEC-SGD compressed step for gfx950 (CDNA4, wave64).
//
// Element ownership in the streaming kernels: a wave walks "wave tiles" of 1024 consecutive
// columns (4 chunks of 256); in chunk u, lane l owns columns 256u + 4l .. 256u + 4l + 3 (one
// 128-bit access per lane, 1 KiB contiguous per wave and instruction).  A block of 256 threads
// (4 waves) covers 4096 consecutive columns per iteration.  All fp32 arithmetic that reaches the
// outputs is written as single IEEE operations (__fadd_rn / __fsub_rn / __fmaf_rn) so that the
// result does not depend on compiler contraction.  Streams that are read or written once are
// accessed with non-temporal hints.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace liec {

constexpr int kBlock = 256;             // threads per block (4 waves)
constexpr int kChunk = 256;             // columns per wave and load instruction
constexpr int kWaveTile = 1024;         // columns per wave iteration
constexpr int kColTile = 1024;          // columns per block of the update kernel
constexpr int kHistBins = 4096;         // first radix digit of a whole row (12 bits)
constexpr int kSureStripes = 16;        // counters per row for the keys above the band
constexpr int kListBits = 13;           // widest radix digit of the list select (two digits cover a band of 2^26 keys)
constexpr int kListBins = 1 << kListBits;
constexpr int kStage = 512;             // per-wave LDS staging slots of the candidate filter
constexpr int kTieCap = 4096;           // ties at the threshold the fast path resolves
constexpr uint32_t kBandMargin = 1u << 18;   // least half width, in key units, of the predicted band (about 2 % in value)
constexpr uint32_t kUpdatePanel = 4096; // column tiles per panel of the update kernel

enum Comp : int { kIdentity = 0, kSign = 1, kTopk = 2, kBlockSign = 3, kRandk = 4 };

// Progress of a row's top-k threshold search within one step.
enum SelMode : uint32_t {
    kWarm = 0,      // a band [lo, hi) predicted from the previous step is filtered
    kCold = 1,      // no usable prediction: the first radix digit of the whole row is needed
    kColdBand = 2,  // band = the first-digit bin holding rank k; filtered by the second filter pass
    kSlow = 4       // needs the general (single block, multi pass) search over the row
};

// One per worker row, plus one (index N) for the server's vector v.
struct RowDesc {
    double l1;             // scaled sign: sum |v_j| (fp64)
    float scale;           // scaled sign: fp32(l1 / d)
    uint32_t tau;          // top-k: key of the k-th kept entry
    uint32_t rank;         // top-k: how many entries with key == tau are kept
    uint32_t ties;         // top-k: how many entries have key == tau
    uint32_t cutoff;       // top-k: largest kept index among entries with key == tau
    uint32_t nonfinite;    // a NaN/Inf reached the L1 sum or a key (last step)
    uint32_t nonfinite_acc;
    uint32_t lo, hi;       // candidate band: keys in [lo, hi) are listed, keys >= hi are surely kept
    uint32_t mode;         // SelMode
    uint32_t n_cand;       // candidates appended so far (may exceed the capacity: overflow)
    uint32_t n_sure[kSureStripes];   // keys at or above the band seen by the filter pass; block b of the filter adds
                           // to stripe b % kSureStripes (one address would serialise the blocks' atomics)
    uint32_t n_ties;       // ties collected
    uint32_t n_list;       // candidates that were listed when the search finished (random-k marks the kept ones)
    uint32_t dense;        // the row's candidate bitmap is not valid: test every column
    uint32_t sel_bin;      // list select: first digit of (tau - lo)
    uint32_t sel_rank;     // list select: rank of tau inside that digit's bin
    uint32_t prev_tau;     // tau of the step before (valid when have_prev)
    uint32_t have_prev;
    uint32_t was_cold;     // this step's band came from the first-digit histogram, not from a prediction
};

__host__ __device__ __forceinline__ uint32_t sure_count(const RowDesc& r) {
    uint32_t n = 0;
#pragma unroll
    for (int q = 0; q < kSureStripes; ++q) n += r.n_sure[q];
    return n;
}
__host__ __device__ __forceinline__ void clear_sure(RowDesc& r) {
#pragma unroll
    for (int q = 0; q < kSureStripes; ++q) r.n_sure[q] = 0;
}

// After a filter pass: the band is usable when its list did not overflow and rank k falls inside it.
__device__ __forceinline__ bool band_ok(const RowDesc& r, uint32_t cap, uint32_t k) {
    const uint32_t n_sure = sure_count(r);
    return r.n_cand <= cap && n_sure < k && (uint64_t)k <= (uint64_t)n_sure + r.n_cand &&
           r.hi - r.lo <= (1u << (2 * kListBits));       // the list select's two digits must span the band
}
// Rows that need the first-digit histogram: no prediction, or the predicted band failed.
__device__ __forceinline__ bool wants_cold(const RowDesc& r, uint32_t cap, uint32_t k) {
    return r.mode == kCold || (r.mode == kWarm && !band_ok(r, cap, k));
}
// Rows whose candidate list holds rank k (evaluated after both filter passes).
__device__ __forceinline__ bool listable(const RowDesc& r, uint32_t cap, uint32_t k) {
    return (r.mode == kWarm || r.mode == kColdBand) && band_ok(r, cap, k);
}

// Radix digits of the 31-bit magnitude key, most significant first.
__host__ __device__ constexpr int digit_shift(int pass) { return pass == 0 ? 19 : (pass == 1 ? 9 : 0); }
__host__ __device__ constexpr int digit_bits(int pass) { return pass == 0 ? 12 : (pass == 1 ? 10 : 9); }

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// ---------------------------------------------------------------------------------------------
// Random-k (Definition 3): the k-subset is drawn by giving index j the priority
// rk_priority(stream, j) and keeping the k highest (ties, at most pairs, to the lower index), so the
// draw is a top-k search over keys that do not depend on the data.  `stream` is one 64-bit word per
// (seed, draw, row): three rounds of a multiply-xorshift finalizer over seed, draw counter and row
// (worker index, or N for the server).  The per-index part is a keyed permutation of 32-bit words
// (every step is a bijection) with its lowest bit dropped: a 31-bit key like a magnitude key.
// ---------------------------------------------------------------------------------------------
struct RkState {               // in device memory, so that a captured step draws anew on every replay
    uint64_t seed, draw;       // draw: number of the draw the next step makes
};
struct RkDraw {
    const RkState* state;
    uint32_t fix_lo, fix_hi;   // band that holds rank k of uniform priorities (set by the host); fix_hi == 0: not random-k
};

__host__ __device__ __forceinline__ uint64_t rk_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t rk_stream(uint64_t seed, uint64_t draw, uint32_t row) {
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    uint64_t z = rk_mix64(seed + gamma);
    z = rk_mix64(z + draw + gamma);
    return rk_mix64(z + (uint64_t)row + gamma);
}
__host__ __device__ __forceinline__ uint32_t rk_priority(uint32_t k0, uint32_t k1, uint32_t j) {
    uint32_t h = j ^ k0;
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h += k1;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h >> 1;
}

typedef float v4f __attribute__((ext_vector_type(4)));

// 4 consecutive floats starting at column j of a row of length d; zero beyond d.
template <bool VEC, bool NT = false>
__device__ __forceinline__ float4 ld4(const float* __restrict__ row, uint32_t j, uint32_t d) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (VEC) {
        if (j < d) {
            if (NT) {
                const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(row + j));
                r = make_float4(t.x, t.y, t.z, t.w);
            } else {
                r = *reinterpret_cast<const float4*>(row + j);
            }
        }
    } else {
        if (j < d) r.x = row[j];
        if (j + 1 < d) r.y = row[j + 1];
        if (j + 2 < d) r.z = row[j + 2];
        if (j + 3 < d) r.w = row[j + 3];
    }
    return r;
}

template <bool VEC, bool NT = false>
__device__ __forceinline__ void st4(float* __restrict__ row, uint32_t j, uint32_t d, float4 v) {
    if (VEC) {
        if (j < d) {
            if (NT) {
                const v4f t = {v.x, v.y, v.z, v.w};
                __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(row + j));
            } else {
                *reinterpret_cast<float4*>(row + j) = v;
            }
        }
    } else {
        if (j < d) row[j] = v.x;
        if (j + 1 < d) row[j + 1] = v.y;
        if (j + 2 < d) row[j + 2] = v.z;
        if (j + 3 < d) row[j + 3] = v.w;
    }
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {   // set bits of mask below this lane
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Sum over the block in a fixed order (lanes by halving, then waves in order).  Valid on thread 0.
__device__ __forceinline__ double block_sum_f64(double v, double* lds_waves) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    if (lane == 0) lds_waves[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < nw; ++w) r += lds_waves[w];
    return r;
}

__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* lds_waves) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    if (lane == 0) lds_waves[wave] = v;
    __syncthreads();
    uint32_t r = 0;
    if (threadIdx.x == 0)
        for (int w = 0; w < nw; ++w) r += lds_waves[w];
    return r;
}

// Walks a histogram of nbins (a power of two from 256 to 8192) counts from the top bin down to the bin that
// holds the entry of rank `rank` (1-based, largest first).  Needs blockDim.x >= 256; every thread
// of the block must call it.  part: 256 words of LDS, res: 3 words of LDS.
struct Pick {
    uint32_t bin, rank_in, count;
};
__device__ __forceinline__ Pick block_pick(const uint32_t* __restrict__ h, int nbins, uint32_t rank,
                                           uint32_t* part, uint32_t* res) {
    const int per = nbins >> 8;   // 1 .. 32 bins per thread
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t local[32];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < 32; ++q) {
        local[q] = (tid < 256 && q < per) ? h[tid * per + q] : 0u;
        sum += local[q];
    }
    // count in the bins above this thread's range: suffix sum over the 256 threads (lanes, then waves)
    uint32_t incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += up;
    }
    if (tid < 256 && lane == 0) part[wave] = incl;             // total of wave `wave`
    if (tid == 0) {
        res[0] = 0;
        res[1] = 1;
        res[2] = 0;
    }
    __syncthreads();
    if (tid < 256) {
        uint32_t above = incl - sum;
        for (uint32_t w = wave + 1; w < 4; ++w) above += part[w];
        if (above < rank && rank <= above + sum) {   // true for exactly one thread
            uint32_t run = above, bin = tid * per, cnt = local[0];
            bool done = false;
#pragma unroll
            for (int q = 31; q >= 0; --q) {
                if (q < per) {
                    if (!done && run + local[q] >= rank) {
                        bin = tid * per + q;
                        cnt = local[q];
                        done = true;
                    }
                    if (!done) run += local[q];
                }
            }
            res[0] = bin;
            res[1] = rank - run;
            res[2] = cnt;
        }
    }
    __syncthreads();
    Pick p;
    p.bin = res[0];
    p.rank_in = res[1];
    p.count = res[2];
    __syncthreads();
    return p;
}

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
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
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
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
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

// ---------------------------------------------------------------------------------------------
// Top-k (Definition 2).  The k-th largest magnitude key tau of a row and the index cut-off
// among its ties are found without sorting:
//   1. k_filter streams the row once against a band [lo, hi) of keys expected to hold tau:
//      keys >= hi are only counted, keys inside the band are appended to a candidate list
//      (key, index), and a group bitmap is written for the aggregation kernel: 4 words of 64 bits
//      per wave tile, bit l of word u set when any of the 4 columns 1024t + 256u + 4l .. + 3 has
//      key >= lo (a quarter of the bytes a per-column bitmap would take; writes are what a
//      read stream pays most for).
//      The band is predicted from the previous step's tau (kWarm).  It is usable when the list
//      did not overflow and rank k falls inside it (band_ok); when there is no prediction, or it is not
//      usable, the band becomes the first-radix-digit bin holding rank k, found by k_hist0 +
//      k_pick_band over the whole row (-> kColdBand), and the row is filtered again.
//   2. k_list_hist<0>, k_list_hist<1>, k_list_ties and k_list_finish run a 2-digit radix select on
//      the listed keys, taken relative to the band's lower end, and order the ties by index.
//   3. Rows the list cannot hold (massive ties, degenerate data) take k_slow_select.
// All decisions are taken on the device per row, each kernel re-deriving from the row's counters
// whether it has work; only the one-block-per-row kernels (k_pick_band, k_list_finish,
// k_slow_select) change a row's mode.  The host always enqueues the same kernels.
// `row0` is added to blockIdx.y to address per-row state (the server's vector uses row N).
// ---------------------------------------------------------------------------------------------
// One chunk (256 columns, 4 per lane) of the filter: updates the per-lane count of keys >= hi and the
// running maximum key, returns the ballot of "any of my 4 columns has key >= lo" and, per component,
// the ballots of the candidates lo <= key < hi.  FULL: every column of the chunk is below d.
template <bool FULL>
__device__ __forceinline__ uint64_t filter_chunk(const uint32_t (&keys)[4], uint32_t j, uint32_t d, uint32_t lo, uint32_t hi,
                                                 uint32_t& cand4, uint64_t& any_cand,
                                                 uint32_t& n_hi, uint32_t& kmax, uint32_t& hi4) {
    // per lane: which of its 4 columns reach the band (lo4) and which lie above it (hi4); two ballots per
    // chunk tell the wave whether anything has to be listed (the per-column ballots are made only then)
    uint32_t lo4 = 0;
    hi4 = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t key = keys[q];
        const bool valid = FULL || j + q < d;
        const bool ge_lo = valid && key >= lo, ge_hi = valid && key >= hi;
        kmax = max(kmax, valid ? key : 0u);
        n_hi += ge_hi ? 1u : 0u;
        lo4 |= (ge_lo ? 1u : 0u) << q;
        hi4 |= (ge_hi ? 1u : 0u) << q;
    }
    cand4 = lo4 & ~hi4;
    any_cand = __ballot(cand4 != 0);
    return __ballot(lo4 != 0);
}

// RK: the keys are the priorities of a random-k draw (nothing is read from src), and instead of the
// group bitmap the kernel writes, per column, whether its key is at or above the band (lane-major
// half-words like the sign bits, at row `row` of kbits); k_rk_mark later adds the kept candidates.
template <bool VEC, bool RK>
__global__ __launch_bounds__(kBlock) void k_filter(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                    uint32_t nwt, uint32_t row0, RowDesc* __restrict__ desc,
                                                    uint32_t expect_mode, uint64_t* __restrict__ gbits,
                                                    uint16_t* __restrict__ kbits, uint2* __restrict__ list, uint32_t cap,
                                                    RkDraw rk) {
    __shared__ uint2 stage[4][kStage];
    __shared__ uint32_t wsure[4];
    const uint32_t row = row0 + blockIdx.y;
    if (desc[row].mode != expect_mode) return;                 // uniform for the block
    const uint32_t lo = desc[row].lo, hi = desc[row].hi;
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    uint2* __restrict__ out = list + (size_t)row * cap;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t k0 = 0, k1 = 0;
    if (RK) {
        const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
        k0 = (uint32_t)stream;
        k1 = (uint32_t)(stream >> 32);
    }
    uint2* st = stage[wave];
    uint32_t cnt = 0;                                           // staged candidates (wave-uniform)
    uint32_t n_hi = 0, kmax = 0;                                // per lane: keys >= hi seen, largest key seen
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        float4 a[4];
        if (!RK) {
#pragma unroll
            for (int u = 0; u < 4; ++u) a[u] = ld4<VEC, true>(g, t * kWaveTile + u * kChunk + lane * 4, d);
        }
        const bool full = (t + 1) * (uint32_t)kWaveTile <= d;  // wave-uniform
        uint64_t word = 0;                                      // lane u (< 4) ends up holding group word u
        uint32_t sure16 = 0;                                    // RK: bit 4u + q: my column q of chunk u has key >= hi
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            uint32_t keys[4];
            if (RK) {
#pragma unroll
                for (int q = 0; q < 4; ++q) keys[q] = rk_priority(k0, k1, j + q);
            } else {
                keys[0] = key_of(a[u].x);
                keys[1] = key_of(a[u].y);
                keys[2] = key_of(a[u].z);
                keys[3] = key_of(a[u].w);
            }
            uint64_t any_cand;
            uint32_t cand4, hi4;
            const uint64_t any_lo = full ? filter_chunk<true>(keys, j, d, lo, hi, cand4, any_cand, n_hi, kmax, hi4)
                                         : filter_chunk<false>(keys, j, d, lo, hi, cand4, any_cand, n_hi, kmax, hi4);
            word = lane == (uint32_t)u ? any_lo : word;
            sure16 |= hi4 << (4 * u);
            if (any_cand) {                                     // wave-uniform
                uint64_t bc[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) bc[q] = __ballot((cand4 >> q) & 1u);
                const uint32_t m = __popcll(bc[0]) + __popcll(bc[1]) + __popcll(bc[2]) + __popcll(bc[3]);
                if (cnt + m > kStage) {                         // flush the staged candidates
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    uint32_t base = 0;
                    if (lane == 0) base = atomicAdd(&desc[row].n_cand, cnt);
                    base = __builtin_amdgcn_readfirstlane(base);
                    for (uint32_t s = lane; s < cnt; s += 64)
                        if (base + s < cap) out[base + s] = st[s];
                    cnt = 0;
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
                uint32_t off = cnt;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((bc[q] >> lane) & 1) st[off + lanes_below(bc[q])] = make_uint2(keys[q], j + q);
                    off += __popcll(bc[q]);
                }
                cnt += m;
            }
        }
        if (RK) {
            kbits[((size_t)row * nwt + t) * 64 + lane] = (uint16_t)sure16;
        } else {
            if (gbits && lane < 4) gbits[((size_t)blockIdx.y * nwt + t) * 4 + lane] = word;
        }
    }
    // keys at or above 0x7f800000 are Inf / NaN (magnitude keys only: priorities use the whole range)
    if (!RK && __ballot(kmax >= 0x7f800000u) && lane == 0) atomicOr(&desc[row].nonfinite_acc, 1u);
    if (cnt) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&desc[row].n_cand, cnt);
        base = __builtin_amdgcn_readfirstlane(base);
        for (uint32_t s = lane; s < cnt; s += 64)
            if (base + s < cap) out[base + s] = st[s];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) n_hi += __shfl_down(n_hi, o, 64);
    if (lane == 0) wsure[wave] = n_hi;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t n = wsure[0] + wsure[1] + wsure[2] + wsure[3];
        if (n) atomicAdd(&desc[row].n_sure[blockIdx.x % kSureStripes], n);
    }
}

// First radix digit (12 bits) of every key of the rows that have no usable band.  grid = (blocks, rows).
template <bool VEC, bool RK>
__global__ __launch_bounds__(kBlock) void k_hist0(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                   uint32_t nwt, uint32_t row0, const RowDesc* __restrict__ desc,
                                                   uint32_t* __restrict__ hist, uint32_t cap, uint32_t k, RkDraw rk) {
    __shared__ uint32_t h[kHistBins];
    const uint32_t row = row0 + blockIdx.y;
    if (!wants_cold(desc[row], cap, k)) return;
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) h[b] = 0;
    __syncthreads();
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t k0 = 0, k1 = 0;
    if (RK) {
        const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
        k0 = (uint32_t)stream;
        k1 = (uint32_t)(stream >> 32);
    }
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        float4 a[4];
        if (!RK) {
#pragma unroll
            for (int u = 0; u < 4; ++u) a[u] = ld4<VEC, true>(g, t * kWaveTile + u * kChunk + lane * 4, d);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            uint32_t keys[4];
            if (RK) {
#pragma unroll
                for (int q = 0; q < 4; ++q) keys[q] = rk_priority(k0, k1, j + q);
            } else {
                keys[0] = key_of(a[u].x);
                keys[1] = key_of(a[u].y);
                keys[2] = key_of(a[u].z);
                keys[3] = key_of(a[u].w);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + q < d) atomicAdd(&h[keys[q] >> 19], 1u);
        }
    }
    __syncthreads();
    uint32_t* __restrict__ out = hist + (size_t)row * kHistBins;
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// grid = rows.  For the rows k_hist0 worked on: the band becomes the first-digit bin that holds rank k.
__global__ __launch_bounds__(kBlock) void k_pick_band(uint32_t row0, RowDesc* __restrict__ desc,
                                                       uint32_t* __restrict__ hist, uint32_t cap, uint32_t k) {
    __shared__ uint32_t part[256], res[3];
    const uint32_t row = row0 + blockIdx.x;
    if (!wants_cold(desc[row], cap, k)) return;
    uint32_t* __restrict__ h = hist + (size_t)row * kHistBins;
    const Pick p = block_pick(h, kHistBins, k, part, res);
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) h[b] = 0;
    if (threadIdx.x == 0) {
        RowDesc r = desc[row];
        r.lo = p.bin << 19;
        r.hi = (p.bin + 1) << 19;            // 0x80000000 for the top bin: no key reaches it
        r.n_cand = 0;
        clear_sure(r);
        r.was_cold = 1;
        r.mode = p.count <= cap ? kColdBand : kSlow;
        desc[row] = r;
    }
}

// Blocks of a list kernel that take part for a list of n entries: one per 2048 entries, so that a short
// list does not pay every block's fixed cost (histogram pick, LDS clear, flush).
__device__ __forceinline__ uint32_t list_blocks_for(uint32_t n, uint32_t grid) {
    const uint32_t want = (n + 2047u) / 2048u;
    return want < 1u ? 1u : (want > grid ? grid : want);
}

// List select: the keys of a band are taken relative to its lower end; the b bits that the band's width
// needs (b <= 26) are split into a low digit of ceil(b/2) bits and a high digit of the rest, so a narrow
// band (the usual 2^19 keys) gets two short histograms and a wide one still fits kListBins bins each.
struct ListDigits {
    int low_bits;
    uint32_t low_bins, high_bins;    // histogram sizes, at least 256 (what block_pick walks)
};
__device__ __forceinline__ ListDigits list_digits(const RowDesc& r) {
    const uint32_t width = r.hi - r.lo;                     // 1 .. 2^26 for a listable row
    const int b = width > 1 ? 32 - __clz((int)(width - 1)) : 1;
    ListDigits g;
    g.low_bits = (b + 1) / 2;
    g.low_bins = max(256u, 1u << g.low_bits);
    g.high_bins = max(256u, 1u << (b - g.low_bits));
    return g;
}

// P = 0: histogram of the high digit of every listed key.  P = 1: each block first redoes the pick of
// the high digit from its finished histogram, then counts the low digits of the keys in that bin.
// grid = (blocks, rows); lhist: [row][P][kListBins].
template <int P>
__global__ __launch_bounds__(kBlock) void k_list_hist(uint32_t row0, RowDesc* __restrict__ desc,
                                                       const uint2* __restrict__ list, uint32_t cap, uint32_t k,
                                                       uint32_t* __restrict__ lhist) {
    __shared__ uint32_t h[kListBins];
    __shared__ uint32_t part[256], res[3];
    const uint32_t row = row0 + blockIdx.y;
    if (!listable(desc[row], cap, k)) return;
    const uint32_t n = desc[row].n_cand;                       // <= cap for a listable row
    const uint32_t nb = list_blocks_for(n, gridDim.x);
    if (blockIdx.x >= nb) return;
    uint32_t* __restrict__ hrow = lhist + (size_t)row * 2 * kListBins;
    const uint32_t lo = desc[row].lo;
    const ListDigits dg = list_digits(desc[row]);
    const int nbins = (int)(P == 0 ? dg.high_bins : dg.low_bins);
    uint32_t bin0 = 0;
    if constexpr (P == 1) {
        const Pick p = block_pick(hrow, (int)dg.high_bins, k - sure_count(desc[row]), part, res);
        bin0 = p.bin;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            desc[row].sel_bin = p.bin;
            desc[row].sel_rank = p.rank_in;
        }
    }
    for (int b = threadIdx.x; b < nbins; b += kBlock) h[b] = 0;
    __syncthreads();
    const uint2* __restrict__ in = list + (size_t)row * cap;
    const uint32_t low_mask = (1u << dg.low_bits) - 1u;
    for (uint32_t e = blockIdx.x * kBlock + threadIdx.x; e < n; e += nb * kBlock) {
        const uint32_t rel = in[e].x - lo;
        if (P == 0) atomicAdd(&h[rel >> dg.low_bits], 1u);
        else if ((rel >> dg.low_bits) == bin0) atomicAdd(&h[rel & low_mask], 1u);
    }
    __syncthreads();
    uint32_t* __restrict__ out = hrow + P * kListBins;
    for (int b = threadIdx.x; b < nbins; b += kBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// Picks the low digit (-> tau, how many of its ties are kept, how many there are) and collects the
// indices of the listed entries whose key equals tau.  grid = (blocks, rows).
__global__ __launch_bounds__(kBlock) void k_list_ties(uint32_t row0, RowDesc* __restrict__ desc,
                                                       const uint2* __restrict__ list, uint32_t cap, uint32_t k,
                                                       const uint32_t* __restrict__ lhist,
                                                       uint32_t* __restrict__ tiebuf) {
    __shared__ uint32_t part[256], res[3];
    const uint32_t row = row0 + blockIdx.y;
    if (!listable(desc[row], cap, k)) return;
    const uint32_t n = desc[row].n_cand;
    const uint32_t nb = list_blocks_for(n, gridDim.x);
    if (blockIdx.x >= nb) return;
    const uint32_t* __restrict__ hrow = lhist + (size_t)row * 2 * kListBins;
    const ListDigits dg = list_digits(desc[row]);
    const Pick p = block_pick(hrow + kListBins, (int)dg.low_bins, desc[row].sel_rank, part, res);
    const uint32_t tau = desc[row].lo + ((desc[row].sel_bin << dg.low_bits) | p.bin);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        desc[row].tau = tau;
        desc[row].rank = p.rank_in;
        desc[row].ties = p.count;
    }
    const uint2* __restrict__ in = list + (size_t)row * cap;
    uint32_t* __restrict__ tb = tiebuf + (size_t)row * kTieCap;
    for (uint32_t e = blockIdx.x * kBlock + threadIdx.x; e < n; e += nb * kBlock) {
        const uint2 kv = in[e];
        if (kv.x == tau) {
            const uint32_t pos = atomicAdd(&desc[row].n_ties, 1u);
            if (pos < kTieCap) tb[pos] = kv.y;
        }
    }
}

// Band for the next step: centred on tau extrapolated by its last change, at least kBandMargin wide
// on either side, wider when tau is moving or when the last prediction failed.
__device__ __forceinline__ void predict_band(RowDesc& r, uint32_t fix_lo, uint32_t fix_hi) {
    if (fix_hi) {                                   // random-k: the band does not depend on the data
        r.lo = fix_lo;
        r.hi = fix_hi;
        r.prev_tau = r.tau;
        r.have_prev = 1;
        r.was_cold = 0;
        return;
    }
    const int64_t tau = (int64_t)r.tau;
    const int64_t delta = r.have_prev ? tau - (int64_t)r.prev_tau : 0;
    int64_t margin = 2 * (delta < 0 ? -delta : delta);
    if (margin < (int64_t)kBandMargin) margin = kBandMargin;
    if (r.was_cold && margin < 4 * (int64_t)kBandMargin) margin = 4 * (int64_t)kBandMargin;
    if (margin > (int64_t)1 << 25) margin = (int64_t)1 << 25;   // two list digits cover a band of 2^26 keys
    int64_t centre = tau + delta;
    if (centre < 0) centre = 0;
    if (centre > 0x7fffffffll) centre = 0x7fffffffll;
    const int64_t lo = centre - margin, hi = centre + margin;
    r.lo = lo < 0 ? 0u : (uint32_t)lo;
    r.hi = hi > 0x80000000ll ? 0x80000000u : (uint32_t)hi;
    r.prev_tau = r.tau;
    r.have_prev = 1;
    r.was_cold = 0;
}

// grid = rows.  Orders the collected ties by index, sets the cut-off, clears the list state and
// predicts the next step's band.  Rows whose band failed twice, or with more ties than the buffer
// holds, go to the slow search.
__global__ __launch_bounds__(kBlock) void k_list_finish(uint32_t row0, RowDesc* __restrict__ desc,
                                                         uint32_t* __restrict__ lhist,
                                                         const uint32_t* __restrict__ tiebuf, uint32_t cap, uint32_t k,
                                                         uint32_t fix_lo, uint32_t fix_hi) {
    __shared__ uint32_t t_idx[kTieCap];
    __shared__ uint32_t s_cut;
    const uint32_t row = row0 + blockIdx.x;
    if (desc[row].mode == kSlow) return;
    if (!listable(desc[row], cap, k)) {                        // uniform for the block
        if (threadIdx.x == 0) {
            RowDesc r = desc[row];
            r.n_cand = 0;
            clear_sure(r);
            r.n_ties = 0;
            r.n_list = 0;
            r.mode = kSlow;
            desc[row] = r;
        }
        return;
    }
    uint32_t* __restrict__ hrow = lhist + (size_t)row * 2 * kListBins;
    for (int b = threadIdx.x; b < 2 * kListBins; b += kBlock) hrow[b] = 0;
    const uint32_t ties = desc[row].ties, want = desc[row].rank;
    const bool fits = ties <= (uint32_t)kTieCap;
    if (fits) {
        const uint32_t* __restrict__ tb = tiebuf + (size_t)row * kTieCap;
        for (uint32_t q = threadIdx.x; q < ties; q += kBlock) t_idx[q] = tb[q];
        if (threadIdx.x == 0) s_cut = 0xffffffffu;
        __syncthreads();
        for (uint32_t q = threadIdx.x; q < ties; q += kBlock) {
            const uint32_t mine = t_idx[q];
            uint32_t below = 0;
            for (uint32_t r = 0; r < ties; ++r) below += t_idx[r] < mine;
            if (below + 1 == want) s_cut = mine;            // indices are distinct: one writer
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        RowDesc r = desc[row];
        r.n_list = r.n_cand;
        r.n_cand = 0;
        clear_sure(r);
        r.n_ties = 0;
        if (fits) {
            r.cutoff = s_cut;
            r.dense = 0;
            r.nonfinite = r.nonfinite_acc;
            r.nonfinite_acc = 0;
            predict_band(r, fix_lo, fix_hi);
            r.mode = kWarm;
        } else {
            r.mode = kSlow;
        }
        desc[row] = r;
    }
}

// General search for rows in kSlow mode, one block of 1024 threads per row: three radix digits
// over the whole row, then the ties in index order.  Slow by design; only degenerate rows (a
// threshold shared by thousands of entries) come here.  grid = rows.
template <bool VEC, bool RK>
__global__ __launch_bounds__(1024) void k_slow_select(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                       uint32_t row0, RowDesc* __restrict__ desc, uint32_t k,
                                                       RkDraw rk) {
    __shared__ uint32_t h[kHistBins];
    __shared__ uint32_t part[256], res[3];
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t s_cut, s_bad;
    const uint32_t row = row0 + blockIdx.x;
    if (desc[row].mode != kSlow) return;
    const float* __restrict__ g = src + (size_t)blockIdx.x * row_stride;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t k0 = 0, k1 = 0;
    if (RK) {
        const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
        k0 = (uint32_t)stream;
        k1 = (uint32_t)(stream >> 32);
    }
    // the 4 keys of columns j .. j + 3 (columns at or beyond d give unspecified keys; callers test j + q < d)
    auto keys_at = [&](uint32_t j, uint32_t (&key)[4]) {
        if (RK) {
#pragma unroll
            for (int q = 0; q < 4; ++q) key[q] = rk_priority(k0, k1, j + q);
        } else {
            const float4 a = ld4<VEC>(g, j, d);
            key[0] = key_of(a.x);
            key[1] = key_of(a.y);
            key[2] = key_of(a.z);
            key[3] = key_of(a.w);
        }
    };
    uint32_t prefix = 0, rank = k, ties = 0;
    if (tid == 0) s_bad = 0;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = digit_shift(pass), nbins = 1 << digit_bits(pass);
        const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);
        for (int b = tid; b < nbins; b += 1024) h[b] = 0;
        __syncthreads();
        for (uint32_t j = tid * 4; j < d; j += 4096) {
            uint32_t key[4];
            keys_at(j, key);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + q < d && ((key[q] ^ prefix) >> hi_shift) == 0) atomicAdd(&h[(key[q] >> shift) & (nbins - 1)], 1u);
        }
        __syncthreads();
        if (pass == 0 && !RK) {                       // keys >= 0x7f800000 (Inf/NaN) sit in the bins from 0xff0 up
            bool bad = false;
            for (int b = 0xff0 + (int)tid; b < kHistBins; b += 1024) bad |= h[b] != 0;
            if (bad) s_bad = 1;
        }
        const Pick p = block_pick(h, nbins, rank, part, res);
        prefix |= p.bin << shift;
        rank = p.rank_in;
        ties = p.count;
    }
    // the rank-th entry with key == prefix, in index order
    if (tid == 0) s_cut = 0xffffffffu;
    __syncthreads();
    uint32_t seen = 0;
    for (uint32_t base = 0; base < d; base += 4096) {          // uniform trip count and exit
        const uint32_t j = base + tid * 4;
        uint32_t key[4];
        keys_at(j, key);
        const bool m0 = j < d && key[0] == prefix, m1 = j + 1 < d && key[1] == prefix;
        const bool m2 = j + 2 < d && key[2] == prefix, m3 = j + 3 < d && key[3] == prefix;
        const uint32_t mine = m0 + m1 + m2 + m3;
        uint32_t incl = mine;                                   // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += up;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        uint32_t before = seen, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < (int)wave) before += wtot[w];
            total += wtot[w];
        }
        before += incl - mine;
        if (before < rank && rank <= before + mine) {
            uint32_t need = rank - before, idx = j + 3;
            if (m0 && --need == 0) idx = j;
            else if (m1 && --need == 0) idx = j + 1;
            else if (m2 && --need == 0) idx = j + 2;
            s_cut = idx;
        }
        seen += total;
        __syncthreads();
        if (seen >= rank) break;
    }
    __syncthreads();
    if (tid == 0) {
        RowDesc r = desc[row];
        r.tau = prefix;
        r.rank = rank;
        r.ties = ties;
        r.cutoff = s_cut;
        r.dense = 1;
        r.nonfinite = s_bad | r.nonfinite_acc;
        r.nonfinite_acc = 0;
        r.n_cand = 0;
        clear_sure(r);
        r.n_ties = 0;
        r.n_list = 0;
        r.have_prev = 0;
        r.was_cold = 0;
        r.mode = kCold;
        if (RK) {                              // the band of a random-k draw is known without a prediction
            r.lo = rk.fix_lo;
            r.hi = rk.fix_hi;
            r.mode = kWarm;
        }
        desc[row] = r;
    }
}

// Random-k: completes the kept bitmap of each row once (tau, cut-off) are known.  k_filter has set the
// bits of the columns whose key is above the band; here the listed candidates that are kept get
// theirs (atomic OR on the 32-bit word holding the lane's half-word).  Rows that went through the
// slow search have no valid list: every block recomputes the priorities of its tiles and writes
// whole half-words.  grid = (blocks, rows).
__global__ __launch_bounds__(kBlock) void k_rk_mark(uint32_t d, uint32_t nwt, uint32_t row0, const RowDesc* __restrict__ desc,
                                                     const uint2* __restrict__ list, uint32_t cap,
                                                     uint16_t* __restrict__ kbits, RkDraw rk) {
    const uint32_t row = row0 + blockIdx.y;
    const uint32_t tau = desc[row].tau, cut = desc[row].cutoff;
    if (!desc[row].dense) {
        const uint32_t n = desc[row].n_list;
        const uint2* __restrict__ in = list + (size_t)row * cap;
        uint32_t* __restrict__ words = reinterpret_cast<uint32_t*>(kbits + (size_t)row * nwt * 64);
        for (uint32_t e = blockIdx.x * kBlock + threadIdx.x; e < n; e += gridDim.x * kBlock) {
            const uint2 kv = in[e];
            if (kv.x > tau || (kv.x == tau && kv.y <= cut)) {
                const uint32_t t = kv.y / kWaveTile, o = kv.y % kWaveTile;
                const uint32_t u = o / kChunk, l = (o % kChunk) / 4, q = o % 4;
                const uint32_t half = t * 64 + l;                     // half-word of the row holding the column
                atomicOr(&words[half >> 1], 1u << ((half & 1) * 16 + 4 * u + q));
            }
        }
        return;
    }
    const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
    const uint32_t k0 = (uint32_t)stream, k1 = (uint32_t)(stream >> 32);
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (uint32_t t = blockIdx.x * 4 + wave; t < nwt; t += gridDim.x * 4) {
        uint32_t m = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t j = t * kWaveTile + u * kChunk + lane * 4 + q;
                const uint32_t key = rk_priority(k0, k1, j);
                m |= ((j < d && (key > tau || (key == tau && j <= cut))) ? 1u : 0u) << (4 * u + q);
            }
        kbits[((size_t)row * nwt + t) * 64 + lane] = (uint16_t)m;
    }
}

// One thread, after the last kernel of a step that used the draw.
__global__ void k_rk_advance(RkState* __restrict__ state) { state->draw += 1; }

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
//   WC == kTopk     reads each row's group bitmap and fetches only the flagged groups of 4
//                   gradients, testing them against (tau, cut-off); per-lane sums live in LDS;
//   WC == kRandk    reads each row's kept bitmap and fetches only the groups of 4 gradients that hold a
//                   kept column;
//   WC == kIdentity reads the gradients.
// ---------------------------------------------------------------------------------------------
template <int WC, bool SRV_L1, bool VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate(const float* __restrict__ grads, const uint16_t* __restrict__ bits,
                                                       const uint64_t* __restrict__ gbits,
                                                       int N, uint32_t d, uint32_t nwt, float inv_n,
                                                       const RowDesc* __restrict__ desc, const float* __restrict__ e_in,
                                                       float* __restrict__ v_out, double* __restrict__ srv_partial,
                                                       BlockTable bt) {
    __shared__ double lds_w[4];
    __shared__ float accs[(WC == kTopk || WC == kRandk) ? 16 * kBlock : 1];
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
        } else if (WC == kTopk) {
            float* my = accs + threadIdx.x;                    // slot b of this lane: my[b * kBlock]
#pragma unroll
            for (int b = 0; b < 16; ++b) my[b * kBlock] = 0.f;
            const uint64_t* __restrict__ gw = gbits + (size_t)t * 4;   // the tile's 4 group words of row 0
            const size_t grow = (size_t)nwt * 4;
            for (int i = 0; i < N; ++i) {
                const float* __restrict__ gi = grads + (size_t)i * d;
                const uint32_t tau = desc[i].tau, cut = desc[i].cutoff;
                uint32_t mask = 0xfu;                          // bit u: this lane's group of chunk u is flagged
                if (!desc[i].dense) {
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
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = j0 + u * kChunk;
            const float4 e = ld4<VEC>(e_in, j, d);
            float4 v;
            v.x = __fmaf_rn(acc[u].x, inv_n, e.x);
            v.y = __fmaf_rn(acc[u].y, inv_n, e.y);
            v.z = __fmaf_rn(acc[u].z, inv_n, e.z);
            v.w = __fmaf_rn(acc[u].w, inv_n, e.w);
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
                                                    const uint16_t* __restrict__ kbits) {
    const uint32_t per_panel = panel * (uint32_t)N;
    const uint32_t pn = blockIdx.x / per_panel, r = blockIdx.x % per_panel;
    const uint32_t i = r / panel, tile = pn * panel + r % panel;
    if (tile >= ncol_tiles) return;
    const uint32_t j = tile * kColTile + threadIdx.x * 4;
    if (j >= d) return;
    const float* __restrict__ gi = grads + (size_t)i * d;
    float* __restrict__ xi = x + (size_t)i * d;
    uint32_t tb = 0;
    if (WC == kBlockSign || SC == kBlockSign) tb = bt.tile_blk[tile];   // issued ahead of the streams
    // random-k: the 4 kept bits of this thread's columns (the thread is lane `threadIdx.x & 63` of chunk
    // `threadIdx.x >> 6` of wave tile `tile`); row N of the bitmap is the server's draw
    uint32_t wkeep = 0, skeep = 0;
    if (WC == kRandk)
        wkeep = (kbits[((size_t)i * ncol_tiles + tile) * 64 + (threadIdx.x & 63)] >> (4 * (threadIdx.x >> 6))) & 0xfu;
    if (SC == kRandk)
        skeep = (kbits[((size_t)N * ncol_tiles + tile) * 64 + (threadIdx.x & 63)] >> (4 * (threadIdx.x >> 6))) & 0xfu;
    const float4 g = ld4<VEC, true>(gi, j, d);
#if defined(__HIP_DEVICE_COMPILE__)
    // One stream at a time per wave: waiting for the gradients before asking for the model measured
    // 2-4 % faster than having both 128-bit loads in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    const float4 xv = ld4<VEC, true>(xi, j, d);
    const float4 v = ld4<VEC>(v_in, j, d);
    const RowDesc* __restrict__ sd = desc + N;
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
    p.x = message_of<SC>(v.x, j, ss[0], stau, scut, skeep & 1u);
    p.y = message_of<SC>(v.y, j + 1, ss[1], stau, scut, skeep & 2u);
    p.z = message_of<SC>(v.z, j + 2, ss[2], stau, scut, skeep & 4u);
    p.w = message_of<SC>(v.w, j + 3, ss[3], stau, scut, skeep & 8u);
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

// ---------------------------------------------------------------------------------------------
// Wire form of a (blockwise) scaled-sign message: one bit per element, bit j % 8 of byte j / 8 set
// when the element is negative.  k_pack_sign turns one row of the lane-major bitmap into that
// form (one thread per output byte); k_unpack_sign expands wire bits and scale(s) into the dense
// message p_j = -s or +s (one thread per column).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_pack_sign(const uint16_t* __restrict__ row_bits, uint32_t nbytes,
                                                       uint8_t* __restrict__ out) {
    const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= nbytes) return;
    const uint32_t col = b * 8, t = col / kWaveTile, o = col % kWaveTile, u = o / kChunk, lane = (o % kChunk) / 4;
    const uint32_t m0 = row_bits[(size_t)t * 64 + lane], m1 = row_bits[(size_t)t * 64 + lane + 1];
    out[b] = (uint8_t)(((m0 >> (4 * u)) & 0xfu) | (((m1 >> (4 * u)) & 0xfu) << 4));
}

__global__ __launch_bounds__(kBlock) void k_unpack_sign(const uint8_t* __restrict__ bytes, uint32_t d,
                                                         const float* __restrict__ scales, BlockTable bt,
                                                         float* __restrict__ p) {
    const uint32_t j = blockIdx.x * kBlock + threadIdx.x;
    if (j >= d) return;
    float s = scales[0];
    if (bt.B) {
        const uint32_t tb = bt.tile_blk[j / kColTile];
        s = scales[(tb >> 31) ? block_of(bt, tb & 0x7fffffffu, j) : tb];
    }
    p[j] = ((bytes[j / 8] >> (j % 8)) & 1u) ? -s : s;
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

// One block of 1024 threads: exclusive scan of n counts in place; *total receives the sum.
__global__ __launch_bounds__(1024) void k_scan_u32(uint32_t* __restrict__ v, uint32_t n, uint32_t* __restrict__ total) {
    __shared__ uint32_t part[1024];
    const uint32_t per = (n + 1023) / 1024, lo = threadIdx.x * per, hi = min(lo + per, n);
    uint32_t sum = 0;
    for (uint32_t q = lo; q < hi; ++q) sum += v[q];
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int q = 0; q < 1024; ++q) {
            const uint32_t c = part[q];
            part[q] = run;
            run += c;
        }
        *total = run;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (uint32_t q = lo; q < hi; ++q) {
        const uint32_t c = v[q];
        v[q] = run;
        run += c;
    }
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

__global__ __launch_bounds__(kBlock) void k_sumsq_final(const double* __restrict__ partial, uint32_t nparts,
                                                         double* __restrict__ out) {
    __shared__ double lds_w[4];
    double acc = 0.0;
    for (uint32_t q = threadIdx.x; q < nparts; q += kBlock) acc += partial[q];
    const double s = block_sum_f64(acc, lds_w);
    if (threadIdx.x == 0) *out = s;
}

// Plain device copy (128 bits per thread, streaming hints), used to measure the achievable
// read+write bandwidth next to the step's kernels and to calibrate byte counters.
__global__ __launch_bounds__(kBlock) void k_copy16(const v4f* __restrict__ src, v4f* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

}  // namespace liec
