// Shared pieces of the LIEC-SGD device kernels for gfx950 (CDNA4, wave64): constants, the per-row
// descriptor, the random-k generator, 128-bit accessors, block reductions and the histogram walk.
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
constexpr int kListBits = 13;           // widest radix digit of the list select (two digits cover a band of 2^26 keys)
constexpr int kListBins = 1 << kListBits;
constexpr int kStage = 1024;            // LDS staging slots of a block of the candidate filter
constexpr int kWaveStage = 256;         // and of each of its waves once the block's are used up (a chunk lists at most 256)
constexpr int kDirectList = 16384;      // candidate lists up to this length are selected by one block on its own
constexpr int kShortCap = 4096;         // entries of the first list digit's bin that are handed to the list select on their own
constexpr int kTieCap = 4096;           // ties at the threshold the fast path resolves
constexpr uint32_t kBandStart = 1u << 17;    // swing (an eighth of the band's half width) after a step without a prediction
constexpr uint32_t kBandFloor = 1u << 15;    // least half width, in key units, of the predicted band (about 0.27 % in value)
constexpr uint32_t kUpdatePanel = 4096; // column tiles per panel of the update kernel

enum Comp : int { kIdentity = 0, kSign = 1, kTopk = 2, kBlockSign = 3, kRandk = 4 };

// How a row's top-k threshold search starts its step.  A row's mode changes only where one block speaks
// for the row (the list select, the general search); in between, every kernel re-derives what the row
// needs from the mode and the row's counters.
enum SelMode : uint32_t {
    kWarm = 0,      // a band [lo, hi) predicted from the previous step is filtered
    kCold = 1,      // no prediction: the band is the first-radix-digit bin holding rank k
    kSlow = 4       // needs the general (multi pass) search over the row
};

// One per worker row, plus one (index N) for the server's vector v.
struct alignas(128) RowDesc {
    // first 128-byte line: what the kernels read, written once a step by whoever finishes the row's search
    double l1;             // scaled sign: sum |v_j| (fp64)
    float scale;           // scaled sign: fp32(l1 / d)
    uint32_t tau;          // top-k: key of the k-th kept entry
    uint32_t rank;         // top-k: how many entries with key == tau are kept
    uint32_t ties;         // top-k: how many entries have key == tau
    uint32_t cutoff;       // top-k: largest kept index among entries with key == tau
    uint32_t nonfinite;    // a NaN/Inf reached the L1 sum or a key (last step)
    uint32_t lo, hi;       // candidate band: keys in [lo, hi) are listed, keys >= hi are surely kept
    uint32_t mode;         // SelMode
    uint32_t n_list;       // candidates that were listed when the search finished (random-k marks the kept ones)
    uint32_t dense;        // the row's candidate bitmap is not valid: test every column
    uint32_t prev_tau;     // tau of the step before (valid when have_prev)
    uint32_t have_prev;
    uint32_t misses;       // steps in which the predicted band was not usable (since the context was created)
    uint32_t centre;       // where the last prediction expected tau
    uint32_t swing;        // decaying maximum of the distances between tau and that centre
    uint32_t was_cold;     // the last band came from the first-digit histogram, not from a prediction
    // second line: what the blocks of the passes add to with atomics (kept off the line every block reads when
    // it starts).  Counters of the pass over the predicted band, one 64-bit word that a block of the filter adds
    // to with a single atomic.  Low half: candidates appended (may exceed the capacity: overflow); high half:
    // keys at or above the band.
    alignas(128) uint32_t n_cand;
    uint32_t n_sure;
    // the same for the pass over the first-digit band, which runs when there is no prediction or the predicted
    // band failed (its own set, so that every kernel can still tell from the first set that the row needed it)
    alignas(8) uint32_t n_cand2;
    uint32_t n_sure2;
    uint32_t n_short;      // entries of the first list digit's bin collected into the row's short list
    uint32_t nonfinite_acc;   // this step's Inf / NaN sightings (moved to `nonfinite` when the search finishes)
};
static_assert(sizeof(RowDesc) == 256, "two lines per row");

__host__ __device__ __forceinline__ uint32_t sure_count(const RowDesc& r) { return r.n_sure; }
__host__ __device__ __forceinline__ uint32_t sure_count2(const RowDesc& r) { return r.n_sure2; }
// Both passes' counters back to zero (whoever finishes a row's search calls it).
__host__ __device__ __forceinline__ void clear_counts(RowDesc& r) {
    r.n_cand = 0;
    r.n_cand2 = 0;
    r.n_short = 0;
    r.n_sure = r.n_sure2 = 0;
}

// After a filter pass: the band is usable when its list did not overflow and rank k falls inside it.
__device__ __forceinline__ bool band_ok(const RowDesc& r, uint32_t cap, uint32_t k) {
    const uint32_t n_sure = sure_count(r);
    return r.n_cand <= cap && n_sure < k && (uint64_t)k <= (uint64_t)n_sure + r.n_cand &&
           r.hi - r.lo <= (1u << (2 * kListBits));       // the list select's two digits must span the band
}
// Rows that need the first-digit histogram: no prediction, or the predicted band failed.  Stable from the
// end of the pass over the predicted band until the row's search is finished.
__device__ __forceinline__ bool wants_cold(const RowDesc& r, uint32_t cap, uint32_t k) {
    return r.mode == kCold || (r.mode == kWarm && !band_ok(r, cap, k));
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

// The index whose 32-bit word (priority with its dropped bit put back) is y: every step of rk_priority
// undone in reverse order (the multipliers' inverses modulo 2^32; x ^= x >> 13 is undone by two
// shifts, x ^= x >> 16 by itself).
__host__ __device__ __forceinline__ uint32_t rk_index_of(uint32_t k0, uint32_t k1, uint32_t y) {
    uint32_t h = y ^ (y >> 16);
    h *= 0x7ED1B41Du;                  // 0xC2B2AE35^-1
    h -= k1;
    h = h ^ (h >> 13) ^ (h >> 26);
    h *= 0xA5CB9243u;                  // 0x85EBCA6B^-1
    h ^= h >> 16;
    return h ^ k0;
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

// Histogram step of a whole wave (call it in wave-uniform control flow): adds one to LDS bin `bin` for every
// lane with `valid`.  When all of them name the same bin -- a degenerate row puts whole waves on one
// magnitude -- the wave issues one atomic instead of serialising 64 on one address.
__device__ __forceinline__ void wave_count(uint32_t* h, bool valid, uint32_t bin, uint32_t lane) {
    const uint32_t bin0 = __builtin_amdgcn_readfirstlane(bin);
    const uint64_t act = __ballot(valid);
    if (__ballot(valid && bin != bin0) == 0) {
        if (lane == 0 && act) atomicAdd(&h[bin0], (uint32_t)__popcll(act));
    } else if (valid) {
        atomicAdd(&h[bin], 1u);
    }
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
// Thread t < 256 adds up the nbins / 256 consecutive bins t * per .. t * per + per - 1, starting at a bin of its
// own ((q + t) mod per: neighbouring threads then read different LDS banks -- read in the same order, the 32
// bins per thread of an 8192-bin histogram all fell on one bank and the pick took 4 us); a suffix sum over the
// threads finds the one whose bins hold the rank, and one wave walks that thread's bins.
struct Pick {
    uint32_t bin, rank_in, count;
};
__device__ __forceinline__ Pick block_pick(const uint32_t* __restrict__ h, int nbins, uint32_t rank,
                                           uint32_t* part, uint32_t* res) {
    const int per = nbins >> 8;   // 1 .. 32 bins per thread, a power of two
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t sum = 0;
    if (tid < 256) {
#pragma unroll 8
        for (int q = 0; q < per; ++q) sum += h[tid * per + ((q + tid) & (per - 1))];
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
        part[8] = 0xffffffffu;                                  // the thread whose bins hold the rank: none yet
        res[0] = 0;
        res[1] = 1;
        res[2] = 0;
    }
    __syncthreads();
    if (tid < 256) {
        uint32_t above = incl - sum;
        for (uint32_t w = wave + 1; w < 4; ++w) above += part[w];
        if (above < rank && rank <= above + sum) {   // true for at most one thread
            part[8] = tid;
            part[9] = above;
        }
    }
    __syncthreads();
    const uint32_t owner = part[8];
    if (owner != 0xffffffffu && tid < 64) {                     // wave 0 walks the owner's bins from the top
        const uint32_t above = part[9];
        const uint32_t c = (int)lane < per ? h[owner * per + lane] : 0u;
        uint32_t suf = c;                                       // sum over the lanes at and above mine
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_down(suf, o, 64);
            if (lane + o < 64) suf += up;
        }
        const uint64_t reach = __ballot((int)lane < per && above + suf >= rank);    // lane 0 always does
        const uint32_t top = 63u - (uint32_t)__clzll((long long)reach);
        if (lane == top) {
            res[0] = owner * per + lane;
            res[1] = rank - (above + suf - c);
            res[2] = c;
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

}  // namespace liec
