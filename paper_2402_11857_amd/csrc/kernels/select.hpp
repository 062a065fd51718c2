// Threshold search behind top-k (Definition 2) and random-k (Definition 3).
#pragma once
#include "common.hpp"
#include <type_traits>

namespace liec {

// ---------------------------------------------------------------------------------------------
// Top-k (Definition 2).  The k-th largest magnitude key tau of a row and the index cut-off
// among its ties are found without sorting, by five kernels the host enqueues every step:
//   1. k_filter (pass over the predicted band) streams the row once against a band [lo, hi) of keys
//      expected to hold tau, predicted from the previous steps' tau (rows in kWarm mode): keys >= hi are
//      only counted, keys inside the band are appended to a candidate list (key, index), and a group
//      bitmap is written for the aggregation kernel, in one of two forms the host picks from the row
//      length.  Fine: 4 words of 64 bits per wave tile, bit l of word u set when any of the 4 columns
//      1024t + 256u + 4l .. + 3 has key >= lo.  Coarse: one word per wave tile, bit 4m + u set when any
//      of the 16 columns 1024t + 256u + 16m .. + 15 (one 64-byte line, the unit a gather fetches anyway)
//      has one -- 8 bytes written per 4 KiB read (writes are what a read stream pays most for); measured
//      faster for rows of 48M columns and more, slower for 25M.  The band is usable when the list did
//      not overflow and rank k falls inside it (band_ok).
//   2. k_hist0, for rows without a prediction (kCold) or whose predicted band was not usable: the
//      histogram of the first radix digit (12 bits) of the whole row.  For rows on their predicted band
//      with a long list it counts the first digit of the listed keys instead (list_first_digit).
//   3. k_filter (pass over the first-digit band), for the rows of the first kind: every block picks the
//      bin holding rank k from that histogram, and the row is filtered again with that bin as its band,
//      counting into a second set of counters.  For the rows of the second kind every block picks the
//      first list digit's bin and the bin's entries are collected into a short list (list_collect).
//   4. k_list_select, one block per row: radix digits over the listed keys, taken relative to the band's
//      lower end (over the short list when there is one), then the ties in index order (up to 4096 of
//      them through LDS, more by a radix select over the listed indices); writes (tau, cut-off), predicts
//      the next band.  Rows whose band the list cannot hold (constant or near-constant rows) are put
//      into kSlow mode.
//   5. k_slow_select takes the kSlow rows.
// All decisions are taken on the device per row, each kernel re-deriving from the row's mode and
// counters whether it has work; in the steady state kernels 2 and 3 only touch the lists and 5 returns at once.  A row's mode
// and its result are written only by k_list_select and k_slow_select.
// `row0` is added to blockIdx.y to address per-row state (the server's vector uses row N).
// ---------------------------------------------------------------------------------------------
// Coarse group bitmap: bit 4m of the result is set when some lane of 4m .. 4m + 3 has its bit set in the
// ballot (those four lanes own one 64-byte line of the row).  Chunk u of a wave tile shifts its result
// left by u, so bit 4m + u of the tile's word stands for line m of chunk u.
__device__ __forceinline__ uint64_t any_of_four_lanes(uint64_t b) {
    b |= b >> 1;
    b |= b >> 2;
    return b & 0x1111111111111111ull;
}

// One chunk (256 columns, 4 per lane) of the filter: updates the per-lane count of keys >= hi and the
// running maximum key, returns the ballot of "any of my 4 columns has key >= lo" and, per component q,
// the ballot bc[q] of the candidates lo <= key < hi.  The comparisons stay wave ballots (scalar
// registers) and are combined there, which leaves the vector unit two compares, one add and half a
// maximum per key.  FULL: every column of the chunk is below d.  BITS: also hi4, bit q set when my
// column q has key >= hi.
template <bool FULL, bool BITS>
__device__ __forceinline__ uint64_t filter_chunk(const uint32_t (&keys)[4], uint32_t j, uint32_t d, uint32_t lo, uint32_t hi,
                                                 uint64_t (&bc)[4], uint32_t& n_hi, uint32_t& kmax, uint32_t& hi4) {
    uint64_t any_lo = 0;
    hi4 = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t key = keys[q];
        const bool valid = FULL || j + q < d;
        const bool ge_lo = valid && key >= lo, ge_hi = valid && key >= hi;
        kmax = max(kmax, valid ? key : 0u);
        n_hi += ge_hi ? 1u : 0u;
        if (BITS) hi4 |= (ge_hi ? 1u : 0u) << q;
        const uint64_t b_lo = __ballot(ge_lo);
        bc[q] = b_lo & ~__ballot(ge_hi);
        any_lo |= b_lo;
    }
    return any_lo;
}

// List select: the keys of a band are taken relative to its lower end and need b <= 26 bits.  The first
// digit is their top kFirstBits bits when many blocks build its histogram in global memory (256 bins: the
// blocks' LDS histograms then merge with few global atomics, which are slow across the chip's dies), or up
// to kListBits bits when one block builds it in LDS; the following digits take up to kListBits bits each.
constexpr int kFirstBits = 8;
__device__ __forceinline__ int band_bits(uint32_t width) {            // width: 1 .. 2^26
    return width > 1 ? 32 - __clz((int)(width - 1)) : 1;
}
__device__ __forceinline__ int first_shift(uint32_t width, int first_bits) {   // bits below the first digit
    const int b = band_bits(width);
    return b > first_bits ? b - first_bits : 0;
}

// Blocks that share a pass over a list of n entries: one per 2048 entries.
__device__ __forceinline__ uint32_t list_blocks_for(uint32_t n, uint32_t grid) {
    const uint32_t want = (n + 2047u) / 2048u;
    return want < 1u ? 1u : (want > grid ? grid : want);
}

// The two passes over a row's candidate list that are shared by many blocks.  They ride in the two kernels
// that otherwise only work for rows without a usable prediction (k_hist0 and the second k_filter pass), for the
// rows whose predicted band holds rank k:
//   list_first_digit  adds the first digit of every listed key to the row's global histogram;
//   list_collect      picks the bin holding rank k from that histogram (every block redoes the pick) and, when
//                     that bin has at most kShortCap entries, appends them to the row's short list.
// k_list_select then finishes on the short list alone.  Lists of at most kDirectList entries skip both: one block
// walks those as fast as the shared passes' fixed costs.  Every thread of the block calls them.
__device__ __forceinline__ void list_first_digit(const RowDesc* __restrict__ desc, uint32_t row,
                                                 const uint2* __restrict__ in, uint32_t* __restrict__ hrow,
                                                 uint32_t* lds_h /* 256 words */) {
    const uint32_t n = desc[row].n_cand, nb = list_blocks_for(n, gridDim.x);
    if (n <= (uint32_t)kDirectList || blockIdx.x >= nb) return;
    const uint32_t lo = desc[row].lo, lane = threadIdx.x & 63;
    const int shift = first_shift(desc[row].hi - lo, kFirstBits);
    for (uint32_t b = threadIdx.x; b < 256; b += blockDim.x) lds_h[b] = 0;
    __syncthreads();
    for (uint32_t base = blockIdx.x * blockDim.x; base < n; base += nb * blockDim.x) {    // uniform for the block
        const uint32_t e = base + threadIdx.x;
        const bool valid = e < n;
        const uint32_t key = valid ? in[e].x : lo;
        wave_count(lds_h, valid, (key - lo) >> shift, lane);
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < 256; b += blockDim.x) {
        const uint32_t c = lds_h[b];
        if (c) atomicAdd(&hrow[b], c);
    }
}

__device__ __forceinline__ void list_collect(RowDesc* __restrict__ desc, uint32_t row, const uint2* __restrict__ in,
                                             const uint32_t* __restrict__ hrow, uint2* __restrict__ out, uint32_t k,
                                             uint32_t* part, uint32_t* res) {
    const uint32_t n = desc[row].n_cand, nb = list_blocks_for(n, gridDim.x);
    if (n <= (uint32_t)kDirectList || blockIdx.x >= nb) return;
    const uint32_t lo = desc[row].lo, lane = threadIdx.x & 63;
    const int shift = first_shift(desc[row].hi - lo, kFirstBits);
    const Pick p = block_pick(hrow, 1 << kFirstBits, k - sure_count(desc[row]), part, res);
    if (p.count > (uint32_t)kShortCap) return;                  // too many for the short list: k_list_select walks the list
    for (uint32_t base = blockIdx.x * blockDim.x; base < n; base += nb * blockDim.x) {    // uniform for the block
        const uint32_t e = base + threadIdx.x;
        const uint2 kv = e < n ? in[e] : make_uint2(0u, 0u);
        const bool hit = e < n && ((kv.x - lo) >> shift) == p.bin;
        const uint64_t m = __ballot(hit);
        if (m) {                                                // wave-uniform
            uint32_t at = 0;
            if (lane == 0) at = atomicAdd(&desc[row].n_short, (uint32_t)__popcll(m));
            at = __builtin_amdgcn_readfirstlane(at);
            if (hit) out[at + lanes_below(m)] = kv;             // the bin's count bounds the total: at most kShortCap
        }
    }
}

// The band a row is filtered against and the counters the pass adds to.  cold_pass false: rows in kWarm
// mode, their predicted band, the first counter set.  cold_pass true: rows for which wants_cold holds,
// the first-digit bin that holds rank k (every block redoes that pick from the row's finished histogram;
// needs 256 threads and 259 words of LDS), the second counter set.  False when the block has no work.
struct FilterBand {
    uint32_t lo, hi;
    uint2* out;                                  // the row's list and its capacity
    uint32_t cap;
    unsigned long long* counts;                  // the pass's counter word: candidates (low half), keys above the band (high half)
};
__device__ __forceinline__ bool filter_band(RowDesc* __restrict__ desc, uint32_t row, bool cold_pass,
                                            const uint32_t* __restrict__ ghist, uint2* __restrict__ list, uint32_t cap,
                                            uint32_t k, uint32_t* part, uint32_t* res, FilterBand& fb) {
    fb.out = list + (size_t)row * cap;
    fb.cap = cap;
    if (!cold_pass) {
        if (desc[row].mode != kWarm) return false;
        fb.lo = desc[row].lo;
        fb.hi = desc[row].hi;
        fb.counts = reinterpret_cast<unsigned long long*>(&desc[row].n_cand);
        return true;
    }
    if (!wants_cold(desc[row], cap, k)) return false;
    const Pick p = block_pick(ghist + (size_t)row * kHistBins, kHistBins, k, part, res);
    if (p.count > cap) return false;             // the list cannot hold the bin: the row takes the general search
    fb.lo = p.bin << 19;
    fb.hi = (p.bin + 1) << 19;                   // 0x80000000 for the top bin: no key reaches it
    fb.counts = reinterpret_cast<unsigned long long*>(&desc[row].n_cand2);
    return true;
}

// Where the results of a filter block go.  Atomics on a row's counters are what the pass pays most for besides
// its stores.  Measured alone on 16 rows of 138M columns: a pass that writes nothing runs at the read ceiling
// (1.29 ms); one atomic per block, and nothing else written, takes it to 1.44 ms whether 2 000 or 15 000 blocks
// do it; an atomic per wave for the list and one per block for the count gave 1.5-1.6 ms, and 3.7 ms with 2 800
// blocks a row while the counters shared a line with the fields every block reads when it starts.  So the
// block's waves append their candidates to one stage in LDS (an LDS counter hands out the positions), and when
// the block is done a single 64-bit atomic adds its keys above the band to the high half of the row's counter
// word and reserves, in the low half, the list slots of what was staged.  Once that stage (kStage entries) is
// full -- wide bands, candidates crowded into one stretch of the row -- every wave goes on into a small stage
// of its own (kWaveStage entries) that it empties into list slots reserved with an atomic of its own.
struct StagePos {
    uint32_t pos;                                // block position of the wave's first entry
    uint32_t first_spill;                        // first of its positions beyond the block's stage
    uint32_t wbase;                              // slot of that entry in the wave's own stage
    bool drop;                                   // the list is full: nothing is kept any more
};
// Empties the wave's own stage into the list.  staged[1] is set once a reservation of this block has gone past
// the list's capacity: the row's count then stays above the capacity, which is all that anyone reads from an
// overflowed list, and the block stops listing and counting candidates.
__device__ __forceinline__ void flush_wave_stage(const FilterBand& fb, const uint2* wst, uint32_t cnt, uint32_t* staged,
                                                 uint32_t lane) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    uint32_t base = 0;
    if (lane == 0) {
        base = (uint32_t)atomicAdd(fb.counts, (unsigned long long)cnt);
        if ((uint64_t)base + cnt > fb.cap) staged[1] = 1;
    }
    base = __builtin_amdgcn_readfirstlane(base);
    for (uint32_t s = lane; s < cnt; s += 64)
        if (base + s < fb.cap) fb.out[base + s] = wst[s];
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// The wave has m <= kWaveStage entries to append (wave-uniform, every lane calls).  staged[0]: the block's LDS
// counter of stage positions handed out; wst / wcnt: the wave's own stage and how many entries it holds.
__device__ __forceinline__ StagePos reserve_stage(const FilterBand& fb, uint32_t m, uint32_t* staged, const uint2* wst,
                                                  uint32_t& wcnt, uint32_t lane) {
    StagePos sp;
    sp.pos = sp.first_spill = sp.wbase = 0;
    sp.drop = *reinterpret_cast<volatile uint32_t*>(&staged[1]) != 0;   // uniform
    if (sp.drop) return sp;
    uint32_t pos = 0;
    if (lane == 0) pos = atomicAdd(&staged[0], m);              // LDS
    sp.pos = __builtin_amdgcn_readfirstlane(pos);
    sp.first_spill = max(sp.pos, (uint32_t)kStage);
    if (sp.pos + m > (uint32_t)kStage) {                        // uniform
        const uint32_t nsp = sp.pos + m - sp.first_spill;
        if (wcnt + nsp > (uint32_t)kWaveStage) {
            flush_wave_stage(fb, wst, wcnt, staged, lane);
            wcnt = 0;
        }
        sp.wbase = wcnt;
        wcnt += nsp;
    }
    return sp;
}
// Entry number `ord` of those m (any subset of lanes).
__device__ __forceinline__ void put_candidate(uint2* stage, uint2* wst, const StagePos& sp, uint32_t ord, uint2 entry) {
    if (sp.drop) return;
    const uint32_t p = sp.pos + ord;
    if (p < (uint32_t)kStage) stage[p] = entry;
    else wst[sp.wbase + (p - sp.first_spill)] = entry;
}

// End of a filter block.  n_hi: keys above the band, per lane; wst / wcnt: the wave's own stage.  Every thread of
// the block calls it.
__device__ __forceinline__ void finish_filter_block(const FilterBand& fb, const uint2* stage, const uint2* wst, uint32_t wcnt,
                                                    uint32_t n_hi, uint32_t* staged, uint32_t* wsure /* 5 words */) {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) n_hi += __shfl_down(n_hi, o, 64);
    if (lane == 0) wsure[wave] = n_hi;
    if (wcnt) flush_wave_stage(fb, wst, wcnt, staged, lane);    // wave-uniform
    __syncthreads();
    const uint32_t n_staged = min(staged[0], (uint32_t)kStage);
    if (threadIdx.x == 0) {
        const uint32_t sure = wsure[0] + wsure[1] + wsure[2] + wsure[3];
        uint32_t base = 0;
        if (sure | n_staged) base = (uint32_t)atomicAdd(fb.counts, ((unsigned long long)sure << 32) | n_staged);
        wsure[4] = base;
    }
    __syncthreads();
    const uint32_t base = wsure[4];
    for (uint32_t s = threadIdx.x; s < n_staged; s += kBlock)
        if (base + s < fb.cap) fb.out[base + s] = stage[s];
}

// RK: the keys are the priorities of a random-k draw (nothing is read from src), and instead of the
// group bitmap the kernel writes, per column, whether its key is at or above the band (lane-major
// half-words like the sign bits, at row `row` of kbits); k_rk_mark later adds the kept candidates.
template <bool VEC, bool RK>
__global__ __launch_bounds__(kBlock) void k_filter(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                    uint32_t nwt, uint32_t row0, RowDesc* __restrict__ desc,
                                                    bool cold_pass, const uint32_t* __restrict__ ghist, uint32_t k,
                                                    uint64_t* __restrict__ gbits,
                                                    uint16_t* __restrict__ kbits, uint2* __restrict__ list, uint32_t cap,
                                                    uint2* __restrict__ shortl, RkDraw rk, bool coarse, uint32_t run) {
    __shared__ uint2 stage[kStage], wstage[4][kWaveStage];
    __shared__ uint32_t wsure[5], staged[2];
    __shared__ uint32_t part[256], res[3];
    const uint32_t row = row0 + blockIdx.y;
    if (cold_pass && desc[row].mode == kWarm && !wants_cold(desc[row], cap, k)) {   // uniform for the block
        list_collect(desc, row, list + (size_t)row * cap, ghist + (size_t)row * kHistBins,
                     shortl + (size_t)row * kShortCap, k, part, res);
        return;
    }
    FilterBand fb;
    if (!filter_band(desc, row, cold_pass, ghist, list, cap, k, part, res, fb)) return;   // uniform for the block
    if (threadIdx.x < 2) staged[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t lo = fb.lo, hi = fb.hi;
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    uint32_t k0 = 0, k1 = 0;
    if (RK) {
        const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
        k0 = (uint32_t)stream;
        k1 = (uint32_t)(stream >> 32);
    }
    uint32_t n_hi = 0, kmax = 0;                                // per lane: keys >= hi seen, largest key seen
    uint2* wst = wstage[wave];                                  // the wave's own stage and its fill (wave-uniform)
    uint32_t wcnt = 0;
    // the body for one wave tile; FULL (every column of the tile is below d) drops the bounds checks
    uint64_t pend = 0;                                          // group words of the run so far: coarse, lane i holds tile i's;
                                                                // fine, lane 4i + u holds word u of tile i
    auto tile = [&](auto full_c, uint32_t t, uint32_t ti) {
        constexpr bool FULL = decltype(full_c)::value;
        float4 a[4];
        if (!RK) {
            if (VEC && FULL) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const v4f w = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(g + (size_t)t * kWaveTile + u * kChunk + lane * 4));
                    a[u] = make_float4(w.x, w.y, w.z, w.w);
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) a[u] = ld4<VEC, true>(g, t * kWaveTile + u * kChunk + lane * 4, d);
            }
        }
        uint64_t line_word = 0;                                 // the tile's one coarse group word (wave-uniform)
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
            uint64_t bc[4];
            uint32_t hi4;
            const uint64_t any_lo = filter_chunk<FULL, RK>(keys, j, d, lo, hi, bc, n_hi, kmax, hi4);
            if (!RK) {                                          // both forms, without a branch: a few scalar operations
                line_word |= any_of_four_lanes(any_lo) << u;
                if (!coarse) pend = lane == 4 * ti + (uint32_t)u ? any_lo : pend;
            }
            sure16 |= hi4 << (4 * u);
            const uint64_t any_cand = bc[0] | bc[1] | bc[2] | bc[3];
            if (any_cand) {                                     // wave-uniform
                const uint32_t m = __popcll(bc[0]) + __popcll(bc[1]) + __popcll(bc[2]) + __popcll(bc[3]);
                const StagePos sp = reserve_stage(fb, m, staged, wst, wcnt, lane);
                uint32_t off = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((bc[q] >> lane) & 1) put_candidate(stage, wst, sp, off + lanes_below(bc[q]), make_uint2(keys[q], j + q));
                    off += __popcll(bc[q]);
                }
            }
        }
        if (RK) kbits[((size_t)row * nwt + t) * 64 + lane] = (uint16_t)sure16;
        else if (coarse) pend = lane == ti ? line_word : pend;
    };
    // A wave takes `run` (at most 16) consecutive wave tiles at a time and stores their group words together
    // (a block's four waves then fill whole 128-byte lines of the coarse bitmap with run = 4; measured equal to a
    // store per tile, and to longer runs: what the bitmap costs the pass, a tenth of its time, goes with the
    // bytes written, not with the number of stores).  Short rows keep run = 1, so that enough blocks are in flight.
    for (uint32_t tb = (blockIdx.x * 4 + wave) * run; tb < nwt; tb += gridDim.x * 4 * run) {
        const uint32_t te = min(tb + run, nwt);
        for (uint32_t t = tb; t < te; ++t) {
            if ((t + 1) * (uint32_t)kWaveTile <= d) tile(std::true_type{}, t, t - tb);    // wave-uniform
            else tile(std::false_type{}, t, t - tb);
        }
        if (!RK && gbits) {
            if (coarse) {
                if (lane < te - tb) gbits[(size_t)blockIdx.y * nwt + tb + lane] = pend;
            } else if (lane < 4 * (te - tb)) {
                gbits[((size_t)blockIdx.y * nwt + tb) * 4 + lane] = pend;
            }
        }
    }
    // keys at or above 0x7f800000 are Inf / NaN (magnitude keys only: priorities use the whole range)
    if (!RK && __ballot(kmax >= 0x7f800000u) && lane == 0) atomicOr(&desc[row].nonfinite_acc, 1u);
    finish_filter_block(fb, stage, wst, wcnt, n_hi, staged, wsure);
}

// Random-k when the band is thin against the row (k * 2^32 / d well below d): instead of computing the
// priority of every column, walk the 32-bit words y whose priority y >> 1 is at or above the band's
// lower end and invert the permutation; words that land on a column below d are the row's keys >= lo.
// The work is O(k * 2^32 / d) per row instead of O(d).  Same outputs as k_filter<., true>: the count of
// keys above the band, the candidate list, and the bits of the columns above the band -- set with
// atomic ORs into a bitmap that k_rk_zero cleared.  grid = (blocks, rows).
__global__ __launch_bounds__(kBlock) void k_rk_zero(uint32_t nwt, uint32_t row0, const RowDesc* __restrict__ desc,
                                                     bool cold_pass, uint32_t cap, uint32_t k,
                                                     uint16_t* __restrict__ kbits) {
    const uint32_t row = row0 + blockIdx.y;
    if (cold_pass ? !wants_cold(desc[row], cap, k) : desc[row].mode != kWarm) return;
    uint32_t* __restrict__ words = reinterpret_cast<uint32_t*>(kbits + (size_t)row * nwt * 64);
    const uint32_t n = nwt * 32;
    for (uint32_t q = blockIdx.x * kBlock + threadIdx.x; q < n; q += gridDim.x * kBlock) words[q] = 0u;
}

__global__ __launch_bounds__(kBlock) void k_rk_filter_inverse(uint32_t d, uint32_t nwt, uint32_t row0,
                                                               RowDesc* __restrict__ desc, bool cold_pass,
                                                               const uint32_t* __restrict__ ghist, uint32_t k,
                                                               uint16_t* __restrict__ kbits, uint2* __restrict__ list,
                                                               uint32_t cap, uint2* __restrict__ shortl, RkDraw rk) {
    __shared__ uint2 stage[kStage], wstage[4][kWaveStage];
    __shared__ uint32_t wsure[5], staged[2];
    __shared__ uint32_t part[256], res[3];
    const uint32_t row = row0 + blockIdx.y;
    if (cold_pass && desc[row].mode == kWarm && !wants_cold(desc[row], cap, k)) {   // uniform for the block
        list_collect(desc, row, list + (size_t)row * cap, ghist + (size_t)row * kHistBins,
                     shortl + (size_t)row * kShortCap, k, part, res);
        return;
    }
    FilterBand fb;
    if (!filter_band(desc, row, cold_pass, ghist, list, cap, k, part, res, fb)) return;   // uniform for the block
    if (threadIdx.x < 2) staged[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t lo = fb.lo, hi = fb.hi;
    uint32_t* __restrict__ words = reinterpret_cast<uint32_t*>(kbits + (size_t)row * nwt * 64);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
    const uint32_t k0 = (uint32_t)stream, k1 = (uint32_t)(stream >> 32);
    const uint64_t y_begin = 2ull * lo, y_end = 1ull << 32;    // words whose priority is at least lo
    uint32_t n_hi = 0;
    uint2* wst = wstage[wave];
    uint32_t wcnt = 0;
    for (uint64_t base = y_begin + ((uint64_t)blockIdx.x * 4 + wave) * 64; base < y_end; base += (uint64_t)gridDim.x * kBlock) {
        const uint64_t y64 = base + lane;
        const uint32_t y = (uint32_t)y64, key = y >> 1;
        const uint32_t j = rk_index_of(k0, k1, y);
        const bool ok = y64 < y_end && j < d;
        const bool ge_hi = ok && key >= hi;
        if (ge_hi) {
            const uint32_t t = j / kWaveTile, o = j % kWaveTile;
            const uint32_t half = t * 64 + (o % kChunk) / 4;              // half-word of the row holding the column
            atomicOr(&words[half >> 1], 1u << ((half & 1) * 16 + 4 * (o / kChunk) + o % 4));
            ++n_hi;
        }
        const uint64_t bc = __ballot(ok && !ge_hi);             // candidates: lo <= key < hi
        if (bc) {                                               // wave-uniform
            const uint32_t m = __popcll(bc);
            const StagePos sp = reserve_stage(fb, m, staged, wst, wcnt, lane);
            if ((bc >> lane) & 1) put_candidate(stage, wst, sp, lanes_below(bc), make_uint2(key, j));
        }
    }
    finish_filter_block(fb, stage, wst, wcnt, n_hi, staged, wsure);
}

// First radix digit (12 bits) of every key of the rows that have no usable band; for the rows whose
// predicted band holds rank k, the first digit of the listed keys instead (list_first_digit).  Either
// histogram goes to the row's kHistBins words of `hist`.  grid = (blocks, rows).
template <bool VEC, bool RK>
__global__ __launch_bounds__(kBlock) void k_hist0(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                   uint32_t nwt, uint32_t row0, const RowDesc* __restrict__ desc,
                                                   uint32_t* __restrict__ hist, const uint2* __restrict__ list, uint32_t cap,
                                                   uint32_t k, RkDraw rk) {
    __shared__ uint32_t h[kHistBins];
    const uint32_t row = row0 + blockIdx.y;
    if (!wants_cold(desc[row], cap, k)) {                       // uniform for the block
        if (desc[row].mode == kWarm) list_first_digit(desc, row, list + (size_t)row * cap, hist + (size_t)row * kHistBins, h);
        return;
    }
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) h[b] = 0;
    __syncthreads();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
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
            for (int q = 0; q < 4; ++q) wave_count(h, j + q < d, keys[q] >> 19, lane);
        }
    }
    __syncthreads();
    uint32_t* __restrict__ out = hist + (size_t)row * kHistBins;
    for (int b = threadIdx.x; b < kHistBins; b += kBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// Band for the next step: centred on tau extrapolated by its last change.  Its half width follows how
// far the thresholds actually fell from their predicted centres: eight times `swing`, a maximum of those
// misses that decays by an eighth per step -- by a half while the last miss was under 1/512 of the band's
// half width, so that very quiet rows narrow quickly -- never less than twice the last change of tau, between
// kBandFloor and 2^25 key units.  After a step without a usable prediction the band starts 2^20 keys wide
// on either side.  A band that misses costs two more passes over the row; one that is wider than needed
// only lengthens the candidate list, hence the wide safety factor.
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
    int64_t delta = r.have_prev ? tau - (int64_t)r.prev_tau : 0;
    // a change of more than 2^22 keys (a factor of 1.4 in value) that the last prediction missed is a jump, not a
    // trend: extrapolating it would put the next band as far off again
    if (r.was_cold && (delta > ((int64_t)1 << 22) || delta < -((int64_t)1 << 22))) delta = 0;
    int64_t swing = kBandStart;
    if (r.have_prev && !r.was_cold) {
        int64_t miss = tau - (int64_t)r.centre;
        if (miss < 0) miss = -miss;
        const int64_t last = (int64_t)r.swing;
        swing = 64 * miss < last ? last / 2 : last - last / 8;
        if (swing < miss) swing = miss;
    }
    if (swing > (int64_t)1 << 22) swing = (int64_t)1 << 22;
    int64_t margin = 8 * swing;
    if (margin < 2 * (delta < 0 ? -delta : delta)) margin = 2 * (delta < 0 ? -delta : delta);
    if (margin < (int64_t)kBandFloor) margin = kBandFloor;
    if (margin > (int64_t)1 << 25) margin = (int64_t)1 << 25;   // two list digits cover a band of 2^26 keys
    int64_t centre = tau + delta;
    if (centre < 0) centre = 0;
    if (centre > 0x7fffffffll) centre = 0x7fffffffll;
    const int64_t lo = centre - margin, hi = centre + margin;
    r.lo = lo < 0 ? 0u : (uint32_t)lo;
    r.hi = hi > 0x80000000ll ? 0x80000000u : (uint32_t)hi;
    r.centre = (uint32_t)centre;
    r.swing = (uint32_t)swing;
    r.prev_tau = r.tau;
    r.have_prev = 1;
    r.was_cold = 0;
}

// One pass of the block over the n listed entries, two entries per 128-bit load and eight loads in flight
// per thread (a row's list starts 16-byte aligned): fn(entry, valid) is called in wave-uniform control
// flow (valid false beyond n), so it may use wave_count.
constexpr int kSelectBlock = 1024;
template <typename F>
__device__ __forceinline__ void for_each_listed(const uint2* __restrict__ in, uint32_t n, F fn) {
    const uint32_t tid = threadIdx.x;
    const uint4* __restrict__ in2 = reinterpret_cast<const uint4*>(in);
    const uint32_t npairs = (n + 1) / 2;                    // the slot after an odd n is inside the row's capacity
    for (uint32_t base = 0; base < npairs; base += 8 * kSelectBlock) {     // uniform trip count
        uint4 a[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t e = base + q * kSelectBlock + tid;
            a[q] = e < npairs ? in2[e] : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t e = 2 * (base + q * kSelectBlock + tid);
            fn(make_uint2(a[q].x, a[q].y), e < n);
            fn(make_uint2(a[q].z, a[q].w), e + 1 < n);
        }
    }
}

// grid = rows, 1024 threads: finishes the list select of a row.  Which band the row's list was filtered
// against -- the predicted one, or the first-digit bin picked (again, here) from the row's histogram --
// follows from the row's mode and first counter set, as in the filter passes.  Two radix digits over the
// listed keys give tau.  For a row on its predicted band the first digit's histogram is ready (k_hist0) and,
// when the bin holding rank k was small enough, so is the short list of that bin's entries (second k_filter
// pass): the rest of the select then reads those few entries only.  Otherwise the block walks the list
// itself.  The cut-off is the `rank`-th smallest index among the entries whose key is tau: through an LDS
// buffer when at most kTieCap entries share tau, else (quantised gradients: thousands of equal magnitudes)
// by a three-digit radix select over those indices.  Then the row's counters and histogram are cleared, the
// next step's band is predicted and the row is back in kWarm mode.  Rows whose list does not hold rank k
// (overflow, a bin larger than the list, rank outside the band) are put into kSlow mode.
// The same for a list of at most 16 * kSelectBlock entries that the block holds in registers (loaded once by
// hold_listed, walked by every pass of the select instead of going back to memory).
constexpr uint32_t kHeldMax = 16u * kSelectBlock;
__device__ __forceinline__ void hold_listed(const uint2* __restrict__ in, uint32_t n, uint4 (&a)[8]) {
    const uint4* __restrict__ in2 = reinterpret_cast<const uint4*>(in);
    const uint32_t npairs = (n + 1) / 2;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t e = q * kSelectBlock + threadIdx.x;
        a[q] = e < npairs ? in2[e] : make_uint4(0u, 0u, 0u, 0u);
    }
}
template <typename F>
__device__ __forceinline__ void for_each_held(const uint4 (&a)[8], uint32_t n, F fn) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        if (2u * q * kSelectBlock >= n) break;                  // uniform for the block: nothing held from here on
        const uint32_t e = 2 * (q * kSelectBlock + threadIdx.x);
        fn(make_uint2(a[q].x, a[q].y), e < n);
        fn(make_uint2(a[q].z, a[q].w), e + 1 < n);
    }
}

__global__ __launch_bounds__(kSelectBlock) void k_list_select(uint32_t row0, RowDesc* __restrict__ desc,
                                                               uint32_t* __restrict__ ghist,
                                                               const uint2* __restrict__ list, uint32_t cap,
                                                               const uint2* __restrict__ shortl, uint32_t k,
                                                               uint32_t fix_lo, uint32_t fix_hi,
                                                               uint32_t* __restrict__ slow_sync) {
    __shared__ uint32_t h[kListBins];                          // digit histograms, then the tie indices
    __shared__ uint32_t part[256], res[3];
    __shared__ uint32_t s_cut, s_nties;
    static_assert(kTieCap <= kListBins, "the tie indices reuse the histogram");
    __shared__ RowDesc now;                                    // the row's descriptor as the kernel found it
    const uint32_t row = row0 + blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    // one round trip for the whole descriptor instead of one per dependent field; nobody else writes it meanwhile
    static_assert(sizeof(RowDesc) == 64 * sizeof(uint32_t), "64 lanes copy the descriptor");
    if (tid < 64) reinterpret_cast<uint32_t*>(&now)[tid] = reinterpret_cast<const uint32_t*>(&desc[row])[tid];
    // the meeting counter and give-up flag of the general search that may follow start every step at zero
    if (slow_sync && tid < 2) slow_sync[(size_t)blockIdx.x * 2 + tid] = 0;
    __syncthreads();
    if (now.mode == kSlow) return;
    const bool cold = wants_cold(now, cap, k);                  // uniform for the block
    const uint32_t missed = (cold && now.mode == kWarm) ? 1u : 0u;    // there was a prediction and it failed
    uint32_t* __restrict__ hrow = ghist + (size_t)row * kHistBins;
    const uint2* __restrict__ in = list + (size_t)row * cap;
    uint32_t lo, hi, n, n_sure;
    bool ok = true;
    Pick ph;                                                    // first digit: bin holding rank k, rank inside it
    int shift;                                                  // key bits below the digits found so far
    bool direct = cold;                                         // this block builds the first digit's histogram itself
    if (cold) {
        const Pick p = block_pick(hrow, kHistBins, k, part, res);
        lo = p.bin << 19;
        hi = (p.bin + 1) << 19;
        n = now.n_cand2;
        n_sure = sure_count2(now);
        ok = p.count <= cap && n <= cap && n_sure < k && (uint64_t)k <= (uint64_t)n_sure + n;
        shift = first_shift(hi - lo, kListBits);
    } else {                                                    // kWarm and band_ok
        lo = now.lo;
        hi = now.hi;
        n = now.n_cand;
        n_sure = sure_count(now);
        direct = n <= (uint32_t)kDirectList;
        shift = first_shift(hi - lo, direct ? kListBits : kFirstBits);
        if (!direct) ph = block_pick(hrow, 1 << kFirstBits, k - n_sure, part, res);
    }
    if (cold || !direct)
        for (int b = tid; b < kHistBins; b += kSelectBlock) hrow[b] = 0;    // the row's histogram is ready for the next step
    if (!ok) {
        if (tid == 0) {
            RowDesc r = now;
            clear_counts(r);
            r.n_list = 0;
            r.misses += missed;
            r.mode = kSlow;
            desc[row] = r;
        }
        return;
    }
    const uint32_t n_all = n;
    if (!direct && ph.count <= (uint32_t)kShortCap && now.n_short == ph.count) {
        in = shortl + (size_t)row * kShortCap;                  // the bin's entries, collected by the second filter pass
        n = ph.count;
    }
    // a list of up to kHeldMax entries is read once and kept in registers for all the passes below
    const bool held = n <= kHeldMax;                            // uniform for the block
    uint4 own[8];
    if (held) hold_listed(in, n, own);
    auto walk = [&](auto fn) {
        if (held) for_each_held(own, n, fn);
        else for_each_listed(in, n, fn);
    };
    if (direct) {
        // first digit of every listed key, in LDS
        const uint32_t nbins = max(256u, 1u << (band_bits(hi - lo) - shift));
        for (uint32_t b = tid; b < nbins; b += kSelectBlock) h[b] = 0;
        __syncthreads();
        walk([&](uint2 kv, bool valid) { wave_count(h, valid, (kv.x - lo) >> shift, lane); });
        __syncthreads();
        ph = block_pick(h, (int)nbins, k - n_sure, part, res);
    }
    // the following digits, over the entries that carry the digits found so far
    uint32_t prefix = ph.bin, want = ph.rank_in, ties = ph.count;
#pragma unroll 1
    while (shift > 0) {
        const int bits = shift < kListBits ? shift : kListBits, below = shift - bits;
        const uint32_t nbins = max(256u, 1u << bits), mask = (1u << bits) - 1u;
        for (uint32_t b = tid; b < nbins; b += kSelectBlock) h[b] = 0;
        __syncthreads();
        walk([&](uint2 kv, bool valid) {
            const uint32_t rel = kv.x - lo;
            wave_count(h, valid && (rel >> shift) == prefix, (rel >> below) & mask, lane);
        });
        __syncthreads();
        const Pick p = block_pick(h, (int)nbins, want, part, res);
        prefix = (prefix << bits) | p.bin;
        want = p.rank_in;
        ties = p.count;
        shift = below;
    }
    const uint32_t tau = lo + prefix;
    if (ties <= (uint32_t)kTieCap) {
        if (tid == 0) {
            s_nties = 0;
            s_cut = 0xffffffffu;
        }
        __syncthreads();
        walk([&](uint2 kv, bool valid) {
            if (valid && kv.x == tau) {
                const uint32_t pos = atomicAdd(&s_nties, 1u);
                if (pos < (uint32_t)kTieCap) h[pos] = kv.y;
            }
        });
        __syncthreads();
        for (uint32_t q = tid; q < ties; q += kSelectBlock) {
            const uint32_t mine = h[q];
            uint32_t below = 0;
            for (uint32_t r = 0; r < ties; ++r) below += h[r] < mine;
            if (below + 1 == want) s_cut = mine;                // indices are distinct: one writer
        }
        __syncthreads();
    } else {
        // Indices are below 2^31; taking 0x7fffffff - index as the key turns "want-th smallest index" into
        // "want-th largest key", which is what block_pick finds.  Digits of 11, 10 and 10 bits.
        uint32_t prefix = 0, rank = want;
#pragma unroll 1
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const int above = pass == 0 ? 31 : (pass == 1 ? 20 : 10);   // bits above this digit are the prefix
            const int nbins = pass == 0 ? 2048 : 1024;
            for (int b = tid; b < nbins; b += kSelectBlock) h[b] = 0;
            __syncthreads();
            walk([&](uint2 kv, bool valid) {
                const uint32_t inv = 0x7fffffffu - kv.y;
                wave_count(h, valid && kv.x == tau && (inv >> above) == prefix, (inv >> shift) & (uint32_t)(nbins - 1), lane);
            });
            __syncthreads();
            const Pick p = block_pick(h, nbins, rank, part, res);
            prefix = (prefix << (pass == 0 ? 11 : 10)) | p.bin;
            rank = p.rank_in;
        }
        if (tid == 0) s_cut = 0x7fffffffu - prefix;
        __syncthreads();
    }
    if (tid == 0) {
        RowDesc r = now;
        r.n_list = n_all;
        clear_counts(r);
        r.tau = tau;
        r.rank = want;
        r.ties = ties;
        r.cutoff = s_cut;
        r.dense = 0;
        r.nonfinite = r.nonfinite_acc;
        r.nonfinite_acc = 0;
        r.was_cold = cold ? 1u : 0u;
        r.misses += missed;
        predict_band(r, fix_lo, fix_hi);
        r.mode = kWarm;
        desc[row] = r;
    }
}

// ---------------------------------------------------------------------------------------------
// General search for rows in kSlow mode: three radix digits over the whole row, then the ties in
// index order.  Only degenerate rows come here (constant or mostly-zero rows, values on a handful of
// levels: a threshold shared by more entries than the candidate list holds).
//   grid = (B, rows), 1024 threads.  With B > 1 the B blocks of a row split it into contiguous ranges
// and meet between the phases at a counter in the row's descriptor (every block adds one and polls
// until all B have arrived); the histograms of the three digits and the blocks' tie counts live in
// global memory.  The poll is bounded: when a wait runs out (blocks that could not all be resident
// at once, a GPU shared with other work) the row is flagged, every block leaves, and block 0
// repeats the search on its own with LDS histograms -- the B = 1 path.  Results are identical.
// Block 0 is the only writer of the row's result on either path, so a row cannot leave the kernel
// still in kSlow mode whatever the order in which waits run out.
// The host chooses B so that B * rows blocks fit the chip at one block per compute unit.
// ---------------------------------------------------------------------------------------------
constexpr int kSlowMaxBlocks = 64;
constexpr uint32_t kSlowHistWords = 4096 + 1024 + 512;        // the three digit histograms of a row

struct SlowLds {
    uint32_t h[kHistBins];
    uint32_t part[256], res[3];
    uint32_t wtot[16];
    uint32_t cut, bad, ok;
};

// the 4 keys of columns j .. j + 3 (columns at or beyond d give unspecified keys; callers test j + q < d)
template <bool VEC, bool RK>
__device__ __forceinline__ void slow_keys_at(const float* __restrict__ g, uint32_t d, uint32_t k0, uint32_t k1, uint32_t j,
                                             uint32_t (&key)[4]) {
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
}

// What either path leaves in the row's descriptor (one thread calls it).
__device__ __forceinline__ void slow_write_result(RowDesc* __restrict__ desc, uint32_t row, uint32_t tau, uint32_t rank,
                                                  uint32_t ties, uint32_t cut, uint32_t bad, bool is_rk, RkDraw rk) {
    RowDesc r = desc[row];
    r.tau = tau;
    r.rank = rank;
    r.ties = ties;
    r.cutoff = cut;
    r.dense = 1;
    r.nonfinite = bad | r.nonfinite_acc;
    r.nonfinite_acc = 0;
    clear_counts(r);
    r.n_list = 0;
    r.have_prev = 0;
    r.was_cold = 0;
    r.mode = kCold;
    if (is_rk) {                               // the band of a random-k draw is known without a prediction
        r.lo = rk.fix_lo;
        r.hi = rk.fix_hi;
        r.mode = kWarm;
    }
    desc[row] = r;
}

// One block on its own, histograms in LDS.
template <bool VEC, bool RK>
__device__ void slow_single(SlowLds& s, const float* __restrict__ g, uint32_t d, uint32_t row, RowDesc* __restrict__ desc,
                            uint32_t k, RkDraw rk, uint32_t k0, uint32_t k1) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t prefix = 0, rank = k, ties = 0;
    if (tid == 0) s.bad = 0;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = digit_shift(pass), nbins = 1 << digit_bits(pass);
        const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);
        for (int b = tid; b < nbins; b += 1024) s.h[b] = 0;
        __syncthreads();
        for (uint32_t j = tid * 4; j < d; j += 4096) {
            uint32_t key[4];
            slow_keys_at<VEC, RK>(g, d, k0, k1, j, key);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (j + q < d && ((key[q] ^ prefix) >> hi_shift) == 0) atomicAdd(&s.h[(key[q] >> shift) & (nbins - 1)], 1u);
        }
        __syncthreads();
        if (pass == 0 && !RK) {                       // keys >= 0x7f800000 (Inf/NaN) sit in the bins from 0xff0 up
            bool bad = false;
            for (int b = 0xff0 + (int)tid; b < kHistBins; b += 1024) bad |= s.h[b] != 0;
            if (bad) s.bad = 1;
        }
        const Pick p = block_pick(s.h, nbins, rank, s.part, s.res);
        prefix |= p.bin << shift;
        rank = p.rank_in;
        ties = p.count;
    }
    // the rank-th entry with key == prefix, in index order
    if (tid == 0) s.cut = 0xffffffffu;
    __syncthreads();
    uint32_t seen = 0;
    for (uint32_t base = 0; base < d; base += 4096) {          // uniform trip count and exit
        const uint32_t j = base + tid * 4;
        uint32_t key[4];
        slow_keys_at<VEC, RK>(g, d, k0, k1, j, key);
        const bool m0 = j < d && key[0] == prefix, m1 = j + 1 < d && key[1] == prefix;
        const bool m2 = j + 2 < d && key[2] == prefix, m3 = j + 3 < d && key[3] == prefix;
        const uint32_t mine = m0 + m1 + m2 + m3;
        uint32_t incl = mine;                                   // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, 64);
            if ((int)lane >= o) incl += up;
        }
        if (lane == 63) s.wtot[wave] = incl;
        __syncthreads();
        uint32_t before = seen, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < (int)wave) before += s.wtot[w];
            total += s.wtot[w];
        }
        before += incl - mine;
        if (before < rank && rank <= before + mine) {
            uint32_t need = rank - before, idx = j + 3;
            if (m0 && --need == 0) idx = j;
            else if (m1 && --need == 0) idx = j + 1;
            else if (m2 && --need == 0) idx = j + 2;
            s.cut = idx;
        }
        seen += total;
        __syncthreads();
        if (seen >= rank) break;
    }
    __syncthreads();
    if (tid == 0) slow_write_result(desc, row, prefix, rank, ties, s.cut, s.bad, RK, rk);
}

// Meeting point of the B blocks of a row: true when all have arrived `target / B` times, false when the
// wait ran out or another block has given up (the row is then flagged).  Every thread calls it.
__device__ __forceinline__ bool slow_meet(SlowLds& s, uint32_t* __restrict__ sync, uint32_t target, uint32_t spin_limit) {
    __threadfence();                           // my stores and atomics are out before my block arrives
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicAdd(&sync[0], 1u);                // sync[0]: arrivals, sync[1]: some block has given up
        uint32_t ok = 0;
        for (uint32_t spin = 0; spin < spin_limit; ++spin) {
            if (__hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
            if (__hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
                ok = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(16);
        }
        if (!ok) atomicExch(&sync[1], 1u);
        s.ok = ok;
    }
    __syncthreads();
    __threadfence();                           // what the other blocks wrote before arriving is visible from here on
    return s.ok != 0;
}

// Arrival without a wait: my stores are out, then the counter says so.  Every thread calls it.
__device__ __forceinline__ void slow_arrive(uint32_t* __restrict__ sync) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(&sync[0], 1u);
}

// The B blocks of a row together.  Only block 0 ever writes the row's descriptor, and only its return
// value matters: false when one of its waits ran out (the descriptor is untouched then, and the caller
// repeats the search on block 0 alone), true when it has written the result.  A block other than 0 whose
// wait runs out just leaves (block 0 then fails its next wait, because the give-up flag is set or the
// arrivals never add up).
template <bool VEC, bool RK>
__device__ bool slow_multi(SlowLds& s, const float* __restrict__ g, uint32_t d, uint32_t nwt, uint32_t row,
                           RowDesc* __restrict__ desc, uint32_t k, RkDraw rk, uint32_t k0, uint32_t k1,
                           uint32_t* __restrict__ ghist, uint32_t* __restrict__ gcnt, uint32_t* __restrict__ sync,
                           uint32_t spin_limit) {
    const uint32_t B = gridDim.x, b = blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t tpb = (nwt + B - 1) / B;                     // wave tiles per block: a contiguous range of the row
    const uint32_t t0 = min(b * tpb, nwt), t1 = min(t0 + tpb, nwt);
    uint32_t meetings = 0;
    // whatever an earlier, abandoned search left in the global histograms goes first
    for (uint32_t q = b * 1024 + tid; q < kSlowHistWords; q += B * 1024) ghist[q] = 0;
    if (tid == 0) s.bad = 0;
    if (!slow_meet(s, sync, B * ++meetings, spin_limit)) return false;
    uint32_t prefix = 0, rank = k, ties = 0, off = 0;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = digit_shift(pass), nbins = 1 << digit_bits(pass);
        const int hi_shift = pass == 0 ? 31 : digit_shift(pass - 1);
        for (int q = tid; q < nbins; q += 1024) s.h[q] = 0;
        __syncthreads();
        for (uint32_t t = t0 + wave; t < t1; t += 16) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
                uint32_t key[4];
                slow_keys_at<VEC, RK>(g, d, k0, k1, j, key);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool valid = j + q < d && ((key[q] ^ prefix) >> hi_shift) == 0;
                    const uint32_t bin = (key[q] >> shift) & (uint32_t)(nbins - 1);
                    wave_count(s.h, valid, bin, lane);
                }
            }
        }
        __syncthreads();
        for (int q = tid; q < nbins; q += 1024) {
            const uint32_t c = s.h[q];
            if (c) atomicAdd(&ghist[off + q], c);
        }
        if (!slow_meet(s, sync, B * ++meetings, spin_limit)) return false;
        if (pass == 0 && !RK) {                       // keys >= 0x7f800000 (Inf/NaN) sit in the bins from 0xff0 up
            if (tid < 16 && ghist[0xff0 + tid] != 0) s.bad = 1;
        }
        const Pick p = block_pick(ghist + off, nbins, rank, s.part, s.res);
        prefix |= p.bin << shift;
        rank = p.rank_in;
        ties = p.count;
        off += nbins;
    }
    // ties inside my range; block 0 then walks the range that holds the rank-th tie in index order
    uint32_t mine = 0;
    for (uint32_t t = t0 + wave; t < t1; t += 16) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            uint32_t key[4];
            slow_keys_at<VEC, RK>(g, d, k0, k1, j, key);
#pragma unroll
            for (int q = 0; q < 4; ++q) mine += (j + q < d && key[q] == prefix) ? 1u : 0u;
        }
    }
    const uint32_t total = block_sum_u32(mine, s.wtot);         // valid on thread 0
    if (tid == 0) gcnt[b] = total;
    // Last meeting.  From here on block 0 alone speaks for the row: the other blocks publish their count,
    // arrive and leave without waiting, so no block can pass this meeting while the one that would have
    // written the result gives up.  Block 0 either sees every count and walks the range that holds the
    // rank-th tie itself (1/B of the row), or its wait runs out and the caller repeats the search alone.
    ++meetings;
    if (b != 0) {
        slow_arrive(sync);
        return true;
    }
    if (!slow_meet(s, sync, B * meetings, spin_limit)) return false;
    uint32_t before = 0, owner = B;
    for (uint32_t q = 0; q < B; ++q) {                          // uniform for the block
        const uint32_t here = gcnt[q];
        if (before < rank && rank <= before + here) {
            owner = q;
            break;
        }
        before += here;
    }
    if (owner == B) return false;                               // counts that do not add up to the histogram: search alone
    const uint32_t need = rank - before;
    const uint32_t w0 = min(owner * tpb, nwt), w1 = min(w0 + tpb, nwt);   // the owner's range of wave tiles
    if (tid == 0) s.cut = 0xffffffffu;
    __syncthreads();
    uint32_t seen = 0;
    for (uint32_t tb = w0; tb < w1; tb += 16) {                 // uniform trip count and exit
        const uint32_t t = tb + wave;
        uint64_t kb[4][4];
        uint32_t cnt = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
            uint32_t key[4] = {0, 0, 0, 0};
            if (t < w1) slow_keys_at<VEC, RK>(g, d, k0, k1, j, key);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                kb[u][q] = __ballot(t < w1 && j + q < d && key[q] == prefix);
                cnt += (uint32_t)__popcll(kb[u][q]);
            }
        }
        if (lane == 0) s.wtot[wave] = cnt;
        __syncthreads();
        uint32_t below = seen, all = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < (int)wave) below += s.wtot[w];
            all += s.wtot[w];
        }
        if (below < need && need <= below + cnt) {              // uniform for the wave: the tie is in my tile
            uint32_t n = need - below;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t cu =
                    (uint32_t)(__popcll(kb[u][0]) + __popcll(kb[u][1]) + __popcll(kb[u][2]) + __popcll(kb[u][3]));
                if (n != 0 && n <= cu) {
                    const uint32_t j = t * kWaveTile + u * kChunk + lane * 4;
                    const uint32_t lb = lanes_below(kb[u][0]) + lanes_below(kb[u][1]) + lanes_below(kb[u][2]) +
                                        lanes_below(kb[u][3]);
                    uint32_t r = n > lb ? n - lb : 0u;           // 1-based rank among my own ties, 0: before me
                    uint32_t own = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if ((kb[u][q] >> lane) & 1) {
                            ++own;
                            if (own == r) s.cut = j + q;
                        }
                    }
                    n = 0;                                      // found in this chunk
                } else if (n != 0) {
                    n -= cu;
                }
            }
        }
        seen += all;
        __syncthreads();
        if (seen >= need) break;
    }
    __syncthreads();
    if (tid == 0) slow_write_result(desc, row, prefix, rank, ties, s.cut, s.bad, RK, rk);
    return true;
}

template <bool VEC, bool RK>
__global__ __launch_bounds__(1024) void k_slow_select(const float* __restrict__ src, size_t row_stride, uint32_t d,
                                                       uint32_t nwt, uint32_t row0, RowDesc* __restrict__ desc, uint32_t k,
                                                       RkDraw rk, uint32_t* __restrict__ slow_hist,
                                                       uint32_t* __restrict__ slow_cnt, uint32_t* __restrict__ slow_sync,
                                                       uint32_t spin_limit) {
    __shared__ SlowLds s;
    const uint32_t row = row0 + blockIdx.y;
    if (desc[row].mode != kSlow) return;
    const float* __restrict__ g = src + (size_t)blockIdx.y * row_stride;
    uint32_t k0 = 0, k1 = 0;
    if (RK) {
        const uint64_t stream = rk_stream(rk.state->seed, rk.state->draw, row);
        k0 = (uint32_t)stream;
        k1 = (uint32_t)(stream >> 32);
    }
    if (gridDim.x == 1) {
        slow_single<VEC, RK>(s, g, d, row, desc, k, rk, k0, k1);
        return;
    }
    const bool done = slow_multi<VEC, RK>(s, g, d, nwt, row, desc, k, rk, k0, k1,
                                          slow_hist + (size_t)blockIdx.y * kSlowHistWords,
                                          slow_cnt + (size_t)blockIdx.y * kSlowMaxBlocks,
                                          slow_sync + (size_t)blockIdx.y * 2, spin_limit);
    if (!done && blockIdx.x == 0) slow_single<VEC, RK>(s, g, d, row, desc, k, rk, k0, k1);
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
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
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

}  // namespace liec
