// Host side of the C ABI declared in include/liec.h and include/liec_testing.h: argument checks, scratch ownership and
// the launch sequence of one compressed LIEC-SGD iteration (Algorithm 1) on a HIP stream.
#include "liec.h"
#include "liec_testing.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "liec_kernels.hpp"

using namespace liec;

namespace {

// Kernel slots for per-kernel timing: worker side, aggregation, server side, update.
constexpr int kSelSlots = 6;
enum Slot : int {
    S_W_L1 = 0, S_W_L1_FINAL,
    S_W_SEL,                       // kSelSlots slots of the worker-side top-k / random-k search
    S_AGGREGATE = S_W_SEL + kSelSlots,
    S_S_L1, S_S_L1_FINAL,
    S_S_SEL,                       // kSelSlots slots of the server-side top-k / random-k search
    S_UPDATE = S_S_SEL + kSelSlots,
    S_SYNC,
    S_COUNT
};

const char* const kWorkerSel[kSelSlots] = {"worker_filter_warm", "worker_hist0", "worker_filter_cold", "worker_list_select",
                                           "worker_slow_select", "worker_randk_mark"};
const char* const kServerSel[kSelSlots] = {"server_filter_warm", "server_hist0", "server_filter_cold", "server_list_select",
                                           "server_slow_select", "server_randk_mark"};

const char* slot_name(int s) {
    if (s == S_W_L1) return "worker_l1_bits";
    if (s == S_W_L1_FINAL) return "worker_l1_final";
    if (s >= S_W_SEL && s < S_W_SEL + kSelSlots) return kWorkerSel[s - S_W_SEL];
    if (s == S_AGGREGATE) return "server_aggregate";
    if (s == S_S_L1) return "server_l1";
    if (s == S_S_L1_FINAL) return "server_l1_final";
    if (s >= S_S_SEL && s < S_S_SEL + kSelSlots) return kServerSel[s - S_S_SEL];
    if (s == S_SYNC) return "sync";
    return "update";
}

struct ProfEvent {
    hipEvent_t start, stop;
    int slot;
};

}  // namespace

// Block partials of liec_l2_norm_static: device memory the library never allocates or frees.  Every GPU
// the library runs on holds its own copy (32 KiB) at its own address until the process ends; in host code
// the name below only stands for the symbol, the address on a device comes from static_scratch().
constexpr int kL2StaticBlocks = 4096;
static __device__ __align__(256) double scratch[kL2StaticBlocks];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device, looked up once per device with that device current.
hipError_t static_scratch(double** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<double*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct liec_ctx {
    int32_t N = 0;
    int64_t d = 0;
    int worker_comp = 0, server_comp = 0;
    int64_t worker_k = 0, server_k = 0;
    float lr = 0.f;
    hipStream_t stream = nullptr;
    int device = 0;
    bool broken = false;
    int64_t steps_done = 0;

    uint32_t nwt = 0;                          // wave tiles of 1024 columns per row
    uint32_t ncol_tiles = 0;                   // column tiles of the update kernel
    uint32_t row_blocks = 0;                   // scaled-sign pass over grads: grid (row_blocks, N)
    uint32_t filter_row_blocks = 0, filter_srv_blocks = 0;   // top-k filter pass (fewer, longer-lived blocks)
    uint32_t filter_run = 1;                   // consecutive wave tiles a wave of the filter takes at a time
    bool agg_batch = false;                    // top-k workers: the aggregation gathers 8 rows at a time (short rows)
    uint32_t agg_blocks = 0;                   // aggregation kernel
    uint32_t cold_row_blocks = 0, cold_srv_blocks = 0;   // first-digit histogram (rarely needed)
    uint32_t cap = 0;                          // candidate list capacity per row

    // device scratch
    RowDesc* desc = nullptr;                   // [N + 1]
    float* vbuf = nullptr;                     // [d]  compensated average v
    double* w_partial = nullptr;               // [N * row_blocks]
    double* s_partial = nullptr;               // [agg_blocks]
    uint16_t* bits = nullptr;                  // [(N or N + 1) * nwt * 64] sign bits (sign operators) / kept bits (random-k; row N: server)
    RkState* rk_state = nullptr;               // random-k: seed and number of the next draw (device)
    uint32_t rk_wlo = 0, rk_whi = 0, rk_slo = 0, rk_shi = 0;   // random-k: threshold bands of the worker / server draws
    bool rk_winv = false, rk_sinv = false;     // random-k: the band is thin enough to walk the priorities instead of the columns
    uint64_t* gbits = nullptr;                 // [N * nwt * 4] group bitmap of the candidates (top-k workers), either form
    bool gb_coarse = false;                    // one bit per 64-byte line instead of one per 4 columns
    uint16_t* vbits = nullptr;                 // [nwt * 64] sign bits of v (scaled-sign server, either form)
    uint64_t* sgbits = nullptr;                // [nwt * 4] group bitmap of the server's candidates in v (top-k server), fine form
    uint2* list = nullptr;                     // [(N + 1) * cap] candidates (key, index)
    uint32_t* ghist = nullptr;                 // [(N + 1) * kHistBins] first digit of a row (12 bits) or of its list (8 bits)
    uint2* shortl = nullptr;                   // [(N + 1) * kShortCap] listed entries of the first list digit's bin
    // general (degenerate-row) search: B thread blocks share a row when B * rows fit the chip
    uint32_t slow_bw = 1, slow_bs = 1;         // blocks per worker row / for the server's vector
    uint32_t slow_spin = 1u << 16;             // bound, in polls, of the waits between those blocks
    uint32_t* slow_hist = nullptr;             // [rows that share * kSlowHistWords] digit histograms
    uint32_t* slow_cnt = nullptr;              // [rows that share * kSlowMaxBlocks] ties per block
    uint32_t* slow_sync = nullptr;             // [rows that share * 2] arrivals, give-up flag
    int64_t scratch_bytes = 0;

    // blockwise scaled sign (Definition 5): block table and its scratch, set by liec_set_blocks
    uint32_t B = 0, nitems = 0;
    uint32_t* blk_off = nullptr;               // [B + 1]
    uint32_t* tile_blk = nullptr;              // [ncol_tiles]
    uint32_t* item_start = nullptr;            // [B + 1]
    L1Item* items = nullptr;                   // [nitems]
    double* blk_partial = nullptr;             // [(N + 1) * nitems]
    float* blk_scales = nullptr;               // [(N + 1) * B]
    double* blk_l1 = nullptr;                  // [(N + 1) * B]
    int64_t blk_bytes = 0;
    uint32_t* wire_tiles = nullptr;            // [nwt + 1] per-tile counts / offsets of liec_pack_topk_message
    float* wire_scales = nullptr;              // [max(B, 1)] staging for liec_unpack_sign_message
    uint32_t wire_scales_len = 0;

    // profiling
    bool profiling = false;
    bool prof_update_only = false;
    int32_t prof_steps_left = 0;
    std::vector<ProfEvent> prof;
};

namespace {

bool finite_f(float v) { return std::isfinite(v); }

// Makes the context's device current for the length of an entry point (a caller that drives several
// devices may have switched since liec_create) and puts the caller's back on the way out.
struct DeviceScope {
    int prev = -1;
    bool ok = true;
    explicit DeviceScope(const liec_ctx* c) {
        int cur = 0;
        ok = hipGetDevice(&cur) == hipSuccess;
        if (ok && cur != c->device) {
            ok = hipSetDevice(c->device) == hipSuccess;
            if (ok) prev = cur;
        }
    }
    ~DeviceScope() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
    DeviceScope(const DeviceScope&) = delete;
    DeviceScope& operator=(const DeviceScope&) = delete;
};

template <typename T>
hipError_t dev_alloc(liec_ctx* c, T** p, size_t count) {
    const size_t bytes = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes);
    if (e == hipSuccess) c->scratch_bytes += (int64_t)bytes;
    return e;
}

void free_blocks(liec_ctx* c) {
    (void)hipFree(c->blk_off);
    (void)hipFree(c->tile_blk);
    (void)hipFree(c->item_start);
    (void)hipFree(c->items);
    (void)hipFree(c->blk_partial);
    (void)hipFree(c->blk_scales);
    (void)hipFree(c->blk_l1);
    c->blk_off = c->tile_blk = c->item_start = nullptr;
    c->items = nullptr;
    c->blk_partial = c->blk_l1 = nullptr;
    c->blk_scales = nullptr;
    c->scratch_bytes -= c->blk_bytes;
    c->blk_bytes = 0;
    c->B = c->nitems = 0;
}

BlockTable block_table(const liec_ctx* c) { return BlockTable{c->tile_blk, c->blk_off, c->blk_scales, c->B}; }

void free_scratch(liec_ctx* c) {
    free_blocks(c);
    (void)hipFree(c->wire_scales);
    (void)hipFree(c->wire_tiles);
    (void)hipFree(c->desc);
    (void)hipFree(c->vbuf);
    (void)hipFree(c->w_partial);
    (void)hipFree(c->s_partial);
    (void)hipFree(c->bits);
    (void)hipFree(c->rk_state);
    (void)hipFree(c->gbits);
    (void)hipFree(c->vbits);
    (void)hipFree(c->sgbits);
    (void)hipFree(c->list);
    (void)hipFree(c->ghist);
    (void)hipFree(c->shortl);
    (void)hipFree(c->slow_hist);
    (void)hipFree(c->slow_cnt);
    (void)hipFree(c->slow_sync);
}

bool valid_comp(int c) {
    return c == LIEC_COMP_IDENTITY || c == LIEC_COMP_SIGN || c == LIEC_COMP_TOPK || c == LIEC_COMP_BLOCKSIGN ||
           c == LIEC_COMP_RANDK;
}

bool selects_k(int c) { return c == LIEC_COMP_TOPK || c == LIEC_COMP_RANDK; }

// Random-k: band of keys [lo, hi) that holds the k-th largest of d uniform 31-bit priorities, 8 standard
// deviations of that order statistic on either side (the search stays exact if the key falls outside).
void randk_band(int64_t d, int64_t k, uint32_t* lo, uint32_t* hi) {
    const double range = 2147483648.0, dd = (double)d, kk = (double)k;
    const double centre = range * (1.0 - kk / dd);
    const double sigma = range * std::sqrt(kk * (dd - kk) / dd) / dd;
    double margin = 8.0 * sigma + 4.0 * range / dd + 16.0;
    if (margin > 33554432.0) margin = 33554432.0;      // 2^25: the list select spans bands of 2^26 keys
    const double l = std::floor(centre - margin), h = std::ceil(centre + margin);
    *lo = l < 0.0 ? 0u : (uint32_t)l;
    *hi = h > range ? 0x80000000u : (uint32_t)h;
    if (*hi <= *lo) *hi = *lo + 1;
}

struct Launcher {
    liec_ctx* c;
    bool ok = true;
    bool recording = false;
    void begin(int slot) {
        recording = c->profiling && (!c->prof_update_only || slot == S_UPDATE || slot == S_SYNC);
        if (!recording) return;
        ProfEvent ev{nullptr, nullptr, slot};
        if (hipEventCreate(&ev.start) != hipSuccess || hipEventCreate(&ev.stop) != hipSuccess) {
            ok = false;
            return;
        }
        if (hipEventRecord(ev.start, c->stream) != hipSuccess) ok = false;
        c->prof.push_back(ev);
    }
    void end() {
        if (hipGetLastError() != hipSuccess) ok = false;
        if (!recording || c->prof.empty()) return;
        if (hipEventRecord(c->prof.back().stop, c->stream) != hipSuccess) ok = false;
    }
};

// Top-k threshold search (Definition 2) of `rows` rows of `src`; per-row state lives at row0 + r.
// The host enqueues the same five kernels every step; each one acts only on the rows whose state
// asks for it, so the steady state costs one pass over the data, two short passes over the candidate
// lists (in the launches that otherwise serve rows without a prediction) and one block per row of list
// select; the general search returns at once.
// RK: the same search over the priorities of a random-k draw (Definition 3), which read nothing from
// `src`, followed by the kernel that completes the kept bitmap.
template <bool VEC, bool RK>
void launch_select(Launcher& L, const float* src, size_t row_stride, uint32_t rows, uint32_t row0, uint32_t k,
                   uint64_t* gbits, bool coarse, uint32_t blocks, uint32_t cold_blocks, int slot0, RkDraw rk,
                   bool rk_inverse = false) {
    liec_ctx* c = L.c;
    const uint32_t d = (uint32_t)c->d;
    hipStream_t st = c->stream;
    const dim3 grid(blocks, rows), cold_grid(cold_blocks, rows);
    // random-k with a thin band: clear the kept bitmap, then walk the priorities above the band
    // few, long-lived blocks (every block ends with an atomic on the row's counters): one per 32768 words to invert
    const uint64_t inv_words = 2ull * (0x80000000ull - rk.fix_lo);
    const dim3 inv_grid((uint32_t)std::min<uint64_t>(std::max<uint64_t>(inv_words / 32768, 128), 1024), rows);
    const dim3 zero_grid(std::min<uint32_t>((c->nwt * 32 + kBlock - 1) / kBlock, 4096u), rows);
    for (int pass = 0; pass < 2; ++pass) {
        const bool cold_pass = pass == 1;
        if (cold_pass) {
            L.begin(slot0 + 1);
            k_hist0<VEC, RK><<<cold_grid, kBlock, 0, st>>>(src, row_stride, d, c->nwt, row0, c->desc, c->ghist, c->list, c->cap, k, rk);
            L.end();
        }
        L.begin(slot0 + (cold_pass ? 2 : 0));
        if (RK && rk_inverse) {
            // (the second pass is rare: a small grid, so that its blocks' returning at once costs little)
            const dim3 zg(cold_pass ? std::min(zero_grid.x, 256u) : zero_grid.x, rows);
            k_rk_zero<<<zg, kBlock, 0, st>>>(c->nwt, row0, c->desc, cold_pass, c->cap, k, c->bits);
            k_rk_filter_inverse<<<inv_grid, kBlock, 0, st>>>(d, c->nwt, row0, c->desc, cold_pass, c->ghist, k, c->bits,
                                                             c->list, c->cap, c->shortl, rk);
        } else {
            k_filter<VEC, RK><<<grid, kBlock, 0, st>>>(src, row_stride, d, c->nwt, row0, c->desc, cold_pass, c->ghist, k,
                                                        gbits, c->bits, c->list, c->cap, c->shortl, rk, coarse, c->filter_run);
        }
        L.end();
    }
    // scratch of the general search: the worker rows' slots come first, then the server's
    const bool server_side = row0 != 0;
    const uint32_t slow_b = server_side ? c->slow_bs : c->slow_bw;
    const size_t slow_slot = server_side && c->slow_bw > 1 ? (size_t)c->N : 0;
    uint32_t* const shist = slow_b > 1 ? c->slow_hist + slow_slot * kSlowHistWords : nullptr;
    uint32_t* const scnt = slow_b > 1 ? c->slow_cnt + slow_slot * kSlowMaxBlocks : nullptr;
    uint32_t* const ssync = slow_b > 1 ? c->slow_sync + slow_slot * 2 : nullptr;
    L.begin(slot0 + 3);
    k_list_select<<<rows, kSelectBlock, 0, st>>>(row0, c->desc, c->ghist, c->list, c->cap, c->shortl, k, rk.fix_lo, rk.fix_hi,
                                                 ssync);
    L.end();
    L.begin(slot0 + 4);
    k_slow_select<VEC, RK><<<dim3(slow_b, rows), 1024, 0, st>>>(src, row_stride, d, c->nwt, row0, c->desc, k, rk, shist, scnt,
                                                                 ssync, c->slow_spin);
    L.end();
    if (RK) {
        L.begin(slot0 + 5);
        k_rk_mark<<<dim3(cold_blocks, rows), kBlock, 0, st>>>(d, c->nwt, row0, c->desc, c->list, c->cap, c->bits, rk);
        L.end();
    }
}

// Blockwise scaled sign (Definition 5): per-block L1 norms of `rows` rows of `src` -> scales; for the
// workers also the sign bits.  slot0 and slot0 + 1 time the two kernels.
template <bool VEC>
void launch_block_l1(Launcher& L, const float* src, size_t row_stride, uint32_t rows, uint32_t row0, uint16_t* bits,
                     int slot0) {
    liec_ctx* c = L.c;
    L.begin(slot0);
    k_l1_items<VEC><<<dim3(c->nitems, rows), kBlock, 0, c->stream>>>(src, row_stride, (uint32_t)c->d, c->nwt, row0, c->items,
                                                                      c->blk_partial, bits);
    L.end();
    L.begin(slot0 + 1);
    k_l1_items_final<<<dim3(c->B, rows), kBlock, 0, c->stream>>>(c->blk_partial, c->nitems, c->item_start, c->blk_off,
                                                                  c->B, row0, c->blk_scales, c->blk_l1);
    L.end();
}

template <int WC, bool VEC>
void launch_aggregate(Launcher& L, const float* grads, const float* e, bool srv_l1) {
    liec_ctx* c = L.c;
    const float inv_n = 1.0f / (float)c->N;
    const uint32_t d = (uint32_t)c->d;
    L.begin(S_AGGREGATE);
    auto launch = [&](auto kernel) {
        kernel<<<c->agg_blocks, kBlock, 0, c->stream>>>(grads, c->bits, c->gbits, c->N, d, c->nwt, inv_n, c->desc, e, c->vbuf,
                                                       c->s_partial, block_table(c), c->gb_coarse, c->vbits);
    };
    if (WC == kTopk && c->agg_batch) {                          // short rows: the gathers of 8 rows at a time
        if (srv_l1) launch(k_aggregate<WC, true, VEC, WC == kTopk>);
        else launch(k_aggregate<WC, false, VEC, WC == kTopk>);
    } else {
        if (srv_l1) launch(k_aggregate<WC, true, VEC>);
        else launch(k_aggregate<WC, false, VEC>);
    }
    L.end();
}

template <int WC, int SC, bool VEC>
void launch_update(Launcher& L, const float* grads, float* x, float* e) {
    liec_ctx* c = L.c;
    const uint32_t panel = c->ncol_tiles < kUpdatePanel ? c->ncol_tiles : kUpdatePanel;
    const uint32_t npanels = (c->ncol_tiles + panel - 1) / panel;
    const uint64_t blocks = (uint64_t)npanels * panel * (uint64_t)c->N;
    L.begin(S_UPDATE);
    k_update<WC, SC, VEC><<<(uint32_t)blocks, kBlock, 0, c->stream>>>(grads, x, c->vbuf, e, c->N, panel, c->ncol_tiles,
                                                                       (uint32_t)c->d, -c->lr, c->desc, block_table(c),
                                                                       c->bits, c->vbits, c->sgbits);
    L.end();
}

template <int WC, bool VEC>
void launch_update_sc(Launcher& L, int sc, const float* grads, float* x, float* e) {
    switch (sc) {
    case kIdentity: launch_update<WC, kIdentity, VEC>(L, grads, x, e); break;
    case kSign: launch_update<WC, kSign, VEC>(L, grads, x, e); break;
    case kBlockSign: launch_update<WC, kBlockSign, VEC>(L, grads, x, e); break;
    case kRandk: launch_update<WC, kRandk, VEC>(L, grads, x, e); break;
    default: launch_update<WC, kTopk, VEC>(L, grads, x, e); break;
    }
}

template <bool VEC>
void run_step(Launcher& L, const float* grads, float* x, float* e) {
    liec_ctx* c = L.c;
    const uint32_t d = (uint32_t)c->d;
    const size_t stride = (size_t)c->d;

    // ---- workers: p^i = C_w(g_i), reduced to a per-row descriptor (+ packed bits) ------------------
    if (c->worker_comp == kSign) {
        L.begin(S_W_L1);
        k_l1_bits<VEC><<<dim3(c->row_blocks, c->N), kBlock, 0, c->stream>>>(grads, stride, d, c->nwt, c->w_partial,
                                                                             c->bits);
        L.end();
        L.begin(S_W_L1_FINAL);
        k_l1_final<<<c->N, kBlock, 0, c->stream>>>(c->w_partial, c->row_blocks, d, c->desc);
        L.end();
    } else if (c->worker_comp == kBlockSign) {
        launch_block_l1<VEC>(L, grads, stride, (uint32_t)c->N, 0u, c->bits, S_W_L1);
    } else if (c->worker_comp == kTopk) {
        launch_select<VEC, false>(L, grads, stride, (uint32_t)c->N, 0u, (uint32_t)c->worker_k, c->gbits, c->gb_coarse,
                                  c->filter_row_blocks, c->cold_row_blocks, S_W_SEL, RkDraw{nullptr, 0, 0});
    } else if (c->worker_comp == kRandk) {
        launch_select<VEC, true>(L, grads, stride, (uint32_t)c->N, 0u, (uint32_t)c->worker_k, nullptr, false,
                                 c->filter_row_blocks, c->cold_row_blocks, S_W_SEL,
                                 RkDraw{c->rk_state, c->rk_wlo, c->rk_whi}, c->rk_winv);
    }

    // ---- server: v = e + mean_i p^i, then the descriptor of C_s(v) ---------------------------------
    const bool srv_l1 = c->server_comp == kSign;
    switch (c->worker_comp) {
    case kIdentity: launch_aggregate<kIdentity, VEC>(L, grads, e, srv_l1); break;
    case kSign: launch_aggregate<kSign, VEC>(L, grads, e, srv_l1); break;
    case kBlockSign: launch_aggregate<kBlockSign, VEC>(L, grads, e, srv_l1); break;
    case kRandk: launch_aggregate<kRandk, VEC>(L, grads, e, srv_l1); break;
    default: launch_aggregate<kTopk, VEC>(L, grads, e, srv_l1); break;
    }
    if (c->server_comp == kSign) {
        L.begin(S_S_L1_FINAL);
        k_l1_final<<<1, kBlock, 0, c->stream>>>(c->s_partial, c->agg_blocks, d, c->desc + c->N);
        L.end();
    } else if (c->server_comp == kBlockSign) {
        launch_block_l1<VEC>(L, c->vbuf, 0, 1u, (uint32_t)c->N, nullptr, S_S_L1);
    } else if (c->server_comp == kTopk) {
        // v is always 16-byte aligned scratch, but d % 4 decides whether 128-bit loads stay in bounds
        // the server's candidates get the fine group bitmap: the update kernel reads v only where a bit is set
        launch_select<VEC, false>(L, c->vbuf, 0, 1u, (uint32_t)c->N, (uint32_t)c->server_k, c->sgbits, false,
                                  c->filter_srv_blocks, c->cold_srv_blocks, S_S_SEL, RkDraw{nullptr, 0, 0});
    } else if (c->server_comp == kRandk) {
        launch_select<VEC, true>(L, c->vbuf, 0, 1u, (uint32_t)c->N, (uint32_t)c->server_k, nullptr, false,
                                 c->filter_srv_blocks, c->cold_srv_blocks, S_S_SEL,
                                 RkDraw{c->rk_state, c->rk_slo, c->rk_shi}, c->rk_sinv);
    }

    // ---- p = C_s(v), e <- v - p, x^i <- x^i - lr (p + (g_i - p^i)) ---------------------------------
    switch (c->worker_comp) {
    case kIdentity: launch_update_sc<kIdentity, VEC>(L, c->server_comp, grads, x, e); break;
    case kSign: launch_update_sc<kSign, VEC>(L, c->server_comp, grads, x, e); break;
    case kBlockSign: launch_update_sc<kBlockSign, VEC>(L, c->server_comp, grads, x, e); break;
    case kRandk: launch_update_sc<kRandk, VEC>(L, c->server_comp, grads, x, e); break;
    default: launch_update_sc<kTopk, VEC>(L, c->server_comp, grads, x, e); break;
    }
    // the next compressed iteration makes the next draw
    if (c->worker_comp == kRandk || c->server_comp == kRandk) {
        k_rk_advance<<<1, 1, 0, c->stream>>>(c->rk_state);
        if (hipGetLastError() != hipSuccess) L.ok = false;
    }
}

bool overlap(const void* a, size_t na, const void* b, size_t nb) {
    const char* pa = (const char*)a;
    const char* pb = (const char*)b;
    return pa < pb + nb && pb < pa + na;
}

void drop_prof(liec_ctx* c) {
    for (auto& ev : c->prof) {
        if (ev.start) (void)hipEventDestroy(ev.start);
        if (ev.stop) (void)hipEventDestroy(ev.stop);
    }
    c->prof.clear();
}

}  // namespace

extern "C" {

const char* liec_status_string(liec_status s) {
    switch (s) {
    case LIEC_OK: return "ok";
    case LIEC_EINVAL: return "invalid argument";
    case LIEC_ENOMEM: return "out of memory";
    case LIEC_EDEVICE: return "HIP device error";
    case LIEC_ENONFINITE: return "non-finite value met in the last step";
    default: return "unknown status";
    }
}

liec_status liec_create_ex(liec_ctx** out, int32_t N, int64_t d, liec_comp worker_comp, int64_t worker_k,
                           liec_comp server_comp, int64_t server_k, float lr, void* hip_stream) {
    if (!out) return LIEC_EINVAL;
    *out = nullptr;
    // rows are the y dimension of several launch grids (at most 65535 blocks)
    if (N < 1 || N > 65535 || d < 1 || d >= ((int64_t)1 << 31) - ((int64_t)1 << 20)) return LIEC_EINVAL;
    if (!valid_comp((int)worker_comp) || !valid_comp((int)server_comp) || !finite_f(lr)) return LIEC_EINVAL;
    // the update kernel launches one block per (1024-column tile, row): keep that under 2^31
    if (((d + kColTile - 1) / kColTile + kUpdatePanel) * (int64_t)N >= ((int64_t)1 << 31)) return LIEC_EINVAL;
    if (selects_k((int)worker_comp) && (worker_k < 1 || worker_k > d)) return LIEC_EINVAL;
    if (selects_k((int)server_comp) && (server_k < 1 || server_k > d)) return LIEC_EINVAL;

    liec_ctx* c = new (std::nothrow) liec_ctx();
    if (!c) return LIEC_ENOMEM;
    c->N = N;
    c->d = d;
    c->worker_comp = (int)worker_comp;
    c->server_comp = (int)server_comp;
    c->worker_k = selects_k((int)worker_comp) ? worker_k : 0;
    c->server_k = selects_k((int)server_comp) ? server_k : 0;
    if (worker_comp == LIEC_COMP_RANDK) randk_band(d, worker_k, &c->rk_wlo, &c->rk_whi);
    if (server_comp == LIEC_COMP_RANDK) randk_band(d, server_k, &c->rk_slo, &c->rk_shi);
    // 2 * (2^31 - lo) words carry a priority at or above the band: inverting them beats hashing d columns
    // when they are well under d (each inverted word also costs an atomic when it lands on a column)
    c->rk_winv = worker_comp == LIEC_COMP_RANDK && 2.0 * (2147483648.0 - (double)c->rk_wlo) < 0.5 * (double)d;
    c->rk_sinv = server_comp == LIEC_COMP_RANDK && 2.0 * (2147483648.0 - (double)c->rk_slo) < 0.5 * (double)d;
    c->lr = lr;
    c->stream = (hipStream_t)hip_stream;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return LIEC_EDEVICE;
    }

    const bool any_topk = selects_k((int)worker_comp) || selects_k((int)server_comp);   // any threshold search
    const uint32_t un = (uint32_t)N;
    c->nwt = (uint32_t)((d + kWaveTile - 1) / kWaveTile);
    c->ncol_tiles = (uint32_t)((d + kColTile - 1) / kColTile);
    const uint32_t blk_iters = (c->nwt + 3) / 4;               // block iterations that cover one row
    auto clampu = [](uint32_t v, uint32_t lo, uint32_t hi) { return v < lo ? lo : (v > hi ? hi : v); };
    // Grid sizes come from sweeps on the VGG-16- and ResNet-shaped workloads.  Every block gets the same
    // whole number of iterations.
    auto balanced = [&](uint32_t max_blocks) {
        const uint32_t per = (blk_iters + max_blocks - 1) / max_blocks;
        return (blk_iters + per - 1) / per;
    };
    // the scaled-sign pass streams best as one 4096-column iteration per block
    c->row_blocks = balanced(1u << 20);
    // the filter pays one atomic on the row's counters per block: about 1024 long-lived blocks per row
    // (more when there are too few rows to fill the chip)
    // A wave of the filter takes 4 consecutive wave tiles at a time on long rows (a block then covers 16, and the
    // group words it writes fill whole 128-byte lines of the bitmap: measured 2 % faster than 1 on rows of 25M
    // and 138M columns, 2 and 8 in between); short rows keep 1, so that enough blocks are in flight.
    c->filter_run = c->nwt >= 8192u ? 4u : 1u;
    // top-k workers: on rows under 2^23 columns the aggregation is bound by the latency of its dependent loads and
    // gathers 8 rows at a time (C2: 0.032 -> 0.021 ms); on long rows that measured slower (C4 0.127 -> 0.156 ms,
    // C5 0.39 -> 0.57 ms)
    c->agg_batch = c->nwt < 8192u;
    auto balanced_filter = [&](uint32_t max_blocks) {
        const uint32_t iters = (c->nwt + 4 * c->filter_run - 1) / (4 * c->filter_run);
        const uint32_t per = (iters + max_blocks - 1) / max_blocks;
        return (iters + per - 1) / per;
    };
    c->filter_row_blocks = balanced_filter(clampu(4096u / un, 1024u, 4096u));
    c->filter_srv_blocks = balanced_filter(8192u);
    // the aggregation reads sign bits fastest with many short blocks, and gathers fastest with fewer
    const bool gathers = worker_comp == LIEC_COMP_TOPK || worker_comp == LIEC_COMP_RANDK;
    c->agg_blocks = balanced(gathers ? 16384u : 65536u);
    c->cold_row_blocks = clampu(2048u / un, 1u, blk_iters);
    c->cold_srv_blocks = clampu(2048u, 1u, blk_iters);
    // Candidate list capacity per row: the warm band lists a few per cent of k entries and the first-digit
    // bin that holds rank k about k / 2 for bell-shaped rows, so 8 k (at most d / 16) leaves a wide margin;
    // a band that needs more falls to the first-digit histogram or the general search, as any overflow does.
    const int64_t kmax = std::max(c->worker_k, c->server_k);
    const int64_t want = std::min<int64_t>(d / 16, 8 * kmax) + 4096;
    c->cap = (uint32_t)std::min<int64_t>(want, d);
    c->cap += c->cap & 1u;                     // even: every row's list starts 16-byte aligned (read two entries at a time)

    const size_t rows = (size_t)N + 1;
    hipError_t e = dev_alloc(c, &c->desc, rows);
    if (e == hipSuccess) e = dev_alloc(c, &c->vbuf, (size_t)c->nwt * kWaveTile);
    if (e == hipSuccess) e = dev_alloc(c, &c->w_partial, (size_t)N * c->row_blocks);
    if (e == hipSuccess) e = dev_alloc(c, &c->s_partial, (size_t)c->agg_blocks);
    if (e == hipSuccess && server_comp == LIEC_COMP_RANDK)
        e = dev_alloc(c, &c->bits, rows * c->nwt * 64);
    else if (e == hipSuccess && (worker_comp == LIEC_COMP_SIGN || worker_comp == LIEC_COMP_BLOCKSIGN ||
                                 worker_comp == LIEC_COMP_RANDK))
        e = dev_alloc(c, &c->bits, (size_t)N * c->nwt * 64);
    if (e == hipSuccess) e = dev_alloc(c, &c->rk_state, 1);
    if (e == hipSuccess) e = hipMemsetAsync(c->rk_state, 0, sizeof(RkState), c->stream);
    // Which form of the group bitmap: measured over 13 shapes (N 8..64, d 25M..138M, k/d 0.1 % and 0.5 %, three
    // gradient recipes) the row length decides -- one bit per 64-byte line is 1-2 % of a step faster from
    // d = 48M up (filter -3 %, aggregation -10..20 %), even at 36M, and up to 1 % slower at 25M (the
    // aggregation fetches for four times as many lanes and has less bitmap to save on).
    c->gb_coarse = worker_comp == LIEC_COMP_TOPK && d >= 40000000;
    if (e == hipSuccess && worker_comp == LIEC_COMP_TOPK)
        e = dev_alloc(c, &c->gbits, (size_t)N * c->nwt * 4);      // room for either form
    if (e == hipSuccess && (server_comp == LIEC_COMP_SIGN || server_comp == LIEC_COMP_BLOCKSIGN))
        e = dev_alloc(c, &c->vbits, (size_t)c->nwt * 64);
    if (e == hipSuccess && server_comp == LIEC_COMP_TOPK) e = dev_alloc(c, &c->sgbits, (size_t)c->nwt * 4);
    if (e == hipSuccess && any_topk) e = dev_alloc(c, &c->list, rows * c->cap);
    if (e == hipSuccess && any_topk) e = dev_alloc(c, &c->ghist, rows * kHistBins);
    if (e == hipSuccess && any_topk) e = dev_alloc(c, &c->shortl, rows * kShortCap);
    if (e == hipSuccess && any_topk) {
        // blocks that share a row meet inside the kernel, so all of them must be resident at once:
        // at most one per compute unit
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || cus < 1) cus = 1;
        c->slow_bw = clampu((uint32_t)cus / un, 1u, (uint32_t)kSlowMaxBlocks);
        c->slow_bs = clampu((uint32_t)cus, 1u, (uint32_t)kSlowMaxBlocks);
        const size_t slots = (c->slow_bw > 1 ? (size_t)N : 0) + (c->slow_bs > 1 ? 1 : 0);
        if (slots) {
            e = dev_alloc(c, &c->slow_hist, slots * kSlowHistWords);
            if (e == hipSuccess) e = dev_alloc(c, &c->slow_cnt, slots * kSlowMaxBlocks);
            if (e == hipSuccess) e = dev_alloc(c, &c->slow_sync, slots * 2);
            if (e == hipSuccess) e = hipMemsetAsync(c->slow_sync, 0, slots * 2 * sizeof(uint32_t), c->stream);
        }
    }
    if (e == hipSuccess) {
        std::vector<RowDesc> init(rows);
        std::memset(init.data(), 0, rows * sizeof(RowDesc));
        for (auto& r : init) r.mode = kCold;       // no prediction before the first step
        for (size_t r = 0; r < rows; ++r) {        // random-k rows know their band from the start
            const bool rk = r < (size_t)N ? worker_comp == LIEC_COMP_RANDK : server_comp == LIEC_COMP_RANDK;
            if (!rk) continue;
            init[r].mode = kWarm;
            init[r].lo = r < (size_t)N ? c->rk_wlo : c->rk_slo;
            init[r].hi = r < (size_t)N ? c->rk_whi : c->rk_shi;
        }
        e = hipMemcpy(c->desc, init.data(), rows * sizeof(RowDesc), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && any_topk) e = hipMemsetAsync(c->ghist, 0, rows * kHistBins * sizeof(uint32_t), c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_scratch(c);
        delete c;
        return e == hipErrorOutOfMemory ? LIEC_ENOMEM : LIEC_EDEVICE;
    }
    *out = c;
    return LIEC_OK;
}

liec_status liec_create(liec_ctx** out, int32_t N, int64_t d, liec_comp compressor, int64_t k, float lr) {
    return liec_create_ex(out, N, d, compressor, k, compressor, k, lr, nullptr);
}

liec_status liec_step(liec_ctx* c, const float* grads, float* x, float* server_err) {
    if (!c || !grads || !x || !server_err) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    const size_t nd = (size_t)c->N * (size_t)c->d * sizeof(float), db = (size_t)c->d * sizeof(float);
    if (overlap(grads, nd, x, nd) || overlap(grads, nd, server_err, db) || overlap(x, nd, server_err, db))
        return LIEC_EINVAL;
    if (((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 3u) return LIEC_EINVAL;
    const bool vec = (c->d % 4 == 0) && ((((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 15u) == 0);

    if ((c->worker_comp == kBlockSign || c->server_comp == kBlockSign) && c->B == 0) return LIEC_EINVAL;
    Launcher L{c};
    const bool was_profiling = c->profiling;
    if (c->profiling && c->prof_steps_left <= 0) c->profiling = false;
    if (c->profiling) --c->prof_steps_left;
    if (vec)
        run_step<true>(L, grads, x, server_err);
    else
        run_step<false>(L, grads, x, server_err);
    c->profiling = was_profiling;
    if (!L.ok) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    ++c->steps_done;
    return LIEC_OK;
}

liec_status liec_set_random(liec_ctx* c, uint64_t seed, uint64_t draw) {
    if (!c) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    const RkState st{seed, draw};
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(c->rk_state, &st, sizeof st, hipMemcpyHostToDevice) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_force_search_mode(liec_ctx* c, int32_t mode) {
    if (!c || (mode != (int32_t)kWarm && mode != (int32_t)kCold && mode != (int32_t)kSlow)) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    std::vector<RowDesc> h((size_t)c->N + 1);
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(h.data(), c->desc, h.size() * sizeof(RowDesc), hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    for (size_t r = 0; r < h.size(); ++r) {
        if (!selects_k(r < (size_t)c->N ? c->worker_comp : c->server_comp)) continue;
        h[r].mode = (uint32_t)mode;
        clear_counts(h[r]);
    }
    if (hipMemcpy(c->desc, h.data(), h.size() * sizeof(RowDesc), hipMemcpyHostToDevice) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_get_search_state(liec_ctx* c, int32_t row, uint32_t* out) {
    if (!c || !out || row < 0 || row > c->N) return LIEC_EINVAL;
    if (!selects_k(row < c->N ? c->worker_comp : c->server_comp)) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    RowDesc r;
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(&r, c->desc + row, sizeof r, hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    out[0] = r.mode;
    out[1] = r.lo;
    out[2] = r.hi;
    out[3] = r.n_list;
    out[4] = r.misses;
    out[5] = r.swing;
    out[6] = r.dense;
    out[7] = 0;
    return LIEC_OK;
}

liec_status liec_set_group_bitmap(liec_ctx* c, int32_t per_line) {
    if (!c || (per_line != 0 && per_line != 1) || c->worker_comp != kTopk) return LIEC_EINVAL;
    c->gb_coarse = per_line != 0;              // the buffer always has room for the finer form
    return LIEC_OK;
}

liec_status liec_set_gather_batching(liec_ctx* c, int32_t on) {
    if (!c || (on != 0 && on != 1) || c->worker_comp != kTopk) return LIEC_EINVAL;
    c->agg_batch = on != 0;
    return LIEC_OK;
}

liec_status liec_set_search_wait(liec_ctx* c, int32_t polls) {
    if (!c || polls < 0) return LIEC_EINVAL;
    c->slow_spin = (uint32_t)polls;
    return LIEC_OK;
}

liec_status liec_get_random(liec_ctx* c, uint64_t* seed, uint64_t* draw) {
    if (!c || !seed || !draw) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    RkState st{0, 0};
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(&st, c->rk_state, sizeof st, hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    *seed = st.seed;
    *draw = st.draw;
    return LIEC_OK;
}

liec_status liec_step_sync(liec_ctx* c, const float* grads, float* x, float* server_err) {
    if (!c || !grads || !x || !server_err) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    const size_t nd = (size_t)c->N * (size_t)c->d * sizeof(float), db = (size_t)c->d * sizeof(float);
    if (overlap(grads, nd, x, nd) || overlap(grads, nd, server_err, db) || overlap(x, nd, server_err, db))
        return LIEC_EINVAL;
    if (((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 3u) return LIEC_EINVAL;
    const bool vec = (c->d % 4 == 0) && ((((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 15u) == 0);
    Launcher L{c};
    const bool was_profiling = c->profiling;
    if (c->profiling && c->prof_steps_left <= 0) c->profiling = false;
    if (c->profiling) --c->prof_steps_left;
    const float inv_n = 1.0f / (float)c->N;
    const uint32_t panel = c->ncol_tiles < kUpdatePanel ? c->ncol_tiles : kUpdatePanel;
    const uint32_t npanels = (c->ncol_tiles + panel - 1) / panel;
    const uint32_t spread_blocks = (uint32_t)((uint64_t)npanels * panel * (uint64_t)c->N);
    L.begin(S_SYNC);
    if (vec) {
        k_sync_reduce<true><<<c->ncol_tiles, kBlock, 0, c->stream>>>(grads, x, server_err, c->N, (uint32_t)c->d, inv_n, -c->lr);
        k_sync_spread<true><<<spread_blocks, kBlock, 0, c->stream>>>(x, server_err, c->N, panel, c->ncol_tiles, (uint32_t)c->d);
    } else {
        k_sync_reduce<false><<<c->ncol_tiles, kBlock, 0, c->stream>>>(grads, x, server_err, c->N, (uint32_t)c->d, inv_n, -c->lr);
        k_sync_spread<false><<<spread_blocks, kBlock, 0, c->stream>>>(x, server_err, c->N, panel, c->ncol_tiles, (uint32_t)c->d);
    }
    L.end();
    c->profiling = was_profiling;
    if (!L.ok) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    ++c->steps_done;
    return LIEC_OK;
}

liec_status liec_iteration(liec_ctx* c, int64_t t, int64_t period, const float* grads, float* x, float* server_err) {
    if (t < 0 || period < 0 || period == 1) return LIEC_EINVAL;
    if (period >= 2 && (t + 1) % period == 0) return liec_step_sync(c, grads, x, server_err);
    return liec_step(c, grads, x, server_err);
}

liec_status liec_set_blocks(liec_ctx* c, const int64_t* offsets, int32_t nblocks) {
    if (!c || !offsets || nblocks < 1 || nblocks > 65536) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    if (offsets[0] != 0 || offsets[nblocks] != c->d) return LIEC_EINVAL;
    for (int32_t b = 0; b < nblocks; ++b)
        if (offsets[b + 1] <= offsets[b]) return LIEC_EINVAL;
    if (hipStreamSynchronize(c->stream) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    free_blocks(c);
    const uint32_t B = (uint32_t)nblocks, d = (uint32_t)c->d;
    std::vector<uint32_t> off(B + 1), tile_blk(c->ncol_tiles), item_start(B + 1);
    for (uint32_t b = 0; b <= B; ++b) off[b] = (uint32_t)offsets[b];
    for (uint32_t t = 0, b = 0; t < c->ncol_tiles; ++t) {
        const uint32_t first = t * (uint32_t)kColTile, last = std::min(first + (uint32_t)kColTile, d) - 1;
        while (first >= off[b + 1]) ++b;
        tile_blk[t] = b | (last >= off[b + 1] ? 0x80000000u : 0u);
    }
    std::vector<L1Item> items;
    const uint32_t big = 4u * (uint32_t)kWaveTile;                 // columns per block of k_l1_items
    std::vector<uint32_t> owner((d + big - 1) / big, 0xffffffffu); // the first item of a tile writes its bits
    for (uint32_t b = 0; b < B; ++b) {
        item_start[b] = (uint32_t)items.size();
        for (uint32_t t = off[b] / big; t <= (off[b + 1] - 1) / big; ++t) {
            L1Item it;
            it.tile = t;
            it.lo = std::max(off[b], t * big);
            it.hi = std::min(off[b + 1], (t + 1) * big);
            it.write_bits = owner[t] == 0xffffffffu ? 1u : 0u;
            owner[t] = b;
            items.push_back(it);
        }
    }
    item_start[B] = (uint32_t)items.size();
    c->B = B;
    c->nitems = (uint32_t)items.size();
    const size_t rows = (size_t)c->N + 1;
    const int64_t before = c->scratch_bytes;
    hipError_t e = dev_alloc(c, &c->blk_off, (size_t)B + 1);
    if (e == hipSuccess) e = dev_alloc(c, &c->tile_blk, (size_t)c->ncol_tiles);
    if (e == hipSuccess) e = dev_alloc(c, &c->item_start, (size_t)B + 1);
    if (e == hipSuccess) e = dev_alloc(c, &c->items, items.size());
    if (e == hipSuccess) e = dev_alloc(c, &c->blk_partial, rows * items.size());
    if (e == hipSuccess) e = dev_alloc(c, &c->blk_scales, rows * B);
    if (e == hipSuccess) e = dev_alloc(c, &c->blk_l1, rows * B);
    c->blk_bytes = c->scratch_bytes - before;
    if (e == hipSuccess) e = hipMemcpy(c->blk_off, off.data(), off.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->tile_blk, tile_blk.data(), tile_blk.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->item_start, item_start.data(), item_start.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->items, items.data(), items.size() * sizeof(L1Item), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(c->blk_scales, 0, rows * B * sizeof(float));
    if (e == hipSuccess) e = hipMemset(c->blk_l1, 0, rows * B * sizeof(double));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_blocks(c);
        return e == hipErrorOutOfMemory ? LIEC_ENOMEM : LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_get_block_scales(liec_ctx* c, float* worker_scales, float* server_scales) {
    if (!c || c->B == 0) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    hipError_t e = hipStreamSynchronize(c->stream);
    const size_t nb = (size_t)c->N * c->B;
    if (e == hipSuccess && worker_scales) {
        if (c->worker_comp == kBlockSign)
            e = hipMemcpy(worker_scales, c->blk_scales, nb * sizeof(float), hipMemcpyDeviceToHost);
        else
            std::memset(worker_scales, 0, nb * sizeof(float));
    }
    if (e == hipSuccess && server_scales) {
        if (c->server_comp == kBlockSign)
            e = hipMemcpy(server_scales, c->blk_scales + nb, (size_t)c->B * sizeof(float), hipMemcpyDeviceToHost);
        else
            std::memset(server_scales, 0, (size_t)c->B * sizeof(float));
    }
    if (e != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

int64_t liec_message_bytes(liec_comp comp, int64_t d, int64_t k, int32_t nblocks) {
    if (d < 1) return -1;
    switch (comp) {
    case LIEC_COMP_IDENTITY: return 4 * d;
    case LIEC_COMP_SIGN: return (d + 7) / 8 + 4;
    case LIEC_COMP_BLOCKSIGN: return nblocks < 1 ? -1 : (d + 7) / 8 + 4 * (int64_t)nblocks;
    case LIEC_COMP_TOPK: return (k < 1 || k > d) ? -1 : 8 * k;
    case LIEC_COMP_RANDK: return (k < 1 || k > d) ? -1 : 8 * k;
    default: return -1;
    }
}

liec_status liec_comm_cost(int32_t N, int64_t d, liec_comp worker_comp, int64_t worker_k, liec_comp server_comp,
                           int64_t server_k, int32_t nblocks, int32_t period, int32_t count_model_exchange,
                           double* bytes_per_iteration) {
    if (!bytes_per_iteration || N < 1 || period < 0 || period == 1) return LIEC_EINVAL;
    const int64_t up = liec_message_bytes(worker_comp, d, worker_k, nblocks);
    const int64_t down = liec_message_bytes(server_comp, d, server_k, nblocks);
    if (up < 0 || down < 0) return LIEC_EINVAL;
    const double compressed = (double)N * ((double)up + (double)down);
    if (period == 0) {
        *bytes_per_iteration = compressed;
        return LIEC_OK;
    }
    const double full = 4.0 * (double)d;
    const double averaging = (double)N * (2.0 * full) + (count_model_exchange ? (double)N * (2.0 * full) : 0.0);
    *bytes_per_iteration = ((double)(period - 1) * compressed + averaging) / (double)period;
    return LIEC_OK;
}

liec_status liec_pack_sign_bits(liec_ctx* c, int32_t worker, uint8_t* out) {
    if (!c || !out || worker < 0 || worker >= c->N) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    if ((c->worker_comp != kSign && c->worker_comp != kBlockSign) || c->steps_done == 0) return LIEC_EINVAL;
    const uint32_t nbytes = (uint32_t)((c->d + 7) / 8);
    k_pack_sign<<<(nbytes + kBlock - 1) / kBlock, kBlock, 0, c->stream>>>(c->bits + (size_t)worker * c->nwt * 64, nbytes, out);
    if (hipGetLastError() != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_unpack_sign_message(liec_ctx* c, const uint8_t* bits, const float* scales, int32_t blockwise,
                                     float* p_out) {
    if (!c || !bits || !scales || !p_out) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    if (blockwise && c->B == 0) return LIEC_EINVAL;
    // Definition 4 has one scale: it travels as a kernel argument, and nothing is copied or waited for.
    // Definition 5's table of scales is copied to the device first.
    const float scale0 = scales[0];
    if (blockwise) {
        const uint32_t n = c->B;
        hipError_t e = hipSuccess;
        if (c->wire_scales_len < n) {
            e = hipStreamSynchronize(c->stream);
            (void)hipFree(c->wire_scales);
            c->wire_scales = nullptr;
            c->wire_scales_len = 0;
            if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->wire_scales), (size_t)n * sizeof(float));
            if (e == hipSuccess) c->wire_scales_len = n;
        }
        if (e == hipSuccess)
            e = hipMemcpyAsync(c->wire_scales, scales, (size_t)n * sizeof(float), hipMemcpyHostToDevice, c->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(c->stream);    // the host array may be reused on return
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return e == hipErrorOutOfMemory ? LIEC_ENOMEM : LIEC_EDEVICE;
        }
    }
    BlockTable bt = block_table(c);
    if (!blockwise) bt.B = 0;
    const uint32_t d = (uint32_t)c->d;
    const uint32_t nq = (d + 3) / 4, grid = std::min<uint32_t>((nq + kBlock - 1) / kBlock, 16384u);
    if (d % 4 == 0 && ((uintptr_t)p_out & 15u) == 0)
        k_unpack_sign<true><<<grid, kBlock, 0, c->stream>>>(bits, d, c->wire_scales, scale0, bt, p_out);
    else
        k_unpack_sign<false><<<grid, kBlock, 0, c->stream>>>(bits, d, c->wire_scales, scale0, bt, p_out);
    if (hipGetLastError() != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_pack_topk_message(liec_ctx* c, const float* grads, int32_t worker, uint32_t* idx_out, float* val_out) {
    if (!c || !grads || !idx_out || !val_out || worker < 0 || worker >= c->N) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    if (!selects_k(c->worker_comp) || c->steps_done == 0 || ((uintptr_t)grads & 3u)) return LIEC_EINVAL;
    if (!c->wire_tiles) {
        if (hipStreamSynchronize(c->stream) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&c->wire_tiles), ((size_t)c->nwt + 1) * sizeof(uint32_t)) != hipSuccess) {
            (void)hipGetLastError();
            c->wire_tiles = nullptr;
            return LIEC_ENOMEM;
        }
    }
    const uint32_t d = (uint32_t)c->d, k = (uint32_t)c->worker_k;
    const float* row = grads + (size_t)worker * (size_t)c->d;
    const bool vec = (c->d % 4 == 0) && (((uintptr_t)grads & 15u) == 0);
    const RowDesc* rd = c->desc + worker;
    // random-k: the kept set of the last draw is the worker's row of the kept bitmap
    const uint16_t* kept = c->worker_comp == kRandk ? c->bits + (size_t)worker * c->nwt * 64 : nullptr;
    const uint32_t blocks = c->agg_blocks;
    if (vec) k_topk_count<true><<<blocks, kBlock, 0, c->stream>>>(row, d, c->nwt, rd, kept, c->wire_tiles);
    else k_topk_count<false><<<blocks, kBlock, 0, c->stream>>>(row, d, c->nwt, rd, kept, c->wire_tiles);
    k_scan_u32<<<1, 1024, 0, c->stream>>>(c->wire_tiles, c->nwt, c->wire_tiles + c->nwt);
    if (vec) k_topk_emit<true><<<blocks, kBlock, 0, c->stream>>>(row, d, c->nwt, rd, kept, c->wire_tiles, k, idx_out, val_out);
    else k_topk_emit<false><<<blocks, kBlock, 0, c->stream>>>(row, d, c->nwt, rd, kept, c->wire_tiles, k, idx_out, val_out);
    if (hipGetLastError() != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_unpack_topk_message(liec_ctx* c, const uint32_t* idx, const float* val, int64_t k, float* p_out) {
    if (!c || !idx || !val || !p_out || k < 0 || k > c->d) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    const uint32_t d = (uint32_t)c->d;
    k_fill_f32<<<std::min<uint32_t>((d + kBlock - 1) / kBlock, 8192u), kBlock, 0, c->stream>>>(p_out, d, 0.f);
    if (k > 0)
        k_scatter_pairs<<<((uint32_t)k + kBlock - 1) / kBlock, kBlock, 0, c->stream>>>(idx, val, (uint32_t)k, d, p_out);
    if (hipGetLastError() != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    return LIEC_OK;
}

liec_status liec_l2_norm(liec_ctx* c, const float* vec, int64_t n, double* norm_out) {
    if (!c || !vec || !norm_out || n < 1 || ((uintptr_t)vec & 3u)) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    // s_partial holds agg_blocks doubles; one more double behind the worker partials receives the sum
    const uint32_t blocks = (uint32_t)std::min<int64_t>((n + kBlock - 1) / kBlock, (int64_t)std::min<uint32_t>(c->agg_blocks, 4096u));
    k_sumsq<<<blocks, kBlock, 0, c->stream>>>(vec, (uint64_t)n, c->s_partial);
    k_sumsq_final<<<1, kBlock, 0, c->stream>>>(c->s_partial, blocks, c->w_partial, false);
    double sum = 0.0;
    if (hipGetLastError() != hipSuccess ||
        hipMemcpyAsync(&sum, c->w_partial, sizeof sum, hipMemcpyDeviceToHost, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    *norm_out = std::sqrt(sum);
    return LIEC_OK;
}

liec_status liec_l2_norm_static(const float* vec, int64_t n, double* norm_out, void* hip_stream) {
    if (!vec || !norm_out || n < 1 || n > LIEC_L2_STATIC_MAX_N) return LIEC_EINVAL;
    if (((uintptr_t)vec & 3u) || ((uintptr_t)norm_out & 7u)) return LIEC_EINVAL;
    double* partial = nullptr;                                  // this device's copy of `scratch`
    if (static_scratch(&partial) != hipSuccess) {
        (void)hipGetLastError();
        return LIEC_EDEVICE;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    // every partial the second kernel reads is written by the first: nothing of an earlier call survives
    const uint32_t blocks = (uint32_t)std::min<int64_t>((n + kBlock - 1) / kBlock, (int64_t)kL2StaticBlocks);
    k_sumsq<<<blocks, kBlock, 0, st>>>(vec, (uint64_t)n, partial);
    k_sumsq_final<<<1, kBlock, 0, st>>>(partial, blocks, norm_out, true);
    return hipGetLastError() == hipSuccess ? LIEC_OK : LIEC_EDEVICE;
}

liec_status liec_set_lr(liec_ctx* c, float lr) {
    if (!c || !finite_f(lr)) return LIEC_EINVAL;
    c->lr = lr;
    return LIEC_OK;
}

liec_status liec_get_info(liec_ctx* c, liec_info* info) {
    if (!c || !info) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    std::vector<RowDesc> h((size_t)c->N + 1);
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(h.data(), c->desc, h.size() * sizeof(RowDesc), hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    std::memset(info, 0, sizeof *info);
    info->N = c->N;
    info->d = c->d;
    info->worker_comp = c->worker_comp;
    info->server_comp = c->server_comp;
    info->worker_k = c->worker_k;
    info->server_k = c->server_k;
    info->lr = c->lr;
    info->steps_done = c->steps_done;
    const RowDesc& s = h[(size_t)c->N];
    if (c->server_comp == kSign) {
        info->server_scale = s.scale;
        info->server_l1 = s.l1;
    } else if (selects_k(c->server_comp)) {
        info->server_tau_key = s.tau;
        info->server_cutoff = (int64_t)s.cutoff;
    }
    for (size_t r = 0; r < h.size(); ++r) {
        if (!selects_k(r < (size_t)c->N ? c->worker_comp : c->server_comp)) continue;
        if (h[r].dense) ++info->slow_rows;
        info->band_misses += (int64_t)h[r].misses;
    }
    bool bad = (c->server_comp == kSign || c->server_comp == kTopk) && s.nonfinite;
    if (c->worker_comp == kSign || c->worker_comp == kTopk)
        for (int32_t i = 0; i < c->N; ++i) bad = bad || h[(size_t)i].nonfinite;
    if ((c->worker_comp == kBlockSign || c->server_comp == kBlockSign) && c->B) {
        std::vector<double> l1((size_t)(c->N + 1) * c->B);
        if (hipMemcpy(l1.data(), c->blk_l1, l1.size() * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess) {
            c->broken = true;
            return LIEC_EDEVICE;
        }
        const size_t nb = (size_t)c->N * c->B;
        for (size_t q = 0; q < l1.size(); ++q) {
            const bool used = q < nb ? c->worker_comp == kBlockSign : c->server_comp == kBlockSign;
            if (used && !std::isfinite(l1[q])) bad = true;
        }
    }
    info->nonfinite = bad ? 1 : 0;
    return bad ? LIEC_ENONFINITE : LIEC_OK;
}

liec_status liec_get_worker_desc(liec_ctx* c, float* scales, double* l1, uint32_t* tau, int64_t* cutoff) {
    if (!c) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    std::vector<RowDesc> h((size_t)c->N);
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(h.data(), c->desc, h.size() * sizeof(RowDesc), hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    for (int32_t i = 0; i < c->N; ++i) {
        const RowDesc& r = h[(size_t)i];
        const bool sg = c->worker_comp == kSign, tk = selects_k(c->worker_comp);
        if (scales) scales[i] = sg ? r.scale : 0.f;
        if (l1) l1[i] = sg ? r.l1 : 0.0;
        if (tau) tau[i] = tk ? r.tau : 0u;
        if (cutoff) cutoff[i] = tk ? (int64_t)r.cutoff : 0;
    }
    return LIEC_OK;
}

liec_status liec_profile_begin(liec_ctx* c, int32_t max_steps, int32_t update_only) {
    if (!c || max_steps < 1) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    drop_prof(c);
    c->profiling = true;
    c->prof_update_only = update_only != 0;
    c->prof_steps_left = max_steps;
    return LIEC_OK;
}

liec_status liec_profile_end(liec_ctx* c, int32_t* n_slots, const char** names, double* total_ms,
                             int64_t* launches) {
    if (!c || !n_slots || !names || !total_ms || !launches) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    DeviceScope on(c);
    if (!on.ok) return LIEC_EDEVICE;
    c->profiling = false;
    if (hipStreamSynchronize(c->stream) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    double ms[S_COUNT] = {0};
    int64_t cnt[S_COUNT] = {0};
    bool ok = true;
    for (auto& ev : c->prof) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, ev.start, ev.stop) != hipSuccess) ok = false;
        ms[ev.slot] += (double)t;
        ++cnt[ev.slot];
    }
    drop_prof(c);
    if (!ok) return LIEC_EDEVICE;
    int32_t used = 0;
    for (int s = 0; s < S_COUNT; ++s) {
        if (!cnt[s]) continue;
        if (used >= *n_slots) return LIEC_EINVAL;
        names[used] = slot_name(s);
        total_ms[used] = ms[s];
        launches[used] = cnt[s];
        ++used;
    }
    *n_slots = used;
    return LIEC_OK;
}

void liec_destroy(liec_ctx* c) {
    if (!c) return;
    DeviceScope on(c);
    (void)hipStreamSynchronize(c->stream);
    drop_prof(c);
    free_scratch(c);
    delete c;
}

int64_t liec_scratch_bytes(const liec_ctx* c) { return c ? c->scratch_bytes : 0; }

liec_status liec_device_copy(void* dst, const void* src, int64_t bytes, void* hip_stream) {
    if (!dst || !src || bytes < 0 || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15u)) return LIEC_EINVAL;
    if (bytes == 0) return LIEC_OK;
    const size_t n16 = (size_t)bytes / 16;
    const size_t blocks = (n16 + kBlock - 1) / kBlock;
    if (blocks >= ((size_t)1 << 31)) return LIEC_EINVAL;           // 512 GiB per call is plenty
    k_copy16<<<(uint32_t)blocks, kBlock, 0, (hipStream_t)hip_stream>>>((const v4f*)src, (v4f*)dst, n16);
    return hipGetLastError() == hipSuccess ? LIEC_OK : LIEC_EDEVICE;
}

}  // extern "C"
