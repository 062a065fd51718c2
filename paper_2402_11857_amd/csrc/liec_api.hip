// Host side of the C ABI declared in include/liec.h: argument checks, scratch ownership and
// the launch sequence of one compressed LIEC-SGD iteration (Algorithm 1) on a HIP stream.
#include "liec.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "liec_kernels.hpp"

using namespace liec;

namespace {

constexpr int kMaxSlots = 24;

enum Slot : int {
    S_W_L1 = 0, S_W_L1_FINAL, S_W_HIST0, S_W_PICK0, S_W_HIST1, S_W_PICK1, S_W_HIST2, S_W_PICK2,
    S_W_TIE_COUNT, S_W_TIE_PICK, S_AGGREGATE, S_S_L1_FINAL, S_S_HIST0, S_S_PICK0, S_S_HIST1,
    S_S_PICK1, S_S_HIST2, S_S_PICK2, S_S_TIE_COUNT, S_S_TIE_PICK, S_UPDATE, S_COUNT
};
static_assert(S_COUNT <= kMaxSlots, "slot table too small");

const char* const kSlotNames[S_COUNT] = {
    "worker_l1_bits", "worker_l1_final", "worker_hist0", "worker_pick0", "worker_hist1", "worker_pick1",
    "worker_hist2", "worker_pick2", "worker_tie_count", "worker_tie_pick", "server_aggregate",
    "server_l1_final", "server_hist0", "server_pick0", "server_hist1", "server_pick1", "server_hist2",
    "server_pick2", "server_tie_count", "server_tie_pick", "update"};

struct ProfEvent {
    hipEvent_t start, stop;
    int slot;
};

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

    uint32_t ntiles = 0, nchunks = 0;
    uint32_t row_blocks = 0, row_tpb = 0;      // per-row kernels over grads: grid (row_blocks, N)
    uint32_t srv_blocks = 0, srv_tpb = 0;      // kernels over one length-d vector

    // device scratch
    RowDesc* desc = nullptr;                   // [N + 1]
    double* w_partial = nullptr;               // [N * row_blocks]
    double* s_partial = nullptr;               // [srv_blocks]
    uint64_t* bits = nullptr;                  // [N * nchunks * 4]
    uint32_t* hist = nullptr;                  // [(N + 1) * kHistBins]
    uint32_t* w_cnt = nullptr;                 // [N * row_blocks]
    uint32_t* s_cnt = nullptr;                 // [srv_blocks]
    int64_t scratch_bytes = 0;

    // profiling
    bool profiling = false;
    int32_t prof_steps_left = 0;
    std::vector<ProfEvent> prof;
};

namespace {

bool finite_f(float v) { return std::isfinite(v); }

template <typename T>
hipError_t dev_alloc(liec_ctx* c, T** p, size_t count) {
    const size_t bytes = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes);
    if (e == hipSuccess) c->scratch_bytes += (int64_t)bytes;
    return e;
}

void free_scratch(liec_ctx* c) {
    (void)hipFree(c->desc);
    (void)hipFree(c->w_partial);
    (void)hipFree(c->s_partial);
    (void)hipFree(c->bits);
    (void)hipFree(c->hist);
    (void)hipFree(c->w_cnt);
    (void)hipFree(c->s_cnt);
}

bool valid_comp(int c) { return c == LIEC_COMP_IDENTITY || c == LIEC_COMP_SIGN || c == LIEC_COMP_TOPK; }

struct Launcher {
    liec_ctx* c;
    bool ok = true;
    void begin(int slot) {
        if (!c->profiling) return;
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
        if (!c->profiling || c->prof.empty()) return;
        if (hipEventRecord(c->prof.back().stop, c->stream) != hipSuccess) ok = false;
    }
};

// Radix select of the rank-k magnitude in each of `rows` rows of `src` (Definition 2), leaving
// tau / rank / cutoff in desc[0..rows).  Four passes over the data: three digits, then the tie order.
template <bool VEC>
void launch_topk_select(Launcher& L, const float* src, size_t row_stride, uint32_t rows, uint32_t d,
                        uint32_t ntiles, uint32_t blocks, uint32_t tpb, uint32_t k, RowDesc* desc,
                        uint32_t* hist, uint32_t* cnt, int slot0) {
    liec_ctx* c = L.c;
    const dim3 grid(blocks, rows);
    L.begin(slot0 + 0);
    k_hist<VEC><<<grid, kBlock, 0, c->stream>>>(src, row_stride, d, ntiles, tpb, desc, 0, hist);
    L.end();
    L.begin(slot0 + 1);
    k_pick<0><<<rows, kBlock, 0, c->stream>>>(desc, hist, k);
    L.end();
    L.begin(slot0 + 2);
    k_hist<VEC><<<grid, kBlock, 0, c->stream>>>(src, row_stride, d, ntiles, tpb, desc, 1, hist);
    L.end();
    L.begin(slot0 + 3);
    k_pick<1><<<rows, kBlock, 0, c->stream>>>(desc, hist, k);
    L.end();
    L.begin(slot0 + 4);
    k_hist<VEC><<<grid, kBlock, 0, c->stream>>>(src, row_stride, d, ntiles, tpb, desc, 2, hist);
    L.end();
    L.begin(slot0 + 5);
    k_pick<2><<<rows, kBlock, 0, c->stream>>>(desc, hist, k);
    L.end();
    L.begin(slot0 + 6);
    k_tie_count<VEC><<<grid, kBlock, 0, c->stream>>>(src, row_stride, d, ntiles, tpb, desc, cnt);
    L.end();
    L.begin(slot0 + 7);
    k_tie_pick<VEC><<<rows, kBlock, 0, c->stream>>>(src, row_stride, d, ntiles, tpb, blocks, desc, cnt);
    L.end();
}

template <int WC, bool VEC>
void launch_aggregate(Launcher& L, const float* grads, float* e, bool srv_l1) {
    liec_ctx* c = L.c;
    const float inv_n = 1.0f / (float)c->N;
    const uint32_t d = (uint32_t)c->d;
    L.begin(S_AGGREGATE);
    if (WC == kSign) {
        if (srv_l1)
            k_aggregate<kSign, true, true, VEC><<<c->srv_blocks, kBlock, 0, c->stream>>>(
                grads, c->bits, c->nchunks, c->N, d, c->ntiles, c->srv_tpb, inv_n, c->desc, e, c->s_partial);
        else
            k_aggregate<kSign, true, false, VEC><<<c->srv_blocks, kBlock, 0, c->stream>>>(
                grads, c->bits, c->nchunks, c->N, d, c->ntiles, c->srv_tpb, inv_n, c->desc, e, c->s_partial);
    } else {
        if (srv_l1)
            k_aggregate<WC, false, true, VEC><<<c->srv_blocks, kBlock, 0, c->stream>>>(
                grads, c->bits, c->nchunks, c->N, d, c->ntiles, c->srv_tpb, inv_n, c->desc, e, c->s_partial);
        else
            k_aggregate<WC, false, false, VEC><<<c->srv_blocks, kBlock, 0, c->stream>>>(
                grads, c->bits, c->nchunks, c->N, d, c->ntiles, c->srv_tpb, inv_n, c->desc, e, c->s_partial);
    }
    L.end();
}

template <int WC, int SC, bool VEC>
void launch_update(Launcher& L, const float* grads, float* x, float* e) {
    liec_ctx* c = L.c;
    L.begin(S_UPDATE);
    k_update<WC, SC, VEC><<<c->ntiles, kBlock, 0, c->stream>>>(grads, x, e, c->N, (uint32_t)c->d, -c->lr, c->desc);
    L.end();
}

template <int WC, bool VEC>
void launch_update_sc(Launcher& L, int sc, const float* grads, float* x, float* e) {
    switch (sc) {
    case kIdentity: launch_update<WC, kIdentity, VEC>(L, grads, x, e); break;
    case kSign: launch_update<WC, kSign, VEC>(L, grads, x, e); break;
    default: launch_update<WC, kTopk, VEC>(L, grads, x, e); break;
    }
}

template <bool VEC>
void run_step(Launcher& L, const float* grads, float* x, float* e) {
    liec_ctx* c = L.c;
    const uint32_t d = (uint32_t)c->d;
    const size_t stride = (size_t)c->d;

    // ---- workers: p^i = C_w(g_i), reduced to a per-row descriptor --------------------------------
    if (c->worker_comp == kSign) {
        L.begin(S_W_L1);
        k_l1_bits<VEC><<<dim3(c->row_blocks, c->N), kBlock, 0, c->stream>>>(
            grads, stride, d, c->ntiles, c->row_tpb, c->w_partial, c->bits, c->nchunks);
        L.end();
        L.begin(S_W_L1_FINAL);
        k_l1_final<<<c->N, kBlock, 0, c->stream>>>(c->w_partial, c->row_blocks, d, c->desc);
        L.end();
    } else if (c->worker_comp == kTopk) {
        launch_topk_select<VEC>(L, grads, stride, (uint32_t)c->N, d, c->ntiles, c->row_blocks, c->row_tpb,
                                (uint32_t)c->worker_k, c->desc, c->hist, c->w_cnt, S_W_HIST0);
    }

    // ---- server: v = e + mean_i p^i (in place over e), then the descriptor of C_s(v) -------------
    const bool srv_l1 = c->server_comp == kSign;
    switch (c->worker_comp) {
    case kIdentity: launch_aggregate<kIdentity, VEC>(L, grads, e, srv_l1); break;
    case kSign: launch_aggregate<kSign, VEC>(L, grads, e, srv_l1); break;
    default: launch_aggregate<kTopk, VEC>(L, grads, e, srv_l1); break;
    }
    if (c->server_comp == kSign) {
        L.begin(S_S_L1_FINAL);
        k_l1_final<<<1, kBlock, 0, c->stream>>>(c->s_partial, c->srv_blocks, d, c->desc + c->N);
        L.end();
    } else if (c->server_comp == kTopk) {
        launch_topk_select<VEC>(L, e, 0, 1u, d, c->ntiles, c->srv_blocks, c->srv_tpb, (uint32_t)c->server_k,
                                c->desc + c->N, c->hist + (size_t)c->N * kHistBins, c->s_cnt, S_S_HIST0);
    }

    // ---- p = C_s(v), e <- v - p, x^i <- x^i - lr (p + (g_i - p^i)) ---------------------------------
    switch (c->worker_comp) {
    case kIdentity: launch_update_sc<kIdentity, VEC>(L, c->server_comp, grads, x, e); break;
    case kSign: launch_update_sc<kSign, VEC>(L, c->server_comp, grads, x, e); break;
    default: launch_update_sc<kTopk, VEC>(L, c->server_comp, grads, x, e); break;
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
    if (N < 1 || d < 1 || d >= ((int64_t)1 << 31) - ((int64_t)1 << 20)) return LIEC_EINVAL;
    if (!valid_comp((int)worker_comp) || !valid_comp((int)server_comp) || !finite_f(lr)) return LIEC_EINVAL;
    if (worker_comp == LIEC_COMP_TOPK && (worker_k < 1 || worker_k > d)) return LIEC_EINVAL;
    if (server_comp == LIEC_COMP_TOPK && (server_k < 1 || server_k > d)) return LIEC_EINVAL;

    liec_ctx* c = new (std::nothrow) liec_ctx();
    if (!c) return LIEC_ENOMEM;
    c->N = N;
    c->d = d;
    c->worker_comp = (int)worker_comp;
    c->server_comp = (int)server_comp;
    c->worker_k = worker_comp == LIEC_COMP_TOPK ? worker_k : 0;
    c->server_k = server_comp == LIEC_COMP_TOPK ? server_k : 0;
    c->lr = lr;
    c->stream = (hipStream_t)hip_stream;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return LIEC_EDEVICE;
    }

    c->ntiles = (uint32_t)((d + kTile - 1) / kTile);
    c->nchunks = (uint32_t)((d + kChunk - 1) / kChunk);
    // Per-row kernels: aim at about 4096 blocks over all rows, at least 4 tiles per block.
    uint32_t want = 4096u / (uint32_t)N;
    if (want < 1) want = 1;
    c->row_tpb = (c->ntiles + want - 1) / want;
    if (c->row_tpb < 4) c->row_tpb = 4;
    c->row_blocks = (c->ntiles + c->row_tpb - 1) / c->row_tpb;
    c->srv_tpb = (c->ntiles + 4095u) / 4096u;
    if (c->srv_tpb < 1) c->srv_tpb = 1;
    c->srv_blocks = (c->ntiles + c->srv_tpb - 1) / c->srv_tpb;

    hipError_t e = dev_alloc(c, &c->desc, (size_t)N + 1);
    if (e == hipSuccess) e = dev_alloc(c, &c->w_partial, (size_t)N * c->row_blocks);
    if (e == hipSuccess) e = dev_alloc(c, &c->s_partial, (size_t)c->srv_blocks);
    if (e == hipSuccess && worker_comp == LIEC_COMP_SIGN) e = dev_alloc(c, &c->bits, (size_t)N * c->nchunks * 4);
    if (e == hipSuccess) e = dev_alloc(c, &c->hist, ((size_t)N + 1) * kHistBins);
    if (e == hipSuccess) e = dev_alloc(c, &c->w_cnt, (size_t)N * c->row_blocks);
    if (e == hipSuccess) e = dev_alloc(c, &c->s_cnt, (size_t)c->srv_blocks);
    if (e == hipSuccess) e = hipMemsetAsync(c->desc, 0, ((size_t)N + 1) * sizeof(RowDesc), c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->hist, 0, ((size_t)N + 1) * kHistBins * sizeof(uint32_t), c->stream);
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
    const size_t nd = (size_t)c->N * (size_t)c->d * sizeof(float), db = (size_t)c->d * sizeof(float);
    if (overlap(grads, nd, x, nd) || overlap(grads, nd, server_err, db) || overlap(x, nd, server_err, db))
        return LIEC_EINVAL;
    if (((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 3u) return LIEC_EINVAL;
    const bool vec = (c->d % 4 == 0) && ((((uintptr_t)grads | (uintptr_t)x | (uintptr_t)server_err) & 15u) == 0);

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

liec_status liec_set_lr(liec_ctx* c, float lr) {
    if (!c || !finite_f(lr)) return LIEC_EINVAL;
    c->lr = lr;
    return LIEC_OK;
}

liec_status liec_get_info(liec_ctx* c, liec_info* info) {
    if (!c || !info) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
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
    } else if (c->server_comp == kTopk) {
        info->server_tau_key = s.tau;
        info->server_cutoff = (int64_t)s.cutoff;
    }
    bool bad = c->server_comp != kIdentity && s.nonfinite;
    if (c->worker_comp != kIdentity)
        for (int32_t i = 0; i < c->N; ++i) bad = bad || h[(size_t)i].nonfinite;
    info->nonfinite = bad ? 1 : 0;
    return bad ? LIEC_ENONFINITE : LIEC_OK;
}

liec_status liec_get_worker_desc(liec_ctx* c, float* scales, double* l1, uint32_t* tau, int64_t* cutoff) {
    if (!c) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    std::vector<RowDesc> h((size_t)c->N);
    if (hipStreamSynchronize(c->stream) != hipSuccess ||
        hipMemcpy(h.data(), c->desc, h.size() * sizeof(RowDesc), hipMemcpyDeviceToHost) != hipSuccess) {
        c->broken = true;
        return LIEC_EDEVICE;
    }
    for (int32_t i = 0; i < c->N; ++i) {
        const RowDesc& r = h[(size_t)i];
        const bool sg = c->worker_comp == kSign, tk = c->worker_comp == kTopk;
        if (scales) scales[i] = sg ? r.scale : 0.f;
        if (l1) l1[i] = sg ? r.l1 : 0.0;
        if (tau) tau[i] = tk ? r.tau : 0u;
        if (cutoff) cutoff[i] = tk ? (int64_t)r.cutoff : 0;
    }
    return LIEC_OK;
}

liec_status liec_profile_begin(liec_ctx* c, int32_t max_steps) {
    if (!c || max_steps < 1) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
    drop_prof(c);
    c->profiling = true;
    c->prof_steps_left = max_steps;
    return LIEC_OK;
}

liec_status liec_profile_end(liec_ctx* c, int32_t* n_slots, const char** names, double* total_ms,
                             int64_t* launches) {
    if (!c || !n_slots || !names || !total_ms || !launches) return LIEC_EINVAL;
    if (c->broken) return LIEC_EDEVICE;
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
        names[used] = kSlotNames[s];
        total_ms[used] = ms[s];
        launches[used] = cnt[s];
        ++used;
    }
    *n_slots = used;
    return LIEC_OK;
}

void liec_destroy(liec_ctx* c) {
    if (!c) return;
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
    size_t blocks = (n16 + kBlock - 1) / kBlock;
    if (blocks > 256u * 32u) blocks = 256u * 32u;
    k_copy16<<<(uint32_t)blocks, kBlock, 0, (hipStream_t)hip_stream>>>((const uint4*)src, (uint4*)dst, n16);
    return hipGetLastError() == hipSuccess ? LIEC_OK : LIEC_EDEVICE;
}

}  // extern "C"
