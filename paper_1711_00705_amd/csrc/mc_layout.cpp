// Host side of the layout: flat offsets, colour bounds, pack-tile table, options, errors.
// Nothing in this file touches the GPU.
#include <algorithm>
#include <atomic>
#include <new>

#include "mc_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

std::atomic<int> g_ru_shape{0};
std::atomic<int> g_state_policy{MC_STATE_RESIDENT};
std::atomic<int> g_pack_nontemporal{3};
std::atomic<int> g_state_store_sc1{1};
std::atomic<int> g_alternate_sweep{1};
std::atomic<int> g_xcd_run{0};
std::atomic<int> g_xcd_run_pack{-1};
std::atomic<int> g_xcd_run_unpack{0};
std::atomic<int> g_direct_tiles{1};
std::atomic<int> g_lds_cap_update{-1};
std::atomic<int> g_lds_cap_pack{0};

// Capacity of the memory-side cache that sits between the L2s and HBM.
constexpr int64_t kMemorySideCacheBytes = int64_t(256) << 20;

}  // namespace

namespace mc {

int hip_fail(hipError_t e) {
    g_last_hip_error = static_cast<int>(e);
    return MC_ERR_HIP;
}

Shape shape_for(int64_t elems, int n_terms, bool stream_state) {
    const int forced = g_ru_shape.load(std::memory_order_relaxed);
    if (forced == 1) return Shape{64, 1};
    if (forced == 2) return Shape{256, 2};
    (void)elems;
    (void)n_terms;
    (void)stream_state;
    return Shape{64, 1};
}

unsigned lds_reservation(int which, int threads) {
    int v = (which == MC_OPT_LDS_CAP_PACK ? g_lds_cap_pack : g_lds_cap_update).load(std::memory_order_relaxed);
    // automatic: 16 wavefronts per compute unit (10 KB of the 160 KB per wavefront of the workgroup)
    if (v < 0) v = 10240 * (threads / 64);
    return unsigned(v);
}

unsigned update_lds_reservation(const mc_layout* L, int threads, bool state_cached, int terms, bool per_layer) {
    const int v = g_lds_cap_update.load(std::memory_order_relaxed);
    if (v >= 0) return unsigned(v);
    // automatic.  Weights and momentum expected in the memory-side cache (every colour updates, resident
    // policy, state that fits): no cap.  Otherwise (nearly) every stream of a tile comes from HBM, and
    // what the step wants is a fixed amount of loads in flight per compute unit -- about 84 KB for the
    // fused step, 72 KB when the state exceeds the cache or the buffers are flat (no per-layer lookups
    // in front of the loads) -- so the number of wavefronts follows from the (terms + 2) KB each of
    // them keeps in flight.
    // (A launch whose colours differ in term count or update flag runs the general kernel, which sits
    // on a longer chain of argument fetches: 16 wavefronts measured best for it, 10 lose 10 %.)
    if (terms <= 0) return unsigned(10240 * (threads / 64));
    const bool big = L->N * 8 > kMemorySideCacheBytes;
    // (More than eight contributions run the run-time loop, which keeps the state and at most four
    // terms in flight at a time whatever the count; with the state cached it measured 5-6 % faster at 16
    // wavefronts than uncapped.)
    if (!big && state_cached) return terms > 8 ? unsigned(10240 * (threads / 64)) : 0u;
    const int kb = (big || !per_layer) ? 72 : 84;
    const int in_flight = terms > 8 ? 4 : terms;
    int waves = (kb + (in_flight + 2) / 2) / (in_flight + 2);
    if (waves < 4) waves = 4;
    if (waves >= 32) return 0;
    const int per_wave = (160 * 1024 / waves) / 1024 * 1024;   // LDS of a compute unit / wavefronts, in whole KB
    const int bytes = per_wave * (threads / 64);
    return unsigned(bytes < 65536 ? bytes : 65536);   // (64 KB is the most a launch may ask for)
}

bool stream_state(const mc_layout* L, int policy) {
    (void)L;
    if (policy == MC_STATE_DEFAULT) policy = g_state_policy.load(std::memory_order_relaxed);
    return policy == MC_STATE_STREAMING;
}

bool sweep_reversed(const mc_layout* L, int sweep, bool stream_state) {
    if (sweep == MC_SWEEP_FORWARD) return false;
    if (sweep == MC_SWEEP_BACKWARD) return true;
    if (!g_alternate_sweep.load(std::memory_order_relaxed)) return false;
    // Only resident state that cannot all stay in the cache gains from alternating; while it fits,
    // a fixed direction measured 1-2 % faster, and streamed state leaves nothing behind to reuse.
    if (stream_state || L->N * 8 <= kMemorySideCacheBytes) return false;
    return (L->sweep.fetch_add(1, std::memory_order_relaxed) & 1u) != 0;
}

int option(int which) {
    switch (which) {
        case MC_OPT_RU_SHAPE: return g_ru_shape.load(std::memory_order_relaxed);
        case MC_OPT_STATE_POLICY: return g_state_policy.load(std::memory_order_relaxed);
        case MC_OPT_PACK_NONTEMPORAL: return g_pack_nontemporal.load(std::memory_order_relaxed);
        case MC_OPT_STATE_STORE_SC1: return g_state_store_sc1.load(std::memory_order_relaxed);
        case MC_OPT_ALTERNATE_SWEEP: return g_alternate_sweep.load(std::memory_order_relaxed);
        case MC_OPT_XCD_RUN: return g_xcd_run.load(std::memory_order_relaxed);
        case MC_OPT_XCD_RUN_PACK: return g_xcd_run_pack.load(std::memory_order_relaxed);
        case MC_OPT_XCD_RUN_UNPACK: return g_xcd_run_unpack.load(std::memory_order_relaxed);
        case MC_OPT_DIRECT_TILES: return g_direct_tiles.load(std::memory_order_relaxed);
        case MC_OPT_LDS_CAP_UPDATE: return g_lds_cap_update.load(std::memory_order_relaxed);
        case MC_OPT_LDS_CAP_PACK: return g_lds_cap_pack.load(std::memory_order_relaxed);
        default: return kNoSuchOption;
    }
}

}  // namespace mc

extern "C" {

int mc_layout_create(const int64_t* numel, int32_t n_tensors, int32_t k_colours, mc_layout** out) {
    if (out) *out = nullptr;
    if (!numel || !out || n_tensors < 1 || k_colours < 1) return MC_ERR_INVALID_ARG;
    constexpr int64_t kMaxTotal = int64_t(1) << 40;
    int64_t total = 0;
    for (int32_t t = 0; t < n_tensors; ++t) {
        if (numel[t] < 0 || numel[t] > kMaxTotal) return MC_ERR_INVALID_ARG;
        total += numel[t];
        if (total > kMaxTotal) return MC_ERR_INVALID_ARG;
    }
    mc_layout* L = new (std::nothrow) mc_layout;
    if (!L) return MC_ERR_ALLOC;
    try {
        L->n = n_tensors;
        L->k = k_colours;
        L->N = total;
        L->off.resize(size_t(n_tensors) + 1);
        L->off[0] = 0;
        for (int32_t t = 0; t < n_tensors; ++t) L->off[t + 1] = L->off[t] + numel[t];

        // Section 4.2: k contiguous chunks.  Equal length C (a multiple of 256 elements so that
        // every colour starts on a 1 KiB boundary), the last non-empty one shorter.
        const int64_t a = MC_COLOUR_ALIGN_ELEMS;
        int64_t C = total / k_colours + (total % k_colours != 0);
        C = (C + a - 1) / a * a;
        L->chunk = C;
        L->bounds.resize(size_t(k_colours) + 1);
        for (int32_t c = 0; c <= k_colours; ++c) {
            const bool past_end = C == 0 || int64_t(c) >= (total + C - 1) / C;
            L->bounds[c] = past_end ? total : int64_t(c) * C;
        }

        // For each run of kLookupElems flat elements, the first tensor whose range ends after
        // the run's first element.
        const int64_t tiles = (total + mc::kLookupElems - 1) / mc::kLookupElems;
        L->tile_first.resize(size_t(tiles) + 1);
        int32_t t = 0;
        for (int64_t j = 0; j <= tiles; ++j) {
            const int64_t first = j * mc::kLookupElems;
            while (t < n_tensors && L->off[t + 1] <= first) ++t;
            L->tile_first[j] = t;  // == n_tensors only when first >= N
        }

        // Tensor-aligned units of each colour (see mc_internal.h).
        if (k_colours <= 32 && total > 0) {
            const int64_t u = MC_COLOUR_ALIGN_ELEMS;
            std::vector<int32_t> t_lo(size_t(k_colours), 0), t_hi(size_t(k_colours), -1);
            std::vector<int64_t> count(size_t(k_colours), 0);
            int64_t most = 0;
            int32_t tt = 0;
            for (int32_t c = 0; c < k_colours; ++c) {
                const int64_t lo_c = L->bounds[c], hi_c = L->bounds[c + 1];
                if (hi_c <= lo_c) continue;
                while (L->off[tt + 1] <= lo_c) ++tt;        // lo_c < N == off[n]
                t_lo[c] = tt;
                int32_t te = tt;
                for (;; ++te) {
                    const int64_t lo = std::max(lo_c, L->off[te]), hi = std::min(hi_c, L->off[te + 1]);
                    if (hi > lo) count[c] += (hi - L->off[te] + u - 1) / u - (lo - L->off[te]) / u;
                    if (L->off[te + 1] >= hi_c) break;
                }
                t_hi[c] = te;
                most = std::max(most, count[c]);
            }
            if (most * k_colours < 0x7fffffff) {
                L->units_per_colour = int32_t(most);
                L->unit_tensor.assign(size_t(most) * size_t(k_colours), -1);
                L->unit_first.assign(size_t(n_tensors) + size_t(k_colours), 0);
                for (int32_t c = 0; c < k_colours; ++c) {
                    const int64_t lo_c = L->bounds[c], hi_c = L->bounds[c + 1];
                    int64_t local = 0;
                    for (int32_t te = t_lo[c]; te <= t_hi[c]; ++te) {
                        L->unit_first[size_t(c) + size_t(te)] = int32_t(local);
                        const int64_t lo = std::max(lo_c, L->off[te]), hi = std::min(hi_c, L->off[te + 1]);
                        if (hi <= lo) continue;
                        const int64_t nu = (hi - L->off[te] + u - 1) / u - (lo - L->off[te]) / u;
                        for (int64_t j = 0; j < nu; ++j) L->unit_tensor[size_t(c) * size_t(most) + size_t(local + j)] = te;
                        local += nu;
                    }
                }
            }
        }
    } catch (const std::bad_alloc&) {
        delete L;
        return MC_ERR_ALLOC;
    }
    *out = L;
    return MC_OK;
}

int mc_layout_units(const mc_layout* L, int32_t* units_per_colour, int32_t* unit_tensor, int32_t* unit_first) {
    if (!L || !units_per_colour) return MC_ERR_INVALID_ARG;
    *units_per_colour = L->unit_tensor.empty() ? 0 : L->units_per_colour;
    if (unit_tensor) std::copy(L->unit_tensor.begin(), L->unit_tensor.end(), unit_tensor);
    if (unit_first) std::copy(L->unit_first.begin(), L->unit_first.end(), unit_first);
    return MC_OK;
}

int mc_layout_total(const mc_layout* L, int64_t* N) {
    if (!L || !N) return MC_ERR_INVALID_ARG;
    *N = L->N;
    return MC_OK;
}

int mc_layout_counts(const mc_layout* L, int32_t* n_tensors, int32_t* k_colours) {
    if (!L || !n_tensors || !k_colours) return MC_ERR_INVALID_ARG;
    *n_tensors = L->n;
    *k_colours = L->k;
    return MC_OK;
}

int mc_layout_tensor_offsets(const mc_layout* L, int64_t* off) {
    if (!L || !off) return MC_ERR_INVALID_ARG;
    for (size_t i = 0; i < L->off.size(); ++i) off[i] = L->off[i];
    return MC_OK;
}

int mc_layout_colour_bounds(const mc_layout* L, int64_t* b) {
    if (!L || !b) return MC_ERR_INVALID_ARG;
    for (size_t i = 0; i < L->bounds.size(); ++i) b[i] = L->bounds[i];
    return MC_OK;
}

const char* mc_strerror(int code) {
    switch (code) {
        case MC_OK: return "ok";
        case MC_ERR_INVALID_ARG: return "invalid argument";
        case MC_ERR_ALIGN: return "buffer is not sufficiently aligned";
        case MC_ERR_OVERLAP: return "buffers overlap";
        case MC_ERR_ALLOC: return "host allocation failed";
        case MC_ERR_HIP: return "HIP runtime call failed";
        case MC_ERR_LIMIT: return "input exceeds the fixed capacity of this entry point";
        default: return "unknown error code";
    }
}

int mc_last_hip_error(void) { return g_last_hip_error; }

int mc_set_option(int option, int value) {
    switch (option) {
        case MC_OPT_RU_SHAPE:
            if (value != 0 && value != 1 && value != 2) return MC_ERR_INVALID_ARG;
            g_ru_shape.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_STATE_POLICY:
            if (value != MC_STATE_RESIDENT && value != MC_STATE_STREAMING) return MC_ERR_INVALID_ARG;
            g_state_policy.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_PACK_NONTEMPORAL:
            if (value < 0 || value > 3) return MC_ERR_INVALID_ARG;
            g_pack_nontemporal.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_STATE_STORE_SC1:
            if (value != 0 && value != 1) return MC_ERR_INVALID_ARG;
            g_state_store_sc1.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_ALTERNATE_SWEEP:
            if (value != 0 && value != 1) return MC_ERR_INVALID_ARG;
            g_alternate_sweep.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_XCD_RUN:
            if (value < 0 || value > 64) return MC_ERR_INVALID_ARG;
            g_xcd_run.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_XCD_RUN_PACK:
            if (value < -1 || value > 64) return MC_ERR_INVALID_ARG;
            g_xcd_run_pack.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_XCD_RUN_UNPACK:
            if (value < -1 || value > 64) return MC_ERR_INVALID_ARG;
            g_xcd_run_unpack.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_LDS_CAP_UPDATE:
            if (value < -1 || value > 65536) return MC_ERR_INVALID_ARG;
            g_lds_cap_update.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_LDS_CAP_PACK:
            if (value < -1 || value > 65536) return MC_ERR_INVALID_ARG;
            g_lds_cap_pack.store(value, std::memory_order_relaxed);
            return MC_OK;
        case MC_OPT_DIRECT_TILES:
            if (value < 0 || value > 2) return MC_ERR_INVALID_ARG;
            g_direct_tiles.store(value, std::memory_order_relaxed);
            return MC_OK;
        default:
            return MC_ERR_INVALID_ARG;
    }
}

int mc_get_option(int option, int* value) {
    if (!value) return MC_ERR_INVALID_ARG;
    const int v = mc::option(option);
    if (v == mc::kNoSuchOption) return MC_ERR_INVALID_ARG;
    *value = v;
    return MC_OK;
}

}  // extern "C"
