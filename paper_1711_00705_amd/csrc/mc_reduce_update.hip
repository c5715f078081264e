// a3 + a4: per-colour, fixed-order sum of P contributions fused with the SGD update.
//
// The pass is pure streaming: per element it reads P + 2 words and writes 2 or 3, with P + 4
// flops, so it is bound by HBM bandwidth and the kernel's only job is to keep enough 128-bit
// loads in flight.  The grid is partitioned by colour: each colour owns a contiguous run of
// workgroups, and the colour's summation sequence is applied by handing that colour its own,
// already permuted, list of contribution pointers.  Colours never synchronise with each other
// (Section 4.2).  Two kernels: reduce_update_direct_kernel (the usual launch: 256-element tiles,
// a tile's colour found by dividing its index by the chunk length, compile-time term count) and
// reduce_update_kernel (run-time term counts, per-colour roles, the 256-thread shape, and calls
// whose colours do not fit one launch: a prefix table in the kernel arguments maps blockIdx -> colour).
//
// Arithmetic is written operation by operation and the file is compiled with floating-point
// contraction off, so each add and multiply is rounded once to binary32 exactly as in the
// definition; denormals are preserved (HIP's default for fp32 on gfx9).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <vector>

#include "mc_internal.h"
#include "mc_tiles.h"
#include "mc_ru_tile.h"
#include "mc_update.h"

#pragma clang fp contract(off)

namespace {

constexpr int kMaxSegs = 32;     // colour segments per launch
constexpr int kPtrSlots = 256;   // permuted contribution pointers per launch

struct RuArgs {
    const float* x[kPtrSlots];      // x[first + q], first from seg_info[s]: q-th term of segment s
    int64_t lo[kMaxSegs];           // segment s covers flat elements [lo[s], hi[s])
    int64_t hi[kMaxSegs];
    int32_t first_block[kMaxSegs + 1];
    // Per segment, in one 32-bit word (narrower arrays indexed at run time would make the compiler
    // copy the whole argument block to scratch memory): bits 0-15 index of the segment's first
    // pointer in x, bits 16-23 its number of terms, bit 24 whether it applies the update (the
    // last two are read by per-segment launches only).
    uint32_t seg_info[kMaxSegs];
    int32_t n_segs;
    // Direct mapping (tiles_per_colour > 0; only with 256-element tiles, which is the colour
    // alignment): the launch covers flat elements [256 * first_tile, range_hi) tile by tile, segment
    // s is colour s, and a tile's colour is its index divided by the chunk length -- nothing is
    // searched and lo / hi / first_block are not read.
    int32_t tiles_per_colour;
    uint32_t first_tile;
    int64_t range_hi;
    int32_t reverse;                // walk the launch's tiles from the last to the first
    int32_t xcd_run;                // consecutive tiles per die (see mc_tiles.h); <= 1: plain
    float* g;                       // may be null when every segment updates
    float* w;                       // unused when no segment updates
    float* v;
    mc::UpdateParams up;
    uint32_t lds_per_wave;              // host only: dynamic LDS reserved by a launch of 64-thread workgroups
    uint32_t lds_per_4waves;            //            ... of 256-thread workgroups (an occupancy cap, nothing is stored there)
};

// What a launch does with the sum.
enum : int {
    kSumOnly = 0,      // write it to g (colours of which the rank is a leaf or inner node)
    kUpdateAndG = 1,   // write it to g and apply the SGD step
    kUpdateOnly = 2,   // apply the SGD step, g is not wanted
    kPerSegment = 3    // each segment has its own number of terms and its own update flag
};

// A per-segment launch picks the compile-time body for the common term counts (m replicas, or m
// plus one buffer per child, with m and the tree's arity powers of two) and the run-time loop
// otherwise.
template <int U, int THREADS, bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void ru_tile_any(const float* const* xs, int np, int64_t base, int64_t hi, float* g,
                                            float* w, float* v, const mc::Hyper& hp) {
    switch (np) {
        case 2: mc::ru_tile<2, U, THREADS, HAS_G, UPDATE, SS>(xs, np, base, hi, g, w, v, hp); break;
        case 4: mc::ru_tile<4, U, THREADS, HAS_G, UPDATE, SS>(xs, np, base, hi, g, w, v, hp); break;
        case 8: mc::ru_tile<8, U, THREADS, HAS_G, UPDATE, SS>(xs, np, base, hi, g, w, v, hp); break;
        default: mc::ru_tile<0, U, THREADS, HAS_G, UPDATE, SS>(xs, np, base, hi, g, w, v, hp); break;
    }
}

template <int P, int U, int THREADS, int MODE, bool SS>
__global__ __launch_bounds__(THREADS) void reduce_update_kernel(RuArgs a, int Prt) {
    constexpr int64_t kTile = int64_t(THREADS) * 4 * U;
    const mc::Hyper hp = mc::resolve(a.up);

    // blockIdx -> (segment, tile); a handful of scalar compares.
    const int tile = mc::xcd_tile(int(blockIdx.x), int(gridDim.x), a.xcd_run);
    const int blk = a.reverse ? int(gridDim.x) - 1 - tile : tile;
    int s = 0;
    int64_t base, hi;
    if (kTile == MC_COLOUR_ALIGN_ELEMS && a.tiles_per_colour > 0) {
        const uint32_t t = a.first_tile + uint32_t(blk);
        s = int(t / uint32_t(a.tiles_per_colour));
        base = int64_t(t) * kTile;
        const int64_t colour_end = int64_t(s + 1) * a.tiles_per_colour * kTile;
        hi = colour_end < a.range_hi ? colour_end : a.range_hi;
    } else {
        while (s + 1 < a.n_segs && blk >= a.first_block[s + 1]) ++s;
        hi = a.hi[s];
        base = a.lo[s] + int64_t(blk - a.first_block[s]) * kTile;
    }
    const bool direct_uniform = kTile == MC_COLOUR_ALIGN_ELEMS && a.tiles_per_colour > 0 && MODE != kPerSegment;
    const float* const* xs = a.x + (direct_uniform ? s * (P > 0 ? P : Prt) : int(a.seg_info[s] & 0xffffu));

    if (MODE == kPerSegment) {
        const int np = int((a.seg_info[s] >> 16) & 0xffu);
        if (np == 0) return;                       // a colour this call skips (direct mapping only)
        if ((a.seg_info[s] >> 24) & 1u) {
            if (a.g)
                ru_tile_any<U, THREADS, true, true, SS>(xs, np, base, hi, a.g, a.w, a.v, hp);
            else
                ru_tile_any<U, THREADS, false, true, SS>(xs, np, base, hi, a.g, a.w, a.v, hp);
        } else {
            ru_tile_any<U, THREADS, true, false, SS>(xs, np, base, hi, a.g, a.w, a.v, hp);
        }
    } else {
        const int np = P > 0 ? P : Prt;
        mc::ru_tile<P, U, THREADS, MODE != kUpdateOnly, MODE != kSumOnly, SS>(xs, np, base, hi, a.g, a.w, a.v, hp);
    }
}

// The launch most calls get: direct mapping, one wavefront per 256-element tile, a compile-time
// term count shared by all colours.  The scalars a tile needs first are leading kernel arguments,
// which arrive in registers when the wavefront starts (kernel-argument preload); the colour's P
// pointers and the hyper-parameters are then fetched from the argument block in ONE batch, and the
// tile's loads follow.  (The general kernel above reaches its first load after six dependent
// argument fetches, because every branch on the way defers the fetches behind it.)
// flip: index of the last tile when the launch walks backwards, -1 otherwise.
template <int P, int MODE, bool SS>
__global__ __launch_bounds__(64) void reduce_update_direct_kernel(float* g, float* w, float* v, int32_t tiles_per_colour,
                                                                  uint32_t first_tile, int32_t flip, int64_t range_hi,
                                                                  RuArgs a) {
    static_assert(P > 0 && MODE != kPerSegment, "uniform launches with a compile-time term count");
    constexpr int64_t kTile = MC_COLOUR_ALIGN_ELEMS;
    const int blk = flip >= 0 ? flip - int(blockIdx.x) : int(blockIdx.x);
    const uint32_t t = first_tile + uint32_t(blk);
    const int s = int(t / uint32_t(tiles_per_colour));
    const float* xp[P];
#pragma unroll
    for (int q = 0; q < P; ++q) xp[q] = a.x[s * P + q];
    const mc::UpdateParams up = a.up;
    __builtin_amdgcn_sched_barrier(0);
    const mc::Hyper hp = mc::resolve(up);
    const int64_t base = int64_t(t) * kTile;
    const int64_t colour_end = int64_t(s + 1) * tiles_per_colour * kTile;
    const int64_t hi = colour_end < range_hi ? colour_end : range_hi;
    mc::ru_tile<P, 1, 64, MODE != kUpdateOnly, MODE != kSumOnly, SS>(xp, P, base, hi, g, w, v, hp);
}

template <int P>
void launch_direct_mode(int mode, bool ss, unsigned blocks, hipStream_t s, const RuArgs& a) {
    const dim3 grid(blocks), block(64);
    const int32_t flip = a.reverse ? int32_t(blocks) - 1 : -1;
#define MC_RU_LAUNCH(MODE, SS)                                                                                  \
    hipLaunchKernelGGL((reduce_update_direct_kernel<P, MODE, SS>), grid, block,                                    \
                       a.lds_per_wave, s, a.g, a.w, a.v, a.tiles_per_colour, a.first_tile, \
                       flip, a.range_hi, a)
    switch (mode) {
        case kSumOnly: MC_RU_LAUNCH(kSumOnly, false); break;
        case kUpdateAndG: if (ss) MC_RU_LAUNCH(kUpdateAndG, true); else MC_RU_LAUNCH(kUpdateAndG, false); break;
        default: if (ss) MC_RU_LAUNCH(kUpdateOnly, true); else MC_RU_LAUNCH(kUpdateOnly, false); break;
    }
#undef MC_RU_LAUNCH
}

void launch_direct(int P, int mode, bool ss, unsigned blocks, hipStream_t s, const RuArgs& a) {
    switch (P) {
        case 1: launch_direct_mode<1>(mode, ss, blocks, s, a); break;
        case 2: launch_direct_mode<2>(mode, ss, blocks, s, a); break;
        case 3: launch_direct_mode<3>(mode, ss, blocks, s, a); break;
        case 4: launch_direct_mode<4>(mode, ss, blocks, s, a); break;
        case 5: launch_direct_mode<5>(mode, ss, blocks, s, a); break;
        case 6: launch_direct_mode<6>(mode, ss, blocks, s, a); break;
        case 7: launch_direct_mode<7>(mode, ss, blocks, s, a); break;
        default: launch_direct_mode<8>(mode, ss, blocks, s, a); break;
    }
}

template <int P, int U, int T>
void launch_mode(int mode, bool ss, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    const dim3 grid(blocks), block(T);
#define MC_RU_LAUNCH(MODE, SS) hipLaunchKernelGGL((reduce_update_kernel<P, U, T, MODE, SS>), grid, block, (T == 64 ? a.lds_per_wave : a.lds_per_4waves), s, a, Prt)
    switch (mode) {
        case kSumOnly: MC_RU_LAUNCH(kSumOnly, false); break;   // state is not touched: one policy
        case kUpdateAndG: if (ss) MC_RU_LAUNCH(kUpdateAndG, true); else MC_RU_LAUNCH(kUpdateAndG, false); break;
        default: if (ss) MC_RU_LAUNCH(kUpdateOnly, true); else MC_RU_LAUNCH(kUpdateOnly, false); break;
    }
#undef MC_RU_LAUNCH
}

template <int P>
void launch_shape(mc::Shape shape, int mode, bool ss, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    if (shape.threads == 64)
        launch_mode<P, 1, 64>(mode, ss, blocks, s, a, Prt);
    else
        launch_mode<P, 2, 256>(mode, ss, blocks, s, a, Prt);
}

// A launch whose segments all add P terms and agree on updating.
void launch(int P, mc::Shape shape, int mode, bool ss, unsigned blocks, hipStream_t s, const RuArgs& a) {
    switch (P) {
        case 1: launch_shape<1>(shape, mode, ss, blocks, s, a, P); break;
        case 2: launch_shape<2>(shape, mode, ss, blocks, s, a, P); break;
        case 3: launch_shape<3>(shape, mode, ss, blocks, s, a, P); break;
        case 4: launch_shape<4>(shape, mode, ss, blocks, s, a, P); break;
        case 5: launch_shape<5>(shape, mode, ss, blocks, s, a, P); break;
        case 6: launch_shape<6>(shape, mode, ss, blocks, s, a, P); break;
        case 7: launch_shape<7>(shape, mode, ss, blocks, s, a, P); break;
        case 8: launch_shape<8>(shape, mode, ss, blocks, s, a, P); break;
        default: launch_shape<0>(shape, mode, ss, blocks, s, a, P); break;
    }
}

// A launch whose segments differ in term count or update flag (always 64 threads x 1 vector).
void launch_per_segment(bool ss, unsigned blocks, hipStream_t s, const RuArgs& a) {
    const dim3 grid(blocks), block(64);
    if (ss)
        hipLaunchKernelGGL((reduce_update_kernel<0, 1, 64, kPerSegment, true>), grid, block, a.lds_per_wave, s, a, 0);
    else
        hipLaunchKernelGGL((reduce_update_kernel<0, 1, 64, kPerSegment, false>), grid, block, a.lds_per_wave, s, a, 0);
}

// Shared by every entry point.  n_terms / do_update are null for the uniform call (every
// colour adds all P terms and updates).
//
// [r_lo, r_hi) restricts the call to a sub-range of the payload (a packet): every colour is
// intersected with it.  r_lo and r_hi are multiples of the colour alignment (r_hi may also be
// N), so every segment still starts on a 16-byte boundary.
int run_impl(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
             const int32_t* n_terms, const uint8_t* do_update, void* grad_out, void* weights,
             void* momentum, const mc::UpdatePlan& plan, int64_t r_lo, int64_t r_hi, void* stream) {
    if (!L || !contrib || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
    if (plan.up.hyper && !mc::aligned(plan.up.hyper, 4)) return MC_ERR_ALIGN;
    if (r_lo < 0 || r_hi < r_lo || r_hi > L->N) return MC_ERR_INVALID_ARG;
    if (r_lo % MC_COLOUR_ALIGN_ELEMS != 0) return MC_ERR_INVALID_ARG;
    if (r_hi % MC_COLOUR_ALIGN_ELEMS != 0 && r_hi != L->N) return MC_ERR_INVALID_ARG;
    if ((n_terms == nullptr) != (do_update == nullptr)) return MC_ERR_INVALID_ARG;
    const int orc = mc::check_order(L, P, order);
    if (orc != MC_OK) return orc;
    // What colour c contributes to this call: its range cut to [r_lo, r_hi), its term count and
    // whether it updates.
    auto seg_lo = [&](int32_t c) { return std::max(L->bounds[c], r_lo); };
    auto seg_hi = [&](int32_t c) { return std::max(seg_lo(c), std::min(L->bounds[c + 1], r_hi)); };
    auto terms = [&](int32_t c) { return n_terms ? n_terms[c] : P; };
    auto updates = [&](int32_t c) { return do_update ? do_update[c] != 0 : true; };
    auto in_range = [&](int32_t c) { return seg_hi(c) > seg_lo(c); };
    auto active = [&](int32_t c) { return terms(c) > 0 && in_range(c); };
    bool any_update = false, any_sum_only = false, uniform = true, any_skipped = false;
    int32_t first_active = -1;
    int max_terms = 0, total_terms = 0;
    for (int32_t c = 0; c < L->k; ++c) {
        if (n_terms && (n_terms[c] < 0 || n_terms[c] > P)) return MC_ERR_INVALID_ARG;
        if (in_range(c) && terms(c) == 0) any_skipped = true;
        if (!active(c)) continue;
        if (updates(c)) any_update = true; else any_sum_only = true;
        max_terms = std::max(max_terms, int(terms(c)));
        total_terms += terms(c);
        if (first_active < 0) first_active = c;
        else if (terms(c) != terms(first_active) || updates(c) != updates(first_active)) uniform = false;
    }
    if (first_active < 0) return MC_OK;  // nothing in range
    const int rc = mc::check_flat_buffers(L, contrib, P, grad_out, weights, momentum, any_update, any_sum_only);
    if (rc != MC_OK) return rc;

    const bool ss = any_update && mc::stream_state(L, plan.state_policy);
    // Launches that mix term counts or update flags use the one-wavefront shape.
    const mc::Shape shape = uniform ? mc::shape_for(r_hi - r_lo, max_terms, ss) : mc::Shape{64, 1};
    const int64_t tile = shape.tile();
    hipStream_t s = static_cast<hipStream_t>(stream);

    RuArgs a;
    // Only the plain whole-payload step alternates by itself: packets and role calls come several to a step.
    const bool whole = !n_terms && r_lo == 0 && r_hi == L->N;
    a.reverse = mc::sweep_reversed(L, whole ? plan.sweep : (plan.sweep == MC_SWEEP_AUTO ? MC_SWEEP_FORWARD : plan.sweep), ss) ? 1 : 0;
    a.xcd_run = mc::option(MC_OPT_XCD_RUN);
    {
        const int avg_terms = uniform ? int(terms(first_active)) : 0;
        const bool state_cached = !ss && !any_sum_only;
        a.lds_per_wave = mc::update_lds_reservation(L, 64, state_cached, avg_terms, false);
        a.lds_per_4waves = mc::update_lds_reservation(L, 256, state_cached, avg_terms, false);
    }
    a.g = static_cast<float*>(grad_out);
    a.w = static_cast<float*>(weights);
    a.v = static_cast<float*>(momentum);
    a.up = plan.up;
    a.tiles_per_colour = 0;
    a.first_tile = 0;
    a.range_hi = r_hi;
    auto pointer_list = [&](int32_t c, int slot) {
        for (int32_t q = 0; q < terms(c); ++q)
            a.x[slot + q] = static_cast<const float*>(contrib[order ? order[size_t(c) * P + q] : q]);
    };

    // Direct mapping: a 256-element tile is exactly the colour alignment, so the tiles of the call are
    // the 256-element runs of [r_lo, r_hi) and a tile's colour is its index divided by the chunk
    // length.  Needs every colour's pointer list in the one launch.
    const int64_t tiles_total = (r_hi - r_lo + tile - 1) / tile;
    // (A call whose colours agree but for some it skips keeps the table, which simply leaves the
    // skipped colours out and still runs the compile-time body.)
    const int slots_needed = uniform ? L->k * terms(first_active) : total_terms;
    if (tile == MC_COLOUR_ALIGN_ELEMS && !(uniform && any_skipped) && L->k <= kMaxSegs && slots_needed <= kPtrSlots &&
        tiles_total <= 0x7fffffff && L->N / tile < 0x7fffffff && mc::option(MC_OPT_DIRECT_TILES) != 0) {
        a.tiles_per_colour = int32_t(L->chunk / tile);
        a.first_tile = uint32_t(r_lo / tile);
        a.n_segs = L->k;
        for (int i = 0; i < kPtrSlots; ++i) a.x[i] = nullptr;
        for (int i = 0; i < kMaxSegs; ++i) {
            a.lo[i] = a.hi[i] = 0;
            a.seg_info[i] = 0;
            a.first_block[i] = 0;
        }
        a.first_block[kMaxSegs] = 0;
        const bool per_segment = !uniform;
        int slots = 0;
        for (int32_t c = 0; c < L->k; ++c) {
            if (!per_segment) {
                if (in_range(c)) pointer_list(c, c * terms(first_active));
            } else if (active(c)) {
                a.seg_info[c] = uint32_t(slots) | (uint32_t(terms(c)) << 16) | (updates(c) ? (1u << 24) : 0u);
                pointer_list(c, slots);
                slots += terms(c);
            }
        }
        if (per_segment) {
            launch_per_segment(ss, unsigned(tiles_total), s, a);
        } else {
            const int mode = !updates(first_active) ? kSumOnly : (a.g ? kUpdateAndG : kUpdateOnly);
            if (terms(first_active) <= 8 && a.xcd_run < 2)   // (a run of tiles per die is the general kernel's)
                launch_direct(terms(first_active), mode, ss, unsigned(tiles_total), s, a);
            else
                launch(terms(first_active), shape, mode, ss, unsigned(tiles_total), s, a);
        }
        MC_HIP_TRY(hipGetLastError());
        return MC_OK;
    }

    // Otherwise colours are taken in index order, as many per launch as the segment and pointer slots
    // hold, each with its own run of workgroups (a prefix table maps a workgroup to its segment).
    int32_t c = 0;
    while (c < L->k) {
        int ns = 0, slots = 0;
        int64_t blocks = 0;
        a.first_block[0] = 0;
        for (; c < L->k && ns < kMaxSegs; ++c) {
            if (!active(c)) continue;
            const int32_t cnt = terms(c);
            if (slots + cnt > kPtrSlots) break;
            const int64_t lo = seg_lo(c), hi = seg_hi(c);
            const int64_t nblk = (hi - lo + tile - 1) / tile;
            if (blocks + nblk > 0x7fffffff) {
                if (ns == 0) return MC_ERR_INVALID_ARG;
                break;
            }
            a.lo[ns] = lo;
            a.hi[ns] = hi;
            a.seg_info[ns] = uint32_t(slots) | (uint32_t(cnt) << 16) | (updates(c) ? (1u << 24) : 0u);
            pointer_list(c, slots);
            slots += cnt;
            blocks += nblk;
            a.first_block[ns + 1] = int32_t(blocks);
            ++ns;
        }
        if (ns == 0) break;
        for (int i = slots; i < kPtrSlots; ++i) a.x[i] = nullptr;
        for (int i = ns; i < kMaxSegs; ++i) {
            a.lo[i] = a.hi[i] = 0;
            a.seg_info[i] = 0;
            a.first_block[i + 1] = a.first_block[ns];
        }
        a.n_segs = ns;
        if (uniform) {
            const int mode = !updates(first_active) ? kSumOnly : (a.g ? kUpdateAndG : kUpdateOnly);
            launch(terms(first_active), shape, mode, ss, unsigned(blocks), s, a);
        } else {
            launch_per_segment(ss, unsigned(blocks), s, a);
        }
        MC_HIP_TRY(hipGetLastError());
    }
    return MC_OK;
}

// No C++ exception may cross the C boundary.
int run(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
        const int32_t* n_terms, const uint8_t* do_update, void* grad_out, void* weights,
        void* momentum, const mc::UpdatePlan& plan, int64_t r_lo, int64_t r_hi, void* stream) {
    try {
        return run_impl(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, plan,
                        r_lo, r_hi, stream);
    } catch (const std::bad_alloc&) {
        return MC_ERR_ALLOC;
    }
}

mc::UpdatePlan immediate(float lr, float mu, float wd) {
    mc::UpdatePlan plan;
    plan.up.lr = lr;
    plan.up.mu = mu;
    plan.up.wd = wd;
    plan.up.hyper = nullptr;
    plan.up.nesterov = 0;
    plan.up.state_store_sc1 = mc::option(MC_OPT_STATE_STORE_SC1);
    plan.state_policy = MC_STATE_DEFAULT;
    plan.sweep = MC_SWEEP_AUTO;
    return plan;
}

}  // namespace

namespace mc {

int check_order(const mc_layout* L, int32_t P, const int32_t* order) {
    if (!L || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
    if (order) {
        for (int32_t c = 0; c < L->k; ++c) {
            uint64_t seen = 0;
            for (int32_t q = 0; q < P; ++q) {
                const int32_t o = order[size_t(c) * P + q];
                if (o < 0 || o >= P || (seen >> o) & 1) return MC_ERR_INVALID_ARG;
                seen |= uint64_t(1) << o;
            }
        }
    }
    return MC_OK;
}

int check_flat_buffers(const mc_layout* L, const void* const* contrib, int32_t P, const void* grad_out,
                       const void* weights, const void* momentum, bool needs_state, bool needs_g) {
    if (!L || !contrib || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
    if (needs_state && (!weights || !momentum)) return MC_ERR_INVALID_ARG;
    if (needs_g && !grad_out) return MC_ERR_INVALID_ARG;
    for (int32_t p = 0; p < P; ++p)
        if (!contrib[p]) return MC_ERR_INVALID_ARG;
    const void* written[3];
    int nw = 0;
    if (weights) written[nw++] = weights;
    if (momentum) written[nw++] = momentum;
    if (grad_out) written[nw++] = grad_out;
    for (int32_t p = 0; p < P; ++p)
        if (!aligned(contrib[p], 16)) return MC_ERR_ALIGN;
    for (int i = 0; i < nw; ++i)
        if (!aligned(written[i], 16)) return MC_ERR_ALIGN;
    const uint64_t bytes = uint64_t(L->N) * 4;
    for (int i = 0; i < nw; ++i) {
        for (int j = i + 1; j < nw; ++j)
            if (overlaps(written[i], bytes, written[j], bytes)) return MC_ERR_OVERLAP;
        for (int32_t p = 0; p < P; ++p)
            if (overlaps(written[i], bytes, contrib[p], bytes)) return MC_ERR_OVERLAP;
    }
    return MC_OK;
}

int update_plan(const mc_update_spec* spec, UpdatePlan* out) {
    if (!spec || (spec->nesterov != 0 && spec->nesterov != 1)) return MC_ERR_INVALID_ARG;
    if (spec->state_policy < MC_STATE_DEFAULT || spec->state_policy > MC_STATE_STREAMING) return MC_ERR_INVALID_ARG;
    if (spec->sweep < MC_SWEEP_AUTO || spec->sweep > MC_SWEEP_BACKWARD) return MC_ERR_INVALID_ARG;
    out->up.lr = spec->lr;
    out->up.mu = spec->mu;
    out->up.wd = spec->wd;
    out->up.hyper = spec->hyper_dev;
    out->up.nesterov = spec->nesterov;
    out->up.state_store_sc1 = mc::option(MC_OPT_STATE_STORE_SC1);
    out->state_policy = spec->state_policy;
    out->sweep = spec->sweep;
    return MC_OK;
}

}  // namespace mc

extern "C" {

int mc_reduce_update(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
                     void* grad_out, void* weights, void* momentum, float lr, float mu, float wd,
                     void* stream) {
    if (!L) return MC_ERR_INVALID_ARG;
    return run(L, contrib, P, order, nullptr, nullptr, grad_out, weights, momentum, immediate(lr, mu, wd),
               0, L->N, stream);
}

int mc_reduce_update_roles(const mc_layout* L, const void* const* contrib, int32_t P,
                           const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                           void* grad_out, void* weights, void* momentum, float lr, float mu,
                           float wd, void* stream) {
    if (!L || !n_terms || !do_update) return MC_ERR_INVALID_ARG;
    return run(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum,
               immediate(lr, mu, wd), 0, L->N, stream);
}

int mc_reduce_update_range(const mc_layout* L, const void* const* contrib, int32_t P,
                           const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                           void* grad_out, void* weights, void* momentum, float lr, float mu,
                           float wd, int64_t elem_begin, int64_t elem_end, void* stream) {
    if (!L) return MC_ERR_INVALID_ARG;
    return run(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum,
               immediate(lr, mu, wd), elem_begin, elem_end, stream);
}

int mc_reduce_update_ex(const mc_layout* L, const void* const* contrib, int32_t P,
                        const int32_t* order, const int32_t* n_terms, const uint8_t* do_update,
                        void* grad_out, void* weights, void* momentum, const mc_update_spec* spec,
                        int64_t elem_begin, int64_t elem_end, void* stream) {
    if (!L) return MC_ERR_INVALID_ARG;
    mc::UpdatePlan plan;
    const int rc = mc::update_plan(spec, &plan);
    if (rc != MC_OK) return rc;
    return run(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, plan,
               elem_begin, elem_end < 0 ? L->N : elem_end, stream);
}

}  // extern "C"
