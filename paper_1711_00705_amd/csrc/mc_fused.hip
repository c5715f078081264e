// Fused step: sum the P contributions straight out of their per-layer tensors, apply the SGD
// update to per-layer weights and momentum in place, and emit the reduced gradient as the flat
// colour-chunked payload -- no staging copy of any contribution, no separate unpack.
//
// The flat index space (and with it the colour chunks and each colour's summation sequence) is
// exactly that of pack + reduce_update + unpack: element i of the payload is element
// i - off[t] of tensor t.  A tensor set is the device-resident list of one tensor pointer per
// layer.  Four kernels, chosen by the host:
//   fused_unit_kernel    the default: one wavefront per tensor-aligned unit of the layout (a run of 256
//                        elements counted from its tensor's first element), compile-time term count;
//   fused_unit_roles_kernel  the same units for calls whose colours differ in term count (up to
//                        eight) or update flag: a rank's role-dependent step;
//   fused_direct_kernel  flat 256-element tiles, a tile's colour found by division (layouts without a
//                        unit table, MC_OPT_DIRECT_TILES = 2);
//   fused_step_kernel    the general one: run-time term counts (9..32), roles with such counts, the
//                        256-thread shape, colour segments searched in a per-launch table.
// In all of them a work item that lies inside one tensor with every operand 16-byte aligned (almost
// all of a CNN payload) resolves its P + 2 base pointers once and runs the same 128-bit streaming
// body as reduce_update; anything else (a tensor's end, a colour bound, unaligned operands) takes a
// masked or per-element path.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <vector>

#include "mc_internal.h"
#include "mc_tiles.h"
#include "mc_update.h"

#pragma clang fp contract(off)

namespace {

constexpr int kMaxSegs = 32;
constexpr int kPtrSlots = 256;

struct FusedArgs {
    const float* const* x[kPtrSlots];   // x[first + q], first from seg_info[s]: pointer table of the q-th term of segment s
    int64_t lo[kMaxSegs];
    int64_t hi[kMaxSegs];
    int32_t first_block[kMaxSegs + 1];
    // Per segment, in one 32-bit word (narrower arrays indexed at run time would make the compiler
    // copy the whole argument block to scratch memory): bits 0-15 index of the segment's first
    // pointer in x, bits 16-23 its number of terms, bit 24 whether it applies the update (the
    // last two are read by per-segment launches only).
    uint32_t seg_info[kMaxSegs];
    int32_t n_segs;
    // Direct mapping (tiles_per_colour > 0; only with 256-element tiles, which is the colour
    // alignment): the launch covers the whole payload tile by tile, segment s is colour s, and a
    // tile's colour is its index divided by the chunk length -- nothing is searched and lo / hi /
    // first_block are not read.
    int32_t tiles_per_colour;
    int64_t range_hi;               // N
    int32_t reverse;                // walk the launch's tiles from the last to the first
    int32_t xcd_run;                // consecutive tiles per die (see mc_tiles.h); <= 1: plain
    float* const* w;                    // pointer tables of weights and momentum (per layer)
    float* const* v;
    float* g;                           // flat payload, may be null
    const int64_t* off;                 // n+1 flat offsets
    const int32_t* first_tensor;        // lookup: first tensor per kLookupElems flat elements
    int64_t chunk;                      // unit launches: colour chunk length
    mc::UpdateParams up;
    uint32_t lds_per_wave;              // host only: dynamic LDS reserved by a launch of 64-thread workgroups
    uint32_t lds_per_4waves;            //            ... of 256-thread workgroups (an occupancy cap, nothing is stored there)
};

typedef float native_f4 __attribute__((ext_vector_type(4)));
// Every tensor lives in device global memory.  Pointers read from a tensor set's table arrive as
// generic pointers; dereferencing them through global-address-space types lets the compiler use
// global_ instead of flat_ instructions.
typedef __attribute__((address_space(1))) native_f4 global_f4;
typedef __attribute__((address_space(1))) float global_f1;

template <bool NT>
__device__ __forceinline__ float4 load4(const float* p) {
    const global_f4* gp = (const global_f4*)p;
    const native_f4 r = NT ? __builtin_nontemporal_load(gp) : *gp;
    return make_float4(r.x, r.y, r.z, r.w);
}

template <bool NT>
__device__ __forceinline__ void store4(float* p, const float4& q) {
    const native_f4 val = {q.x, q.y, q.z, q.w};
    global_f4* gp = (global_f4*)p;
    if (NT)
        __builtin_nontemporal_store(val, gp);
    else
        *gp = val;
}

__device__ __forceinline__ float ld1(const float* p) { return *(const global_f1*)p; }
__device__ __forceinline__ void st1(float* p, float x) { *(global_f1*)p = x; }

// Offset of an address from the previous 16-byte boundary, in elements (0..3).
__device__ __forceinline__ int misalignment(const void* p) {
    return int((reinterpret_cast<uintptr_t>(p) >> 2) & 3);
}

__device__ __forceinline__ bool aligned16(const void* p) {
    return (reinterpret_cast<uintptr_t>(p) & 15) == 0;
}

// The arguments a tile needs besides its own position, passed by value (a reference to the kernel's
// argument block would have the compiler keep a private copy of all of it in scratch memory).
struct TileArgs {
    float* const* w;
    float* const* v;
    float* g;
    const int64_t* off;
};

// What a launch does with the sum.
enum : int {
    kSumOnly = 0,      // write it to g (colours of which the rank is a leaf or inner node)
    kUpdateAndG = 1,   // write it to g and apply the SGD step
    kUpdateOnly = 2,   // apply the SGD step, g is not wanted
    kPerSegment = 3    // each segment has its own number of terms and its own update flag
};

// One element: the colour's sum in sequence, the update, the stores.
template <bool HAS_G, bool UPDATE>
__device__ __forceinline__ void one_element(const float* const* const* xs, int np, int32_t t, int64_t r,
                                            float* const* w, float* const* v, float* g, int64_t e,
                                            const mc::Hyper& hp) {
    float acc = ld1(xs[0][t] + r);
    for (int q = 1; q < np; ++q) acc = acc + ld1(xs[q][t] + r);
    if (HAS_G) st1(g + e, acc);
    if (UPDATE) {
        float* wp = w[t] + r;
        float* vp = v[t] + r;
        float we = ld1(wp), ve = ld1(vp);
        mc::sgd(acc, we, ve, hp);
        st1(wp, we);
        st1(vp, ve);
    }
}

// A whole tile that lies inside tensor t0, all operands sharing one alignment.  `rel` is the
// tensor-relative index of the first vectorised element (a 16-byte boundary of every operand),
// gp the matching position in the flat gradient.  SHIFTED: that boundary is not the tile's first
// element, so gp is not 16-byte aligned (g is stored word by word) and the tile has one vector
// less (n_vec); the few elements before and after the vectors are done by the caller.
// SS: weights and momentum are streamed instead of kept resident (see mc_update.h).
// xp: for a compile-time term count, the P operand addresses of the tile's first vector, already
// resolved by the caller (so that their table lookups are issued together, not one after another).
template <int P, int U, int THREADS, bool HAS_G, bool UPDATE, bool SS, bool SHIFTED>
__device__ __forceinline__ void uniform_tile(const float* const* xp, const float* const* const* xs, int np,
                                             int32_t t0, int64_t rel, float* wp, float* vp, float* gp, int n_vec,
                                             const mc::Hyper& hp) {
    int64_t j[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int jv = u * THREADS + int(threadIdx.x);
        on[u] = !SHIFTED || jv < n_vec;
        j[u] = int64_t(jv) * 4;
    }
    float4 acc[U], wv[U], vv[U];
    if (P > 0) {
        float4 t[P > 0 ? P : 1][U];
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const float* xq = xp[q];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (on[u]) t[q][u] = load4<true>(xq + j[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (UPDATE && on[u]) {
                wv[u] = mc::load_state<SS>(wp + j[u]);
                vv[u] = mc::load_state<SS>(vp + j[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc[u] = t[0][u];
#pragma unroll
            for (int q = 1; q < P; ++q) {
                acc[u].x = acc[u].x + t[q][u].x;
                acc[u].y = acc[u].y + t[q][u].y;
                acc[u].z = acc[u].z + t[q][u].z;
                acc[u].w = acc[u].w + t[q][u].w;
            }
        }
    } else {
        // Up to kFirst terms (the counts a tree rank meets that have no compile-time body: 5, 6, 7
        // contributions) have their addresses looked up together and their loads issued together, each
        // guarded by a uniform test of the run-time count.  Larger counts load the first term, then
        // four at a time.  The adds run strictly left to right either way.
        constexpr int kFirst = U == 1 ? 8 : 4;
        int q;
        if (np <= kFirst) {
            const float* xq0[kFirst];
#pragma unroll
            for (int r = 0; r < kFirst; ++r) {
                xq0[r] = nullptr;
                if (r < np) xq0[r] = xs[r][t0] + rel;
            }
            float4 first[kFirst][U];
#pragma unroll
            for (int r = 0; r < kFirst; ++r) {
                if (r < np) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (on[u]) first[r][u] = load4<true>(xq0[r] + j[u]);
                }
            }
            if (UPDATE) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (on[u]) {
                        wv[u] = mc::load_state<SS>(wp + j[u]);
                        vv[u] = mc::load_state<SS>(vp + j[u]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = first[0][u];
#pragma unroll
            for (int r = 1; r < kFirst; ++r) {
                if (r < np) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        acc[u].x = acc[u].x + first[r][u].x;
                        acc[u].y = acc[u].y + first[r][u].y;
                        acc[u].z = acc[u].z + first[r][u].z;
                        acc[u].w = acc[u].w + first[r][u].w;
                    }
                }
            }
            q = np;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (on[u]) {
                    if (UPDATE) {
                        wv[u] = mc::load_state<SS>(wp + j[u]);
                        vv[u] = mc::load_state<SS>(vp + j[u]);
                    }
                    acc[u] = load4<true>(xs[0][t0] + rel + j[u]);
                }
            }
            q = 1;
        }
        for (; q + 4 <= np; q += 4) {
            float4 t[4][U];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float* xq = xs[q + r][t0] + rel;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (on[u]) t[r][u] = load4<true>(xq + j[u]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    acc[u].x = acc[u].x + t[r][u].x;
                    acc[u].y = acc[u].y + t[r][u].y;
                    acc[u].z = acc[u].z + t[r][u].z;
                    acc[u].w = acc[u].w + t[r][u].w;
                }
        }
        for (; q < np; ++q) {
            const float* xq = xs[q][t0] + rel;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (on[u]) {
                    const float4 t = load4<true>(xq + j[u]);
                    acc[u].x = acc[u].x + t.x;
                    acc[u].y = acc[u].y + t.y;
                    acc[u].z = acc[u].z + t.z;
                    acc[u].w = acc[u].w + t.w;
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!on[u]) continue;
        if (HAS_G) {
            if (SHIFTED) {
                float* gq = gp + j[u];
                st1(gq + 0, acc[u].x);
                st1(gq + 1, acc[u].y);
                st1(gq + 2, acc[u].z);
                st1(gq + 3, acc[u].w);
            } else {
                store4<true>(gp + j[u], acc[u]);
            }
        }
        if (UPDATE) {
            mc::sgd(acc[u].x, wv[u].x, vv[u].x, hp);
            mc::sgd(acc[u].y, wv[u].y, vv[u].y, hp);
            mc::sgd(acc[u].z, wv[u].z, vv[u].z, hp);
            mc::sgd(acc[u].w, wv[u].w, vv[u].w, hp);
            mc::store_state<SS>(wp + j[u], wv[u], hp.state_store_sc1);
            mc::store_state<SS>(vp + j[u], vv[u], hp.state_store_sc1);
        }
    }
}

// One tile [base, end) of a segment whose first element lies in tensor t0 = [t0_begin, t0_end).
// P > 0: compile-time number of terms; P == 0: run-time count np.
// UPDATE: the SGD step follows the sum; otherwise only the sum is written to g (the colours of
// which this rank is a leaf or inner node) and weights / momentum are never touched.
// xb / wb / vb: for a compile-time term count, the operands' addresses of tensor t0 (element 0), looked
// up by the caller together with the tensor's bounds; unused (null) for a run-time count.
template <int P, int U, int THREADS, bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void fused_tile(const TileArgs a, const float* const* const* xs, int np,
                                           int64_t base, int64_t end, int32_t t0, int64_t t0_begin,
                                           int64_t t0_end, const float* const* xb, float* wb, float* vb,
                                           const mc::Hyper& hp) {
    static_assert(HAS_G || UPDATE, "a tile must produce something");
    constexpr int kTile = THREADS * 4 * U;
    if (end - base == kTile && end <= t0_end) {
        // Whole tile inside tensor t0.  If every operand has the same offset from a 16-byte
        // boundary (all zero for a CNN payload; equal and non-zero after an odd-sized tensor,
        // because frameworks align the tensors themselves), the tile runs on 128-bit accesses.
        // All operand addresses are looked up first, independently of one another, and compared
        // afterwards without early exits: the lookups then travel together instead of each
        // waiting for the previous one's verdict.
        const int64_t rel = base - t0_begin;
        if (P == 0 && UPDATE) {
            wb = a.w[t0];
            vb = a.v[t0];
        }
        const float* xp[P > 0 ? P : 1];
        if (P > 0) {
#pragma unroll
            for (int q = 0; q < P; ++q) xp[q] = xb[q];
        }
        float* wp = UPDATE ? wb + rel : nullptr;
        float* vp = UPDATE ? vb + rel : nullptr;
        int m;
        bool same = true;
        if (P > 0) {
#pragma unroll
            for (int q = 0; q < P; ++q) xp[q] += rel;
            m = misalignment(xp[0]);
#pragma unroll
            for (int q = 1; q < P; ++q) same &= misalignment(xp[q]) == m;
        } else {
            xp[0] = nullptr;
            m = misalignment(xs[0][t0] + rel);
            for (int q = 1; q < np; ++q) same &= misalignment(xs[q][t0] + rel) == m;
        }
        if (UPDATE) same &= (misalignment(wp) == m) & (misalignment(vp) == m);
        if (same && m == 0) {
            uniform_tile<P, U, THREADS, HAS_G, UPDATE, SS, false>(xp, xs, np, t0, rel, wp, vp, a.g + base, kTile / 4, hp);
            return;
        }
        if (same) {
            const int head = 4 - m;               // elements up to the operands' 16-byte boundary
            const int n_vec = kTile / 4 - 1;      // whole vectors after it
#pragma unroll
            for (int q = 0; q < (P > 0 ? P : 1); ++q) xp[q] += head;
            uniform_tile<P, U, THREADS, HAS_G, UPDATE, SS, true>(xp, xs, np, t0, rel + head, UPDATE ? wp + head : nullptr,
                                                                 UPDATE ? vp + head : nullptr, a.g + base + head,
                                                                 n_vec, hp);
            // the `head` elements before the vectors and the `4 - head` after them
            if (threadIdx.x < 4) {
                const int e = int(threadIdx.x) < head ? int(threadIdx.x)
                                                      : head + 4 * n_vec + (int(threadIdx.x) - head);
                one_element<HAS_G, UPDATE>(xs, np, t0, rel + e, a.w, a.v, a.g, base + e, hp);
            }
            return;
        }
    }

    // General tile: tensor boundaries, the ragged end of the segment, or operands whose
    // alignments differ.
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t(u) * THREADS + threadIdx.x) * 4;
        if (i >= end) break;
        int32_t t = t0;
        while (a.off[t + 1] <= i) ++t;  // ends: i < end <= N == off[n]
        const int64_t rel = i - a.off[t];
        bool vec = i + 4 <= end && i + 4 <= a.off[t + 1];
        if (vec && UPDATE) vec = aligned16(a.w[t] + rel) && aligned16(a.v[t] + rel);
        for (int q = 0; q < np && vec; ++q) vec = aligned16(xs[q][t] + rel);
        if (vec) {
            float4 acc = load4<true>(xs[0][t] + rel);
            for (int q = 1; q < np; ++q) {
                const float4 x = load4<true>(xs[q][t] + rel);
                acc.x = acc.x + x.x;
                acc.y = acc.y + x.y;
                acc.z = acc.z + x.z;
                acc.w = acc.w + x.w;
            }
            if (HAS_G) store4<false>(a.g + i, acc);
            if (UPDATE) {
                float* wp = a.w[t] + rel;
                float* vp = a.v[t] + rel;
                float4 wq = load4<false>(wp);
                float4 vq = load4<false>(vp);
                mc::sgd(acc.x, wq.x, vq.x, hp);
                mc::sgd(acc.y, wq.y, vq.y, hp);
                mc::sgd(acc.z, wq.z, vq.z, hp);
                mc::sgd(acc.w, wq.w, vq.w, hp);
                store4<false>(wp, wq);
                store4<false>(vp, vq);
            }
        } else {
            const int64_t stop = i + 4 < end ? i + 4 : end;
            for (int64_t e = i; e < stop; ++e) {
                while (a.off[t + 1] <= e) ++t;
                one_element<HAS_G, UPDATE>(xs, np, t, e - a.off[t], a.w, a.v, a.g, e, hp);
            }
        }
    }
}

// A per-segment launch picks the compile-time body for the common term counts (m replicas, or m
// plus one buffer per child, with m and the tree's arity powers of two) and the run-time loop
// otherwise.  More bodies than these make the compiler keep a private copy of the kernel's
// argument block in scratch memory (see tests/test_kernel_resources_cpu.py).
template <int U, int THREADS, bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void fused_tile_any(const TileArgs a, const float* const* const* xs, int np,
                                               int64_t base, int64_t end, int32_t t0, int64_t t0_begin,
                                               int64_t t0_end, const mc::Hyper& hp) {
    // per-segment launches look the operands up here, once the term count is known
#define MC_FUSED_CASE(N)                                                                                   \
    case N: {                                                                                              \
        const float* xb[N];                                                                                \
        _Pragma("unroll") for (int q = 0; q < N; ++q) xb[q] = xs[q][t0];                                   \
        float* wb = UPDATE ? a.w[t0] : nullptr;                                                            \
        float* vb = UPDATE ? a.v[t0] : nullptr;                                                            \
        fused_tile<N, U, THREADS, HAS_G, UPDATE, SS>(a, xs, np, base, end, t0, t0_begin, t0_end, xb, wb, vb, hp); \
        break;                                                                                             \
    }
    switch (np) {
        MC_FUSED_CASE(2);
        MC_FUSED_CASE(4);
        MC_FUSED_CASE(8);
        default:
            fused_tile<0, U, THREADS, HAS_G, UPDATE, SS>(a, xs, np, base, end, t0, t0_begin, t0_end, nullptr, nullptr,
                                                         nullptr, hp);
            break;
    }
#undef MC_FUSED_CASE
}

template <int P, int U, int THREADS, int MODE, bool SS>
__global__ __launch_bounds__(THREADS) void fused_step_kernel(FusedArgs a, int Prt) {
    constexpr int kTile = THREADS * 4 * U;
    static_assert(kTile % mc::kLookupElems == 0, "tiles start on lookup entries");
    const mc::Hyper hp = mc::resolve(a.up);

    const int tile = mc::xcd_tile(int(blockIdx.x), int(gridDim.x), a.xcd_run);
    const int blk = a.reverse ? int(gridDim.x) - 1 - tile : tile;
    int s = 0;
    int64_t base, hi;
    if (kTile == MC_COLOUR_ALIGN_ELEMS && a.tiles_per_colour > 0) {
        s = int(uint32_t(blk) / uint32_t(a.tiles_per_colour));
        base = int64_t(blk) * kTile;
        const int64_t colour_end = int64_t(s + 1) * a.tiles_per_colour * kTile;
        hi = colour_end < a.range_hi ? colour_end : a.range_hi;
    } else {
        while (s + 1 < a.n_segs && blk >= a.first_block[s + 1]) ++s;
        hi = a.hi[s];
        base = a.lo[s] + int64_t(blk - a.first_block[s]) * kTile;  // multiple of 256
    }
    const int64_t end = base + kTile < hi ? base + kTile : hi;
    const bool direct_uniform = kTile == MC_COLOUR_ALIGN_ELEMS && a.tiles_per_colour > 0 && MODE != kPerSegment;
    const float* const* const* xs = a.x + (direct_uniform ? s * (P > 0 ? P : Prt) : int(a.seg_info[s] & 0xffffu));

    // The tensor holding the tile's first element (block-uniform).  `base` is a multiple of the
    // lookup granularity, so the table entry is that tensor itself: no scan of off[] is needed.
    const int32_t t0 = a.first_tensor[base / mc::kLookupElems];
    typedef long long ll2 __attribute__((ext_vector_type(2)));
    ll2 t0_bounds;
    __builtin_memcpy(&t0_bounds, a.off + t0, sizeof(t0_bounds));   // both bounds in one 16-byte load
    const int64_t t0_begin = t0_bounds.x;
    const int64_t t0_end = t0_bounds.y;
    const float* xb[P > 0 ? P : 1];
    float* wb = nullptr;
    float* vb = nullptr;
    if (P > 0 && MODE != kPerSegment) {
#pragma unroll
        for (int q = 0; q < P; ++q) xb[q] = xs[q][t0];
        if (MODE != kSumOnly) {
            wb = a.w[t0];
            vb = a.v[t0];
        }
    }

    const TileArgs ta = {a.w, a.v, a.g, a.off};
    if (MODE == kPerSegment) {
        const int np = int((a.seg_info[s] >> 16) & 0xffu);
        if (np == 0) return;                       // a colour this call skips (direct mapping only)
        if ((a.seg_info[s] >> 24) & 1u) {
            if (a.g)
                fused_tile_any<U, THREADS, true, true, SS>(ta, xs, np, base, end, t0, t0_begin, t0_end, hp);
            else
                fused_tile_any<U, THREADS, false, true, SS>(ta, xs, np, base, end, t0, t0_begin, t0_end, hp);
        } else {
            fused_tile_any<U, THREADS, true, false, SS>(ta, xs, np, base, end, t0, t0_begin, t0_end, hp);
        }
    } else {
        const int np = P > 0 ? P : Prt;
        fused_tile<P, U, THREADS, MODE != kUpdateOnly, MODE != kSumOnly, SS>(ta, xs, np, base, end, t0, t0_begin,
                                                                             t0_end, xb, wb, vb, hp);
    }
}

// Flat 256-element tiles with direct tile -> colour mapping, every colour adding the same
// compile-time number of terms, one wavefront per tile (MC_OPT_DIRECT_TILES = 2, and layouts
// without a unit table; the default launch is fused_unit_kernel below, which shares the scheme).
// The lookups are arranged in two batches, each issued as a whole before any of it is waited for:
//   1. what depends only on the tile index: the tile's tensor and the colour's P pointer tables;
//   2. what depends only on that tensor: its bounds and the P + 2 operand addresses.
// The decision which path the tile takes is ONE expression over all of them, evaluated without
// early exits, so every lookup is needed -- and therefore issued -- before the branch.  (Every
// dependent scalar load is a round trip of hundreds of cycles; left to source order, to early exits
// and to the compiler's habit of deferring a load into the branch that uses it, a tile had ten of
// them in a row in front of its first vector load: time a wavefront spends with nothing in flight.)
template <int P, int MODE, bool SS>
__global__ __launch_bounds__(64) void fused_direct_kernel(const int32_t* __restrict__ first_tensor,
                                                          const int64_t* __restrict__ off, float* const* w,
                                                          float* const* v, float* g, int32_t tiles_per_colour,
                                                          int32_t flip, int64_t range_hi, FusedArgs a) {
    // The eight scalars in front of the argument block are what a tile needs before its first
    // lookup; as leading arguments they are delivered in registers when the wavefront starts
    // (kernel-argument preload), so no load stands between the launch and batch 1.
    // flip: index of the last tile when the launch walks backwards, -1 otherwise.
    static_assert(P > 0 && MODE != kPerSegment, "uniform launches with a compile-time term count");
    constexpr int kTile = MC_COLOUR_ALIGN_ELEMS;
    constexpr bool HAS_G = MODE != kUpdateOnly, UPDATE = MODE != kSumOnly;
    const int blk = flip >= 0 ? flip - int(blockIdx.x) : int(blockIdx.x);

    // batch 1 (the argument-block fetches first: nothing here may wait for the table lookup)
    const int s = int(uint32_t(blk) / uint32_t(tiles_per_colour));
    const float* const* const* xs = a.x + s * P;
    const float* const* xt[P];
#pragma unroll
    for (int q = 0; q < P; ++q) xt[q] = xs[q];
    const mc::UpdateParams up = a.up;
    __builtin_amdgcn_sched_barrier(0);
    const int32_t t0 = first_tensor[blk];                       // tile == lookup granularity
    __builtin_amdgcn_sched_barrier(0);

    // batch 2
    typedef long long ll2 __attribute__((ext_vector_type(2)));
    ll2 t0_bounds;
    __builtin_memcpy(&t0_bounds, off + t0, sizeof(t0_bounds));
    const float* xb[P];
#pragma unroll
    for (int q = 0; q < P; ++q) xb[q] = xt[q][t0];
    float* wb = UPDATE ? w[t0] : nullptr;
    float* vb = UPDATE ? v[t0] : nullptr;
    __builtin_amdgcn_sched_barrier(0);
    const mc::Hyper hp = mc::resolve(up);

    const int64_t base = int64_t(blk) * kTile;
    const int64_t colour_end = int64_t(s + 1) * tiles_per_colour * kTile;
    const int64_t hi = colour_end < range_hi ? colour_end : range_hi;
    const int64_t end = base + kTile < hi ? base + kTile : hi;
    const int64_t rel = base - t0_bounds.x;
    // whole tile inside tensor t0 and every operand 16-byte aligned there?
    uintptr_t low_bits = 0;
#pragma unroll
    for (int q = 0; q < P; ++q) low_bits |= reinterpret_cast<uintptr_t>(xb[q] + rel);
    if (UPDATE) low_bits |= reinterpret_cast<uintptr_t>(wb + rel) | reinterpret_cast<uintptr_t>(vb + rel);
    const bool fast = (end - base == kTile) & (end <= t0_bounds.y) & ((low_bits & 15) == 0);
    if (fast) {
        const float* xp[P];
#pragma unroll
        for (int q = 0; q < P; ++q) xp[q] = xb[q] + rel;
        uniform_tile<P, 1, 64, HAS_G, UPDATE, SS, false>(xp, xs, P, t0, rel, UPDATE ? wb + rel : nullptr,
                                                          UPDATE ? vb + rel : nullptr, g + base, kTile / 4, hp);
        return;
    }
    const TileArgs ta = {w, v, g, off};
    fused_tile<P, 1, 64, HAS_G, UPDATE, SS>(ta, xs, P, base, end, t0, t0_bounds.x, t0_bounds.y, xb, wb, vb, hp);
}

// A unit that is not a whole, aligned 256-element run: the end of a tensor, a run cut by a colour
// bound, or operands that are not 16-byte aligned.  Lanes whose four elements all lie inside
// [e_lo, e_hi) use 128-bit accesses when the operands allow it, the rest go element by element.
template <int P, bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void partial_unit(const float* const* const* xs, const float* const* xb, float* wb, float* vb,
                                             float* const* w, float* const* v, float* g, int32_t t, int64_t rel,
                                             int64_t blk_lo, int64_t e_lo, int64_t e_hi, bool operands_aligned,
                                             const mc::Hyper& hp) {
    const int64_t e = blk_lo + int64_t(threadIdx.x) * 4;   // flat index of the lane's first element
    const int64_t r = rel + int64_t(threadIdx.x) * 4;      // the same element inside tensor t
    if (operands_aligned && e >= e_lo && e + 4 <= e_hi) {
        float4 acc = load4<true>(xb[0] + r);
#pragma unroll
        for (int q = 1; q < P; ++q) {
            const float4 x = load4<true>(xb[q] + r);
            acc.x = acc.x + x.x;
            acc.y = acc.y + x.y;
            acc.z = acc.z + x.z;
            acc.w = acc.w + x.w;
        }
        if (HAS_G) {
            if ((blk_lo & 3) == 0) {
                store4<true>(g + e, acc);
            } else {
                st1(g + e + 0, acc.x);
                st1(g + e + 1, acc.y);
                st1(g + e + 2, acc.z);
                st1(g + e + 3, acc.w);
            }
        }
        if (UPDATE) {
            float4 wq = mc::load_state<SS>(wb + r);
            float4 vq = mc::load_state<SS>(vb + r);
            mc::sgd(acc.x, wq.x, vq.x, hp);
            mc::sgd(acc.y, wq.y, vq.y, hp);
            mc::sgd(acc.z, wq.z, vq.z, hp);
            mc::sgd(acc.w, wq.w, vq.w, hp);
            mc::store_state<SS>(wb + r, wq, hp.state_store_sc1);
            mc::store_state<SS>(vb + r, vq, hp.state_store_sc1);
        }
        return;
    }
    for (int i = 0; i < 4; ++i) {
        const int64_t ee = e + i;
        if (ee >= e_lo && ee < e_hi) one_element<HAS_G, UPDATE>(xs, P, t, r + i, w, v, g, ee, hp);
    }
}

// The default launch of the fused step: tensor-aligned units (see mc_layout in mc_internal.h), one
// wavefront per unit.  A unit's tensor-side accesses start on a 1 KiB boundary of its tensor; only
// the flat gradient is reached at the tensor's flat offset.  (With flat tiles, one tensor whose length
// is not a multiple of 32 elements leaves every later tile's P + 2 tensor-side accesses straddling
// cache lines that the neighbouring tile, on another die, fetches again: GoogLeNet's step took 4 %
// longer for it, and a ResNet-50-sized payload split in two at an offset of 4 elements 5 %.)
// The eight scalars in front of the argument block arrive in registers when the wavefront starts
// (kernel-argument preload); the lookups then come in two batches, as in fused_direct_kernel:
// (1) the slot's tensor, and from the argument block the colour's P pointer tables, the chunk length
// and the hyper-parameters; (2) the tensor's bounds, the index of its first unit in the colour, and
// the P + 2 operand addresses.
// flip: index of the last slot when the launch walks backwards, -1 otherwise.
template <int P, int MODE, bool SS>
__global__ __launch_bounds__(64) void fused_unit_kernel(const int32_t* __restrict__ unit_tensor,
                                                        const int32_t* __restrict__ unit_first,
                                                        const int64_t* __restrict__ off, float* const* w,
                                                        float* const* v, int32_t units_per_colour, int32_t flip,
                                                        int64_t range_hi, FusedArgs a) {
    static_assert(P > 0 && MODE != kPerSegment, "uniform launches with a compile-time term count");
    constexpr int kUnit = MC_COLOUR_ALIGN_ELEMS;
    constexpr bool HAS_G = MODE != kUpdateOnly, UPDATE = MODE != kSumOnly;
    const int slot = flip >= 0 ? flip - int(blockIdx.x) : int(blockIdx.x);

    // batch 1
    const int c = int(uint32_t(slot) / uint32_t(units_per_colour));
    const int local = slot - c * units_per_colour;
    const float* const* const* xs = a.x + c * P;
    const float* const* xt[P];
#pragma unroll
    for (int q = 0; q < P; ++q) xt[q] = xs[q];
    const int64_t chunk = a.chunk;
    float* const g = a.g;
    const mc::UpdateParams up = a.up;
    __builtin_amdgcn_sched_barrier(0);
    const int32_t t_raw = unit_tensor[slot];
    __builtin_amdgcn_sched_barrier(0);
    // (A padding slot holds -1.  It leaves only after batch 2 has been issued, with tensor 0 standing in
    // for the lookups: a branch here would push every fetch above to the far side of it.)
    const int32_t t = t_raw < 0 ? 0 : t_raw;

    // batch 2
    typedef long long ll2 __attribute__((ext_vector_type(2)));
    ll2 bounds;
    __builtin_memcpy(&bounds, off + t, sizeof(bounds));
    const int32_t first = unit_first[c + t];
    const float* xb[P];
#pragma unroll
    for (int q = 0; q < P; ++q) xb[q] = xt[q][t];
    float* wb = UPDATE ? w[t] : nullptr;
    float* vb = UPDATE ? v[t] : nullptr;
    __builtin_amdgcn_sched_barrier(0);
    if (t_raw < 0) return;
    const mc::Hyper hp = mc::resolve(up);

    const int64_t c_lo = int64_t(c) * chunk;
    const int64_t c_end = c_lo + chunk;
    const int64_t c_hi = c_end < range_hi ? c_end : range_hi;
    const int64_t lo = c_lo > bounds.x ? c_lo : bounds.x;      // the tensor's part in this colour
    const int64_t hi = c_hi < bounds.y ? c_hi : bounds.y;
    const int64_t j = ((lo - bounds.x) >> 8) + (local - first);
    static_assert(kUnit == 256, "the shift above");
    const int64_t rel = j * kUnit;                             // first element of the run, inside the tensor
    const int64_t blk_lo = bounds.x + rel;                     // ... and in the flat payload
    const int64_t e_lo = blk_lo > lo ? blk_lo : lo;
    const int64_t e_hi = blk_lo + kUnit < hi ? blk_lo + kUnit : hi;
    uintptr_t low_bits = 0;
#pragma unroll
    for (int q = 0; q < P; ++q) low_bits |= reinterpret_cast<uintptr_t>(xb[q]);
    if (UPDATE) low_bits |= reinterpret_cast<uintptr_t>(wb) | reinterpret_cast<uintptr_t>(vb);
    const bool aligned = (low_bits & 15) == 0;
    const bool whole = (e_lo == blk_lo) & (e_hi == blk_lo + kUnit) & aligned;
    if (!whole) {
        partial_unit<P, HAS_G, UPDATE, SS>(xs, xb, wb, vb, w, v, g, t, rel, blk_lo, e_lo, e_hi, aligned, hp);
        return;
    }
    // A whole run: every load of the unit is issued before the first add.
    const int64_t r = rel + int64_t(threadIdx.x) * 4;
    float4 term[P], wq, vq;
#pragma unroll
    for (int q = 0; q < P; ++q) term[q] = load4<true>(xb[q] + r);
    if (UPDATE) {
        wq = mc::load_state<SS>(wb + r);
        vq = mc::load_state<SS>(vb + r);
    }
    float4 acc = term[0];
#pragma unroll
    for (int q = 1; q < P; ++q) {
        acc.x = acc.x + term[q].x;
        acc.y = acc.y + term[q].y;
        acc.z = acc.z + term[q].z;
        acc.w = acc.w + term[q].w;
    }
    if (HAS_G) {
        float* gq = g + blk_lo + int64_t(threadIdx.x) * 4;
        if ((blk_lo & 3) == 0) {
            store4<true>(gq, acc);
        } else {   // the tensor's flat offset is not a multiple of four elements: word by word
            st1(gq + 0, acc.x);
            st1(gq + 1, acc.y);
            st1(gq + 2, acc.z);
            st1(gq + 3, acc.w);
        }
    }
    if (UPDATE) {
        mc::sgd(acc.x, wq.x, vq.x, hp);
        mc::sgd(acc.y, wq.y, vq.y, hp);
        mc::sgd(acc.z, wq.z, vq.z, hp);
        mc::sgd(acc.w, wq.w, vq.w, hp);
        mc::store_state<SS>(wb + r, wq, hp.state_store_sc1);
        mc::store_state<SS>(vb + r, vq, hp.state_store_sc1);
    }
}

// One unit of a colour with a run-time term count np (1..8): the body of fused_unit_roles_kernel.
// Loads are guarded by uniform tests of np, so indexing stays static and nothing beyond the colour's
// pointer list is touched.
template <bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void roles_unit(const float* const* const* xs, int np, const float* const* xb, float* wb,
                                           float* vb, float* const* w, float* const* v, float* g, int32_t t,
                                           int64_t rel, int64_t blk_lo, int64_t e_lo, int64_t e_hi, bool aligned,
                                           const mc::Hyper& hp) {
    constexpr int kMost = 8;
    const int64_t e = blk_lo + int64_t(threadIdx.x) * 4;   // flat index of the lane's first element
    const int64_t r = rel + int64_t(threadIdx.x) * 4;      // the same element inside tensor t
    const bool whole = (e_lo == blk_lo) & (e_hi == blk_lo + MC_COLOUR_ALIGN_ELEMS) & aligned;
    if (whole || (aligned && e >= e_lo && e + 4 <= e_hi)) {
        float4 term[kMost], wq, vq;
#pragma unroll
        for (int q = 0; q < kMost; ++q)
            if (q < np) term[q] = load4<true>(xb[q] + r);
        if (UPDATE) {
            wq = mc::load_state<SS>(wb + r);
            vq = mc::load_state<SS>(vb + r);
        }
        float4 acc = term[0];
#pragma unroll
        for (int q = 1; q < kMost; ++q) {
            if (q < np) {
                acc.x = acc.x + term[q].x;
                acc.y = acc.y + term[q].y;
                acc.z = acc.z + term[q].z;
                acc.w = acc.w + term[q].w;
            }
        }
        if (HAS_G) {
            if ((blk_lo & 3) == 0) {
                store4<true>(g + e, acc);
            } else {
                st1(g + e + 0, acc.x);
                st1(g + e + 1, acc.y);
                st1(g + e + 2, acc.z);
                st1(g + e + 3, acc.w);
            }
        }
        if (UPDATE) {
            mc::sgd(acc.x, wq.x, vq.x, hp);
            mc::sgd(acc.y, wq.y, vq.y, hp);
            mc::sgd(acc.z, wq.z, vq.z, hp);
            mc::sgd(acc.w, wq.w, vq.w, hp);
            mc::store_state<SS>(wb + r, wq, hp.state_store_sc1);
            mc::store_state<SS>(vb + r, vq, hp.state_store_sc1);
        }
        return;
    }
    for (int i = 0; i < 4; ++i) {
        const int64_t ee = e + i;
        if (ee >= e_lo && ee < e_hi) one_element<HAS_G, UPDATE>(xs, np, t, r + i, w, v, g, ee, hp);
    }
}

// Tensor-aligned units for a launch whose colours differ in term count or update flag (a rank's
// role-dependent step on per-layer tensors, Section 4.2), every count at most eight.  As
// fused_unit_kernel, with one more fetch in front: the colour's descriptor word (first pointer slot,
// term count, update flag) comes from the argument block before its pointer tables can be read.
template <bool SS>
__global__ __launch_bounds__(64) void fused_unit_roles_kernel(const int32_t* __restrict__ unit_tensor,
                                                              const int32_t* __restrict__ unit_first,
                                                              const int64_t* __restrict__ off, float* const* w,
                                                              float* const* v, int32_t units_per_colour, int32_t flip,
                                                              int64_t range_hi, FusedArgs a) {
    constexpr int kUnit = MC_COLOUR_ALIGN_ELEMS;
    constexpr int kMost = 8;
    const int slot = flip >= 0 ? flip - int(blockIdx.x) : int(blockIdx.x);
    const int c = int(uint32_t(slot) / uint32_t(units_per_colour));
    const int local = slot - c * units_per_colour;
    const uint32_t info = a.seg_info[c];
    const int64_t chunk = a.chunk;
    float* const g = a.g;
    const mc::UpdateParams up = a.up;
    const int32_t t_raw = unit_tensor[slot];
    __builtin_amdgcn_sched_barrier(0);
    const int np = int((info >> 16) & 0xffu);
    if (np == 0 || t_raw < 0) return;                // a colour this call skips, or a padding slot
    const bool update = ((info >> 24) & 1u) != 0;
    const int32_t t = t_raw;
    const float* const* const* xs = a.x + int(info & 0xffffu);
    const float* const* xt[kMost];
#pragma unroll
    for (int q = 0; q < kMost; ++q) {
        xt[q] = nullptr;
        if (q < np) xt[q] = xs[q];
    }
    __builtin_amdgcn_sched_barrier(0);
    typedef long long ll2 __attribute__((ext_vector_type(2)));
    ll2 bounds;
    __builtin_memcpy(&bounds, off + t, sizeof(bounds));
    const int32_t first = unit_first[c + t];
    const float* xb[kMost];
#pragma unroll
    for (int q = 0; q < kMost; ++q) {
        xb[q] = nullptr;
        if (q < np) xb[q] = xt[q][t];
    }
    float* wb = nullptr;
    float* vb = nullptr;
    if (update) {
        wb = w[t];
        vb = v[t];
    }
    __builtin_amdgcn_sched_barrier(0);
    const mc::Hyper hp = mc::resolve(up);

    const int64_t c_lo = int64_t(c) * chunk;
    const int64_t c_end = c_lo + chunk;
    const int64_t c_hi = c_end < range_hi ? c_end : range_hi;
    const int64_t lo = c_lo > bounds.x ? c_lo : bounds.x;
    const int64_t hi = c_hi < bounds.y ? c_hi : bounds.y;
    const int64_t j = ((lo - bounds.x) >> 8) + (local - first);
    static_assert(kUnit == 256, "the shift above");
    const int64_t rel = j * kUnit;
    const int64_t blk_lo = bounds.x + rel;
    const int64_t e_lo = blk_lo > lo ? blk_lo : lo;
    const int64_t e_hi = blk_lo + kUnit < hi ? blk_lo + kUnit : hi;
    uintptr_t low_bits = reinterpret_cast<uintptr_t>(wb) | reinterpret_cast<uintptr_t>(vb);
#pragma unroll
    for (int q = 0; q < kMost; ++q) low_bits |= reinterpret_cast<uintptr_t>(xb[q]);
    const bool aligned = (low_bits & 15) == 0;
    if (update) {
        if (g)
            roles_unit<true, true, SS>(xs, np, xb, wb, vb, w, v, g, t, rel, blk_lo, e_lo, e_hi, aligned, hp);
        else
            roles_unit<false, true, SS>(xs, np, xb, wb, vb, w, v, g, t, rel, blk_lo, e_lo, e_hi, aligned, hp);
    } else {
        roles_unit<true, false, SS>(xs, np, xb, wb, vb, w, v, g, t, rel, blk_lo, e_lo, e_hi, aligned, hp);
    }
}

void launch_unit_roles(bool ss, hipStream_t s, const FusedArgs& a, const mc::DeviceTables* dt, int32_t units_per_colour,
                       int32_t k) {
    const unsigned blocks = unsigned(units_per_colour) * unsigned(k);
    const dim3 grid(blocks), block(64);
    const int32_t flip = a.reverse ? int32_t(blocks) - 1 : -1;
    if (ss)
        hipLaunchKernelGGL((fused_unit_roles_kernel<true>), grid, block, a.lds_per_wave, s, dt->unit_tensor, dt->unit_first,
                           a.off, a.w, a.v, units_per_colour, flip, a.range_hi, a);
    else
        hipLaunchKernelGGL((fused_unit_roles_kernel<false>), grid, block, a.lds_per_wave, s, dt->unit_tensor, dt->unit_first,
                           a.off, a.w, a.v, units_per_colour, flip, a.range_hi, a);
}

template <int P>
void launch_unit_mode(int mode, bool ss, hipStream_t s, const FusedArgs& a, const mc::DeviceTables* dt,
                      int32_t units_per_colour, int32_t k) {
    const unsigned blocks = unsigned(units_per_colour) * unsigned(k);
    const dim3 grid(blocks), block(64);
    const int32_t flip = a.reverse ? int32_t(blocks) - 1 : -1;
#define MC_FUSED_LAUNCH(MODE, SS)                                                                               \
    hipLaunchKernelGGL((fused_unit_kernel<P, MODE, SS>), grid, block, a.lds_per_wave, s, dt->unit_tensor,          \
                       dt->unit_first, a.off, a.w, a.v, units_per_colour, flip, a.range_hi, a)
    switch (mode) {
        case kSumOnly: MC_FUSED_LAUNCH(kSumOnly, false); break;
        case kUpdateAndG: if (ss) MC_FUSED_LAUNCH(kUpdateAndG, true); else MC_FUSED_LAUNCH(kUpdateAndG, false); break;
        default: if (ss) MC_FUSED_LAUNCH(kUpdateOnly, true); else MC_FUSED_LAUNCH(kUpdateOnly, false); break;
    }
#undef MC_FUSED_LAUNCH
}

void launch_units(int P, int mode, bool ss, hipStream_t s, const FusedArgs& a, const mc::DeviceTables* dt,
                  int32_t units_per_colour, int32_t k) {
    switch (P) {
        case 1: launch_unit_mode<1>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 2: launch_unit_mode<2>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 3: launch_unit_mode<3>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 4: launch_unit_mode<4>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 5: launch_unit_mode<5>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 6: launch_unit_mode<6>(mode, ss, s, a, dt, units_per_colour, k); break;
        case 7: launch_unit_mode<7>(mode, ss, s, a, dt, units_per_colour, k); break;
        default: launch_unit_mode<8>(mode, ss, s, a, dt, units_per_colour, k); break;
    }
}

template <int P>
void launch_direct_mode(int mode, bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a) {
    const dim3 grid(blocks), block(64);
    const int32_t flip = a.reverse ? int32_t(blocks) - 1 : -1;
#define MC_FUSED_LAUNCH(MODE, SS)                                                                                       \
    hipLaunchKernelGGL((fused_direct_kernel<P, MODE, SS>), grid, block, a.lds_per_wave, s, \
                       a.first_tensor, a.off, a.w, a.v, a.g, a.tiles_per_colour, flip, a.range_hi, a)
    switch (mode) {
        case kSumOnly: MC_FUSED_LAUNCH(kSumOnly, false); break;
        case kUpdateAndG: if (ss) MC_FUSED_LAUNCH(kUpdateAndG, true); else MC_FUSED_LAUNCH(kUpdateAndG, false); break;
        default: if (ss) MC_FUSED_LAUNCH(kUpdateOnly, true); else MC_FUSED_LAUNCH(kUpdateOnly, false); break;
    }
#undef MC_FUSED_LAUNCH
}

void launch_direct(int P, int mode, bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a) {
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
void launch_mode(int mode, bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a, int Prt) {
    const dim3 grid(blocks), block(T);
#define MC_FUSED_LAUNCH(MODE, SS) hipLaunchKernelGGL((fused_step_kernel<P, U, T, MODE, SS>), grid, block, (T == 64 ? a.lds_per_wave : a.lds_per_4waves), s, a, Prt)
    switch (mode) {
        case kSumOnly: MC_FUSED_LAUNCH(kSumOnly, false); break;   // state is not touched: one policy
        case kUpdateAndG: if (ss) MC_FUSED_LAUNCH(kUpdateAndG, true); else MC_FUSED_LAUNCH(kUpdateAndG, false); break;
        default: if (ss) MC_FUSED_LAUNCH(kUpdateOnly, true); else MC_FUSED_LAUNCH(kUpdateOnly, false); break;
    }
#undef MC_FUSED_LAUNCH
}

template <int P>
void launch_shape(mc::Shape shape, int mode, bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a, int Prt) {
    if (shape.threads == 64)
        launch_mode<P, 1, 64>(mode, ss, blocks, s, a, Prt);
    else
        launch_mode<P, 2, 256>(mode, ss, blocks, s, a, Prt);
}

// A launch whose segments all add P terms and agree on updating.
void launch(int P, mc::Shape shape, int mode, bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a) {
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
void launch_per_segment(bool ss, unsigned blocks, hipStream_t s, const FusedArgs& a) {
    const dim3 grid(blocks), block(64);
    if (ss)
        hipLaunchKernelGGL((fused_step_kernel<0, 1, 64, kPerSegment, true>), grid, block, a.lds_per_wave, s, a, 0);
    else
        hipLaunchKernelGGL((fused_step_kernel<0, 1, 64, kPerSegment, false>), grid, block, a.lds_per_wave, s, a, 0);
}

// Do two sorted lists of [begin, end) spans intersect anywhere?
bool spans_overlap(const std::vector<std::pair<uintptr_t, uintptr_t>>& A,
                   const std::vector<std::pair<uintptr_t, uintptr_t>>& B) {
    size_t i = 0, j = 0;
    while (i < A.size() && j < B.size()) {
        if (A[i].second <= B[j].first)
            ++i;
        else if (B[j].second <= A[i].first)
            ++j;
        else
            return true;
    }
    return false;
}

}  // namespace

extern "C" {

int mc_tensor_set_create(mc_layout* L, const void* const* tensors, mc_tensor_set** out) {
    if (out) *out = nullptr;
    if (!L || !tensors || !out) return MC_ERR_INVALID_ARG;
    mc_tensor_set* S = new (std::nothrow) mc_tensor_set;
    if (!S) return MC_ERR_ALLOC;
    S->layout = L;
    try {
        S->ptrs.assign(tensors, tensors + L->n);
        for (int32_t t = 0; t < L->n; ++t) {
            const int64_t cnt = L->off[t + 1] - L->off[t];
            if (cnt == 0) continue;
            if (!tensors[t]) {
                delete S;
                return MC_ERR_INVALID_ARG;
            }
            if (!mc::aligned(tensors[t], 4)) {
                delete S;
                return MC_ERR_ALIGN;
            }
            const uintptr_t b = reinterpret_cast<uintptr_t>(tensors[t]);
            S->spans.emplace_back(b, b + uintptr_t(cnt) * 4);
        }
        std::sort(S->spans.begin(), S->spans.end());
        for (size_t i = 1; i < S->spans.size(); ++i) {
            if (S->spans[i].first < S->spans[i - 1].second) {
                delete S;
                return MC_ERR_OVERLAP;
            }
        }
    } catch (const std::bad_alloc&) {
        delete S;
        return MC_ERR_ALLOC;
    }
    const mc::DeviceTables* dt = nullptr;
    int rc = mc::device_tables(L, &dt);  // the kernels that read a set also read the layout's tables
    if (rc == MC_OK) {
        hipError_t e = hipGetDevice(&S->device);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&S->d_ptrs), size_t(L->n) * sizeof(void*));
        if (e == hipSuccess)
            e = hipMemcpy(S->d_ptrs, S->ptrs.data(), size_t(L->n) * sizeof(void*), hipMemcpyHostToDevice);
        if (e != hipSuccess) rc = mc::hip_fail(e);
    }
    if (rc != MC_OK) {
        if (S->d_ptrs) (void)hipFree(S->d_ptrs);
        delete S;
        return rc;
    }
    *out = S;
    return MC_OK;
}

int mc_tensor_set_destroy(mc_tensor_set* S) {
    if (!S) return MC_OK;
    int rc = MC_OK;
    if (S->d_ptrs) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e == hipSuccess && cur != S->device) e = hipSetDevice(S->device);
        if (e == hipSuccess) e = hipFree(S->d_ptrs);
        if (e != hipSuccess) rc = mc::hip_fail(e);
        if (cur >= 0 && cur != S->device) (void)hipSetDevice(cur);
    }
    delete S;
    return rc;
}

static int fused_run_impl(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                          const int32_t* n_terms, const uint8_t* do_update, void* grad_out,
                          const mc_tensor_set* weights, const mc_tensor_set* momentum,
                          const mc::UpdatePlan& plan, void* stream) {
    if (!L || !contrib || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
    if ((n_terms == nullptr) != (do_update == nullptr)) return MC_ERR_INVALID_ARG;
    if (plan.up.hyper && !mc::aligned(plan.up.hyper, 4)) return MC_ERR_ALIGN;
    if ((weights && weights->layout != L) || (momentum && momentum->layout != L)) return MC_ERR_INVALID_ARG;
    for (int32_t p = 0; p < P; ++p)
        if (!contrib[p] || contrib[p]->layout != L) return MC_ERR_INVALID_ARG;
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
    auto terms = [&](int32_t c) { return n_terms ? n_terms[c] : P; };
    auto updates = [&](int32_t c) { return do_update ? do_update[c] != 0 : true; };
    auto active = [&](int32_t c) { return terms(c) > 0 && L->bounds[c + 1] > L->bounds[c]; };
    bool any_update = false, any_sum_only = false, uniform = true, any_skipped = false;
    int32_t first_active = -1;
    int max_terms = 0, total_terms = 0;
    for (int32_t c = 0; c < L->k; ++c) {
        if (n_terms && (n_terms[c] < 0 || n_terms[c] > P)) return MC_ERR_INVALID_ARG;
        if (terms(c) == 0 && L->bounds[c + 1] > L->bounds[c]) any_skipped = true;
        if (!active(c)) continue;
        if (updates(c)) any_update = true; else any_sum_only = true;
        max_terms = std::max(max_terms, int(terms(c)));
        total_terms += terms(c);
        if (first_active < 0) first_active = c;
        else if (terms(c) != terms(first_active) || updates(c) != updates(first_active)) uniform = false;
    }
    if (first_active < 0) return MC_OK;
    if (any_update && (!weights || !momentum)) return MC_ERR_INVALID_ARG;
    if (any_sum_only && !grad_out) return MC_ERR_INVALID_ARG;
    if (grad_out && !mc::aligned(grad_out, 16)) return MC_ERR_ALIGN;

    // Nothing written (weights, momentum, grad_out) may overlap anything else of the call.
    // A contribution may appear twice (it is only read).
    const mc_tensor_set* written[2] = {weights, momentum};
    if (weights && momentum && spans_overlap(weights->spans, momentum->spans)) return MC_ERR_OVERLAP;
    std::vector<std::pair<uintptr_t, uintptr_t>> gspan;
    if (grad_out) {
        const uintptr_t b = reinterpret_cast<uintptr_t>(grad_out);
        gspan.emplace_back(b, b + uintptr_t(L->N) * 4);
        for (const mc_tensor_set* wset : written)
            if (wset && spans_overlap(wset->spans, gspan)) return MC_ERR_OVERLAP;
    }
    for (int32_t p = 0; p < P; ++p) {
        for (const mc_tensor_set* wset : written)
            if (wset && spans_overlap(contrib[p]->spans, wset->spans)) return MC_ERR_OVERLAP;
        if (grad_out && spans_overlap(contrib[p]->spans, gspan)) return MC_ERR_OVERLAP;
    }

    const mc::DeviceTables* dt = nullptr;
    const int rc = mc::device_tables(L, &dt);
    if (rc != MC_OK) return rc;
    int dev = -1;
    MC_HIP_TRY(hipGetDevice(&dev));
    if ((weights && weights->device != dev) || (momentum && momentum->device != dev)) return MC_ERR_INVALID_ARG;
    for (int32_t p = 0; p < P; ++p)
        if (contrib[p]->device != dev) return MC_ERR_INVALID_ARG;

    const bool ss = any_update && mc::stream_state(L, plan.state_policy);
    // Launches that mix term counts or update flags use the one-wavefront shape.
    const mc::Shape shape = uniform ? mc::shape_for(L->N, max_terms, ss) : mc::Shape{64, 1};
    const int64_t tile = shape.tile();
    hipStream_t s = static_cast<hipStream_t>(stream);

    FusedArgs a;
    // Only the plain whole-payload step alternates by itself: role calls come several to a step.
    a.reverse = mc::sweep_reversed(L, (n_terms && plan.sweep == MC_SWEEP_AUTO) ? MC_SWEEP_FORWARD : plan.sweep, ss) ? 1 : 0;
    a.xcd_run = mc::option(MC_OPT_XCD_RUN);
    {
        const int avg_terms = uniform ? int(terms(first_active)) : 0;
        const bool state_cached = !ss && !any_sum_only;
        a.lds_per_wave = mc::update_lds_reservation(L, 64, state_cached, avg_terms, true);
        a.lds_per_4waves = mc::update_lds_reservation(L, 256, state_cached, avg_terms, true);
    }
    a.w = weights ? reinterpret_cast<float* const*>(weights->d_ptrs) : nullptr;
    a.v = momentum ? reinterpret_cast<float* const*>(momentum->d_ptrs) : nullptr;
    a.g = static_cast<float*>(grad_out);
    a.off = dt->off;
    a.first_tensor = dt->tile_first;
    a.up = plan.up;

    a.tiles_per_colour = 0;
    a.range_hi = L->N;
    a.chunk = 0;
    auto pointer_list = [&](int32_t c, int slot) {
        for (int32_t q = 0; q < terms(c); ++q)
            a.x[slot + q] = reinterpret_cast<const float* const*>(contrib[order ? order[size_t(c) * P + q] : q]->d_ptrs);
    };

    // Direct mapping: a 256-element tile is exactly the colour alignment, so the tiles of the call are
    // the 256-element runs of the payload and a tile's colour is its index divided by the chunk
    // length.  Needs every colour's pointer list in the one launch.
    const int64_t tiles_total = (L->N + tile - 1) / tile;
    // (A call whose colours agree but for some it skips keeps the table, which simply leaves the
    // skipped colours out and still runs the compile-time body.)
    const int slots_needed = uniform ? L->k * terms(first_active) : total_terms;
    if (tile == MC_COLOUR_ALIGN_ELEMS && !(uniform && any_skipped) && L->k <= kMaxSegs && slots_needed <= kPtrSlots &&
        tiles_total < 0x7fffffff && mc::option(MC_OPT_DIRECT_TILES) != 0) {
        a.tiles_per_colour = int32_t(L->chunk / tile);
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
                // (Every colour, an empty one too: a padding slot of the unit kernel reads its colour's
                // tables before it leaves.)
                for (int32_t q = 0; q < terms(first_active); ++q)
                    a.x[c * terms(first_active) + q] =
                        reinterpret_cast<const float* const*>(contrib[order ? order[size_t(c) * P + q] : q]->d_ptrs);
            } else if (active(c)) {
                a.seg_info[c] = uint32_t(slots) | (uint32_t(terms(c)) << 16) | (updates(c) ? (1u << 24) : 0u);
                pointer_list(c, slots);
                slots += terms(c);
            }
        }
        if (per_segment) {
            if (max_terms <= 8 && a.xcd_run < 2 && dt->unit_tensor && mc::option(MC_OPT_DIRECT_TILES) == 1) {
                a.chunk = L->chunk;
                launch_unit_roles(ss, s, a, dt, L->units_per_colour, L->k);
            } else {
                launch_per_segment(ss, unsigned(tiles_total), s, a);
            }
        } else {
            const int mode = !updates(first_active) ? kSumOnly : (a.g ? kUpdateAndG : kUpdateOnly);
            const bool few = terms(first_active) <= 8 && a.xcd_run < 2;   // (a run of tiles per die is the general kernel's)
            if (few && dt->unit_tensor && mc::option(MC_OPT_DIRECT_TILES) == 1) {
                a.chunk = L->chunk;
                launch_units(terms(first_active), mode, ss, s, a, dt, L->units_per_colour, L->k);
            } else if (few)
                launch_direct(terms(first_active), mode, ss, unsigned(tiles_total), s, a);
            else
                launch(terms(first_active), shape, mode, ss, unsigned(tiles_total), s, a);
        }
        MC_HIP_TRY(hipGetLastError());
        return MC_OK;
    }

    // Otherwise colours in index order, as many per launch as the segment and pointer slots hold, each
    // with its own run of workgroups (a prefix table maps a workgroup to its segment).
    int32_t c = 0;
    while (c < L->k) {
        int ns = 0, slots = 0;
        int64_t blocks = 0;
        a.first_block[0] = 0;
        for (; c < L->k && ns < kMaxSegs; ++c) {
            if (!active(c)) continue;
            const int32_t cnt = terms(c);
            if (slots + cnt > kPtrSlots) break;
            const int64_t lo = L->bounds[c], hi = L->bounds[c + 1];
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
static int fused_run(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                     const int32_t* n_terms, const uint8_t* do_update, void* grad_out,
                     const mc_tensor_set* weights, const mc_tensor_set* momentum,
                     const mc::UpdatePlan& plan, void* stream) {
    try {
        return fused_run_impl(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, plan, stream);
    } catch (const std::bad_alloc&) {
        return MC_ERR_ALLOC;
    }
}

int mc_fused_step(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                  void* grad_out, const mc_tensor_set* weights, const mc_tensor_set* momentum,
                  float lr, float mu, float wd, void* stream) {
    mc::UpdatePlan plan;
    plan.up.lr = lr;
    plan.up.mu = mu;
    plan.up.wd = wd;
    plan.up.hyper = nullptr;
    plan.up.nesterov = 0;
    plan.up.state_store_sc1 = mc::option(MC_OPT_STATE_STORE_SC1);
    plan.state_policy = MC_STATE_DEFAULT;
    plan.sweep = MC_SWEEP_AUTO;
    if (!weights || !momentum) return MC_ERR_INVALID_ARG;
    return fused_run(L, contrib, P, order, nullptr, nullptr, grad_out, weights, momentum, plan, stream);
}

int mc_fused_step_ex(mc_layout* L, const mc_tensor_set* const* contrib, int32_t P, const int32_t* order,
                     const int32_t* n_terms, const uint8_t* do_update, void* grad_out,
                     const mc_tensor_set* weights, const mc_tensor_set* momentum,
                     const mc_update_spec* spec, void* stream) {
    mc::UpdatePlan plan;
    const int rc = mc::update_plan(spec, &plan);
    if (rc != MC_OK) return rc;
    return fused_run(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, plan, stream);
}

}  // extern "C"
