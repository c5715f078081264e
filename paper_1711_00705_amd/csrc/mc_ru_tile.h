// One tile of the per-colour, fixed-order sum fused with the SGD update: the device code shared by
// the reduce_update kernels and the packet-driven reducer.
//
// Arithmetic is written operation by operation and every file that includes this header is compiled
// with floating-point contraction off, so each add and multiply is rounded once to binary32 exactly
// as in the definition (Section 3, Algorithm 1: sum, then SGD); denormals are preserved.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "mc_update.h"

#pragma clang fp contract(off)

namespace mc {

typedef float native_f4 __attribute__((ext_vector_type(4)));

// Contributions and the reduced gradient are touched once per step: streaming (non-temporal)
// accesses, so that they do not displace weights and momentum from the caches.
__device__ __forceinline__ float4 load_stream(const float* p) {
    const native_f4 r = __builtin_nontemporal_load(reinterpret_cast<const native_f4*>(p));
    return make_float4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ void store_stream(float* p, const float4& q) {
    const native_f4 val = {q.x, q.y, q.z, q.w};
    __builtin_nontemporal_store(val, reinterpret_cast<native_f4*>(p));
}

// One tile of one segment.  P > 0: compile-time number of terms; P == 0: run-time count `np`
// (up to MC_MAX_P).  UPDATE: the SGD step follows the sum; otherwise only the sum is written to g
// and w, v are never touched.  SS: weights and momentum are streamed instead of kept resident.
template <int P, int U, int THREADS, bool HAS_G, bool UPDATE, bool SS>
__device__ __forceinline__ void ru_tile(const float* const* xs, int np, int64_t base, int64_t hi, float* g,
                                        float* w, float* v, const mc::Hyper& hp) {
    static_assert(HAS_G || UPDATE, "a tile must produce something");
    constexpr int64_t kTile = int64_t(THREADS) * 4 * U;
    if (base + kTile <= hi) {
        // Full tile: issue every load of the tile before the first add.
        float4 acc[U], wv[U], vv[U];
        int64_t idx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) idx[u] = base + (int64_t(u) * THREADS + threadIdx.x) * 4;
        if (P > 0) {
            float4 t[P > 0 ? P : 1][U];
#pragma unroll
            for (int q = 0; q < P; ++q)
#pragma unroll
                for (int u = 0; u < U; ++u) t[q][u] = load_stream(xs[q] + idx[u]);
            if (UPDATE) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    wv[u] = mc::load_state<SS>(w + idx[u]);
                    vv[u] = mc::load_state<SS>(v + idx[u]);
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
            // contributions) are loaded together, each load guarded by a uniform test of the run-time
            // count.  Larger counts load the first term, then four at a time: more loads per wavefront
            // measured 3-5 % slower there.  The adds run strictly left to right either way.
            constexpr int kFirst = U == 1 ? 8 : 4;
            int q;
            if (np <= kFirst) {
                float4 first[kFirst][U];
#pragma unroll
                for (int r = 0; r < kFirst; ++r) {
                    if (r < np) {
#pragma unroll
                        for (int u = 0; u < U; ++u) first[r][u] = load_stream(xs[r] + idx[u]);
                    }
                }
                if (UPDATE) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        wv[u] = mc::load_state<SS>(w + idx[u]);
                        vv[u] = mc::load_state<SS>(v + idx[u]);
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
                    if (UPDATE) {
                        wv[u] = mc::load_state<SS>(w + idx[u]);
                        vv[u] = mc::load_state<SS>(v + idx[u]);
                    }
                    acc[u] = load_stream(xs[0] + idx[u]);
                }
                q = 1;
            }
            for (; q + 4 <= np; q += 4) {
                float4 t[4][U];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int u = 0; u < U; ++u) t[r][u] = load_stream(xs[q + r] + idx[u]);
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
                const float* xq = xs[q];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float4 t = load_stream(xq + idx[u]);
                    acc[u].x = acc[u].x + t.x;
                    acc[u].y = acc[u].y + t.y;
                    acc[u].z = acc[u].z + t.z;
                    acc[u].w = acc[u].w + t.w;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (HAS_G) store_stream(g + idx[u], acc[u]);
            if (UPDATE) {
                mc::sgd(acc[u].x, wv[u].x, vv[u].x, hp);
                mc::sgd(acc[u].y, wv[u].y, vv[u].y, hp);
                mc::sgd(acc[u].z, wv[u].z, vv[u].z, hp);
                mc::sgd(acc[u].w, wv[u].w, vv[u].w, hp);
                mc::store_state<SS>(w + idx[u], wv[u], hp.state_store_sc1);
                mc::store_state<SS>(v + idx[u], vv[u], hp.state_store_sc1);
            }
        }
        return;
    }

    // Last, partial tile of the segment: whole vectors while they fit, then single elements.
    // (Segments start on multiples of 256 elements, so base is 16-byte aligned; hi need not be.)
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t(u) * THREADS + threadIdx.x) * 4;
        if (i >= hi) break;
        if (i + 4 <= hi) {
            float4 acc = load_stream(xs[0] + i);
            for (int q = 1; q < np; ++q) {
                const float4 t = load_stream(xs[q] + i);
                acc.x = acc.x + t.x;
                acc.y = acc.y + t.y;
                acc.z = acc.z + t.z;
                acc.w = acc.w + t.w;
            }
            if (HAS_G) *reinterpret_cast<float4*>(g + i) = acc;
            if (UPDATE) {
                float4 wq = *reinterpret_cast<const float4*>(w + i);
                float4 vq = *reinterpret_cast<const float4*>(v + i);
                mc::sgd(acc.x, wq.x, vq.x, hp);
                mc::sgd(acc.y, wq.y, vq.y, hp);
                mc::sgd(acc.z, wq.z, vq.z, hp);
                mc::sgd(acc.w, wq.w, vq.w, hp);
                *reinterpret_cast<float4*>(w + i) = wq;
                *reinterpret_cast<float4*>(v + i) = vq;
            }
        } else {
            for (int64_t e = i; e < hi; ++e) {
                float acc = xs[0][e];
                for (int q = 1; q < np; ++q) acc = acc + xs[q][e];
                if (HAS_G) g[e] = acc;
                if (UPDATE) {
                    float we = w[e], ve = v[e];
                    mc::sgd(acc, we, ve, hp);
                    w[e] = we;
                    v[e] = ve;
                }
            }
        }
    }
}

}  // namespace mc
