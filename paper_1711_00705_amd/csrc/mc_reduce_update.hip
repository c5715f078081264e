// a3 + a4: per-colour, fixed-order sum of P contributions fused with the SGD update.
//
// The pass is pure streaming: per element it reads P + 2 words and writes 2 or 3, with P + 4
// flops, so it is bound by HBM bandwidth and the kernel's only job is to keep enough 128-bit
// loads in flight.  The grid is partitioned by colour: each colour owns a contiguous run of
// workgroups (a prefix table in the kernel arguments maps blockIdx -> colour), and the
// colour's summation sequence is applied by handing that colour its own, already permuted,
// list of contribution pointers.  Colours never synchronise with each other (Section 4.2).
//
// Arithmetic is written operation by operation and the file is compiled with floating-point
// contraction off, so each add and multiply is rounded once to binary32 exactly as in the
// definition; denormals are preserved (HIP's default for fp32 on gfx9).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "mc_internal.h"

#pragma clang fp contract(off)

namespace {

constexpr int kThreads = 256;  // workgroup size
constexpr int kMaxSegs = 32;     // colours per launch
constexpr int kPtrSlots = 256;   // permuted contribution pointers per launch (kMaxSegs*P <= this)

struct RuArgs {
    const float* x[kPtrSlots];      // x[s*P + q]: q-th term of segment s
    int64_t bound[kMaxSegs + 1];    // segment s covers flat elements [bound[s], bound[s+1])
    int32_t first_block[kMaxSegs + 1];
    int32_t n_segs;
    float* g;                       // may be null
    float* w;
    float* v;
    float lr, mu, wd;
};

template <bool NT>
__device__ __forceinline__ float4 load4(const float* p) {
    if (NT) {
        float4 r;
        r.x = __builtin_nontemporal_load(p + 0);
        r.y = __builtin_nontemporal_load(p + 1);
        r.z = __builtin_nontemporal_load(p + 2);
        r.w = __builtin_nontemporal_load(p + 3);
        return r;
    }
    return *reinterpret_cast<const float4*>(p);
}

template <bool NT>
__device__ __forceinline__ void store4(float* p, const float4& q) {
    if (NT) {
        __builtin_nontemporal_store(q.x, p + 0);
        __builtin_nontemporal_store(q.y, p + 1);
        __builtin_nontemporal_store(q.z, p + 2);
        __builtin_nontemporal_store(q.w, p + 3);
    } else {
        *reinterpret_cast<float4*>(p) = q;
    }
}

// The update of one element; returns nothing, rewrites w and v.  Each line is one rounding.
__device__ __forceinline__ void sgd(float g, float& w, float& v, float lr, float mu, float wd) {
    const float decay = wd * w;
    const float d = g + decay;
    const float mv = mu * v;
    const float vn = mv + d;
    const float step = lr * vn;
    w = w - step;
    v = vn;
}

// P > 0: compile-time number of terms; P == 0: run-time count in `Prt` (up to MC_MAX_P).
template <int P, int U, int THREADS, bool HAS_G, bool NT_IN, bool NT_G>
__global__ __launch_bounds__(THREADS) void reduce_update_kernel(RuArgs a, int Prt) {
    constexpr int64_t kTile = int64_t(THREADS) * 4 * U;
    const int np = P > 0 ? P : Prt;

    // blockIdx -> (segment, tile); a handful of scalar compares.
    int s = 0;
    while (s + 1 < a.n_segs && int(blockIdx.x) >= a.first_block[s + 1]) ++s;
    const int64_t lo = a.bound[s];
    const int64_t hi = a.bound[s + 1];
    const int64_t base = lo + int64_t(int(blockIdx.x) - a.first_block[s]) * kTile;
    const float* const* xs = a.x + s * np;

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
                for (int u = 0; u < U; ++u) t[q][u] = load4<NT_IN>(xs[q] + idx[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                wv[u] = *reinterpret_cast<const float4*>(a.w + idx[u]);
                vv[u] = *reinterpret_cast<const float4*>(a.v + idx[u]);
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
#pragma unroll
            for (int u = 0; u < U; ++u) {
                wv[u] = *reinterpret_cast<const float4*>(a.w + idx[u]);
                vv[u] = *reinterpret_cast<const float4*>(a.v + idx[u]);
                acc[u] = load4<NT_IN>(xs[0] + idx[u]);
            }
            for (int q = 1; q < np; ++q) {
                const float* xq = xs[q];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float4 t = load4<NT_IN>(xq + idx[u]);
                    acc[u].x = acc[u].x + t.x;
                    acc[u].y = acc[u].y + t.y;
                    acc[u].z = acc[u].z + t.z;
                    acc[u].w = acc[u].w + t.w;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (HAS_G) store4<NT_G>(a.g + idx[u], acc[u]);
            sgd(acc[u].x, wv[u].x, vv[u].x, a.lr, a.mu, a.wd);
            sgd(acc[u].y, wv[u].y, vv[u].y, a.lr, a.mu, a.wd);
            sgd(acc[u].z, wv[u].z, vv[u].z, a.lr, a.mu, a.wd);
            sgd(acc[u].w, wv[u].w, vv[u].w, a.lr, a.mu, a.wd);
            *reinterpret_cast<float4*>(a.w + idx[u]) = wv[u];
            *reinterpret_cast<float4*>(a.v + idx[u]) = vv[u];
        }
        return;
    }

    // Last, partial tile of the segment: whole vectors while they fit, then single elements.
    // (lo is a multiple of 256 elements, so base is 16-byte aligned; hi need not be.)
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + (int64_t(u) * THREADS + threadIdx.x) * 4;
        if (i >= hi) break;
        if (i + 4 <= hi) {
            float4 acc = load4<NT_IN>(xs[0] + i);
            for (int q = 1; q < np; ++q) {
                const float4 t = load4<NT_IN>(xs[q] + i);
                acc.x = acc.x + t.x;
                acc.y = acc.y + t.y;
                acc.z = acc.z + t.z;
                acc.w = acc.w + t.w;
            }
            float4 wq = *reinterpret_cast<const float4*>(a.w + i);
            float4 vq = *reinterpret_cast<const float4*>(a.v + i);
            if (HAS_G) *reinterpret_cast<float4*>(a.g + i) = acc;
            sgd(acc.x, wq.x, vq.x, a.lr, a.mu, a.wd);
            sgd(acc.y, wq.y, vq.y, a.lr, a.mu, a.wd);
            sgd(acc.z, wq.z, vq.z, a.lr, a.mu, a.wd);
            sgd(acc.w, wq.w, vq.w, a.lr, a.mu, a.wd);
            *reinterpret_cast<float4*>(a.w + i) = wq;
            *reinterpret_cast<float4*>(a.v + i) = vq;
        } else {
            for (int64_t e = i; e < hi; ++e) {
                float acc = xs[0][e];
                for (int q = 1; q < np; ++q) acc = acc + xs[q][e];
                float we = a.w[e], ve = a.v[e];
                if (HAS_G) a.g[e] = acc;
                sgd(acc, we, ve, a.lr, a.mu, a.wd);
                a.w[e] = we;
                a.v[e] = ve;
            }
        }
    }
}

template <int P, int U, bool HAS_G>
void launch_nt(int nt, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    constexpr int T = kThreads;
    switch (nt & 3) {
        case 0: hipLaunchKernelGGL((reduce_update_kernel<P, U, T, HAS_G, false, false>), dim3(blocks), dim3(T), 0, s, a, Prt); break;
        case 1: hipLaunchKernelGGL((reduce_update_kernel<P, U, T, HAS_G, true, false>), dim3(blocks), dim3(T), 0, s, a, Prt); break;
        case 2: hipLaunchKernelGGL((reduce_update_kernel<P, U, T, HAS_G, false, true>), dim3(blocks), dim3(T), 0, s, a, Prt); break;
        default: hipLaunchKernelGGL((reduce_update_kernel<P, U, T, HAS_G, true, true>), dim3(blocks), dim3(T), 0, s, a, Prt); break;
    }
}

template <int P>
void launch_unroll(int unroll, int nt, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    if (unroll == 1) {
        if (a.g) launch_nt<P, 1, true>(nt, blocks, s, a, Prt); else launch_nt<P, 1, false>(nt, blocks, s, a, Prt);
    } else {
        if (a.g) launch_nt<P, 2, true>(nt, blocks, s, a, Prt); else launch_nt<P, 2, false>(nt, blocks, s, a, Prt);
    }
}

void launch(int P, int unroll, int nt, unsigned blocks, hipStream_t s, const RuArgs& a) {
    switch (P) {
        case 1: launch_unroll<1>(unroll, nt, blocks, s, a, P); break;
        case 2: launch_unroll<2>(unroll, nt, blocks, s, a, P); break;
        case 3: launch_unroll<3>(unroll, nt, blocks, s, a, P); break;
        case 4: launch_unroll<4>(unroll, nt, blocks, s, a, P); break;
        case 5: launch_unroll<5>(unroll, nt, blocks, s, a, P); break;
        case 6: launch_unroll<6>(unroll, nt, blocks, s, a, P); break;
        case 7: launch_unroll<7>(unroll, nt, blocks, s, a, P); break;
        case 8: launch_unroll<8>(unroll, nt, blocks, s, a, P); break;
        default: launch_unroll<0>(unroll, nt, blocks, s, a, P); break;
    }
}

}  // namespace

extern "C" int mc_reduce_update(const mc_layout* L, const void* const* contrib, int32_t P,
                                const int32_t* order, void* grad_out, void* weights,
                                void* momentum, float lr, float mu, float wd, void* stream) {
    if (!L || !contrib || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
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
    if (L->N == 0) return MC_OK;
    if (!weights || !momentum) return MC_ERR_INVALID_ARG;
    for (int32_t p = 0; p < P; ++p)
        if (!contrib[p]) return MC_ERR_INVALID_ARG;

    // Alignment and overlap over the whole list {contrib[0..P), weights, momentum, grad_out}.
    const void* bufs[MC_MAX_P + 3];
    int nb = 0;
    for (int32_t p = 0; p < P; ++p) bufs[nb++] = contrib[p];
    bufs[nb++] = weights;
    bufs[nb++] = momentum;
    if (grad_out) bufs[nb++] = grad_out;
    for (int i = 0; i < nb; ++i)
        if (!mc::aligned(bufs[i], 16)) return MC_ERR_ALIGN;
    const uint64_t bytes = uint64_t(L->N) * 4;
    for (int i = 0; i < nb; ++i)
        for (int j = i + 1; j < nb; ++j)
            if (mc::overlaps(bufs[i], bytes, bufs[j], bytes)) return MC_ERR_OVERLAP;

    const int unroll = mc::option(MC_OPT_RU_UNROLL);
    const int threads = kThreads;
    const int nt = mc::option(MC_OPT_RU_NONTEMPORAL);
    const int64_t tile = int64_t(threads) * 4 * unroll;
    const int segs_per_launch = std::min(kMaxSegs, kPtrSlots / P);
    hipStream_t s = static_cast<hipStream_t>(stream);

    RuArgs a;
    a.g = static_cast<float*>(grad_out);
    a.w = static_cast<float*>(weights);
    a.v = static_cast<float*>(momentum);
    a.lr = lr;
    a.mu = mu;
    a.wd = wd;
    int32_t c = 0;
    while (c < L->k) {
        // Gather the next run of non-empty colours into one launch.
        int ns = 0;
        int64_t blocks = 0;
        a.first_block[0] = 0;
        while (c < L->k && ns < segs_per_launch) {
            const int64_t lo = L->bounds[c], hi = L->bounds[c + 1];
            if (hi > lo) {
                if (ns > 0 && a.bound[ns] != lo) break;  // (cannot happen: colours are contiguous)
                const int64_t nblk = (hi - lo + tile - 1) / tile;
                if (blocks + nblk > 0x7fffffff) {
                    if (ns == 0) return MC_ERR_INVALID_ARG;
                    break;
                }
                a.bound[ns] = lo;
                a.bound[ns + 1] = hi;
                for (int32_t q = 0; q < P; ++q) {
                    const int32_t src = order ? order[size_t(c) * P + q] : q;
                    a.x[ns * P + q] = static_cast<const float*>(contrib[src]);
                }
                blocks += nblk;
                a.first_block[ns + 1] = int32_t(blocks);
                ++ns;
            }
            ++c;
        }
        if (ns == 0) continue;
        for (int i = ns * P; i < kPtrSlots; ++i) a.x[i] = nullptr;
        for (int i = ns + 1; i <= kMaxSegs; ++i) {
            a.bound[i] = a.bound[ns];
            a.first_block[i] = a.first_block[ns];
        }
        a.n_segs = ns;
        launch(P, unroll, nt, unsigned(blocks), s, a);
        MC_HIP_TRY(hipGetLastError());
    }
    return MC_OK;
}
