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
#include <new>
#include <vector>

#include "mc_internal.h"
#include "mc_tiles.h"
#include "mc_update.h"

#pragma clang fp contract(off)

namespace {

constexpr int kThreads = 256;  // workgroup size
constexpr int kMaxSegs = 32;     // colours per launch
constexpr int kPtrSlots = 256;   // permuted contribution pointers per launch (kMaxSegs*P <= this)

struct RuArgs {
    const float* x[kPtrSlots];      // x[s*np + q]: q-th term of segment s (np terms per segment)
    int64_t lo[kMaxSegs];           // segment s covers flat elements [lo[s], hi[s])
    int64_t hi[kMaxSegs];
    int32_t first_block[kMaxSegs + 1];
    int32_t n_segs;
    int32_t reverse;                // walk the launch's tiles from the last to the first
    int32_t xcd_run;                // consecutive tiles per die (see mc_tiles.h); <= 1: plain
    float* g;                       // may be null when UPDATE
    float* w;                       // unused when !UPDATE
    float* v;
    mc::UpdateParams up;
};

typedef float native_f4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ float4 load4(const float* p) {
    if (NT) {
        const native_f4 r = __builtin_nontemporal_load(reinterpret_cast<const native_f4*>(p));
        return make_float4(r.x, r.y, r.z, r.w);
    }
    return *reinterpret_cast<const float4*>(p);
}

template <bool NT>
__device__ __forceinline__ void store4(float* p, const float4& q) {
    if (NT) {
        const native_f4 val = {q.x, q.y, q.z, q.w};
        __builtin_nontemporal_store(val, reinterpret_cast<native_f4*>(p));
    } else {
        *reinterpret_cast<float4*>(p) = q;
    }
}

// P > 0: compile-time number of terms; P == 0: run-time count in `Prt` (up to MC_MAX_P).
// UPDATE: the SGD step follows the sum (the rank holds the complete sum of these colours);
// otherwise only the sum is written to g and w, v are never touched.
// NT: streaming (non-temporal) loads of the contributions and store of g.
template <int P, int U, int THREADS, bool HAS_G, bool UPDATE, bool NT>
__global__ __launch_bounds__(THREADS) void reduce_update_kernel(RuArgs a, int Prt) {
    static_assert(HAS_G || UPDATE, "a launch must produce something");
    constexpr bool NT_IN = NT, NT_G = NT;
    constexpr int64_t kTile = int64_t(THREADS) * 4 * U;
    const int np = P > 0 ? P : Prt;
    const mc::Hyper hp = mc::resolve(a.up);

    // blockIdx -> (segment, tile); a handful of scalar compares.
    const int tile = mc::xcd_tile(int(blockIdx.x), int(gridDim.x), a.xcd_run);
    const int blk = a.reverse ? int(gridDim.x) - 1 - tile : tile;
    int s = 0;
    while (s + 1 < a.n_segs && blk >= a.first_block[s + 1]) ++s;
    const int64_t lo = a.lo[s];
    const int64_t hi = a.hi[s];
    const int64_t base = lo + int64_t(blk - a.first_block[s]) * kTile;
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
            if (UPDATE) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    wv[u] = *reinterpret_cast<const float4*>(a.w + idx[u]);
                    vv[u] = *reinterpret_cast<const float4*>(a.v + idx[u]);
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
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (UPDATE) {
                    wv[u] = *reinterpret_cast<const float4*>(a.w + idx[u]);
                    vv[u] = *reinterpret_cast<const float4*>(a.v + idx[u]);
                }
                acc[u] = load4<NT_IN>(xs[0] + idx[u]);
            }
            // Four terms' loads are issued before their adds (more bytes in flight); the adds
            // still run strictly left to right.
            int q = 1;
            for (; q + 4 <= np; q += 4) {
                float4 t[4][U];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int u = 0; u < U; ++u) t[r][u] = load4<NT_IN>(xs[q + r] + idx[u]);
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
            if (UPDATE) {
                mc::sgd(acc[u].x, wv[u].x, vv[u].x, hp);
                mc::sgd(acc[u].y, wv[u].y, vv[u].y, hp);
                mc::sgd(acc[u].z, wv[u].z, vv[u].z, hp);
                mc::sgd(acc[u].w, wv[u].w, vv[u].w, hp);
                mc::store_state(a.w + idx[u], wv[u], hp.state_store_sc1);
                mc::store_state(a.v + idx[u], vv[u], hp.state_store_sc1);
            }
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
            if (HAS_G) *reinterpret_cast<float4*>(a.g + i) = acc;
            if (UPDATE) {
                float4 wq = *reinterpret_cast<const float4*>(a.w + i);
                float4 vq = *reinterpret_cast<const float4*>(a.v + i);
                mc::sgd(acc.x, wq.x, vq.x, hp);
                mc::sgd(acc.y, wq.y, vq.y, hp);
                mc::sgd(acc.z, wq.z, vq.z, hp);
                mc::sgd(acc.w, wq.w, vq.w, hp);
                *reinterpret_cast<float4*>(a.w + i) = wq;
                *reinterpret_cast<float4*>(a.v + i) = vq;
            }
        } else {
            for (int64_t e = i; e < hi; ++e) {
                float acc = xs[0][e];
                for (int q = 1; q < np; ++q) acc = acc + xs[q][e];
                if (HAS_G) a.g[e] = acc;
                if (UPDATE) {
                    float we = a.w[e], ve = a.v[e];
                    mc::sgd(acc, we, ve, hp);
                    a.w[e] = we;
                    a.v[e] = ve;
                }
            }
        }
    }
}

template <int P, int U>
void launch_variant(bool update, bool nt, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    constexpr int T = kThreads;
    const dim3 grid(blocks), block(T);
#define MC_RU_LAUNCH(G, UPD, NT) \
    hipLaunchKernelGGL((reduce_update_kernel<P, U, T, G, UPD, NT>), grid, block, 0, s, a, Prt)
    if (!update) {
        if (nt) MC_RU_LAUNCH(true, false, true); else MC_RU_LAUNCH(true, false, false);
    } else if (a.g) {
        if (nt) MC_RU_LAUNCH(true, true, true); else MC_RU_LAUNCH(true, true, false);
    } else {
        if (nt) MC_RU_LAUNCH(false, true, true); else MC_RU_LAUNCH(false, true, false);
    }
#undef MC_RU_LAUNCH
}

template <int P>
void launch_unroll(int unroll, bool update, bool nt, unsigned blocks, hipStream_t s, const RuArgs& a, int Prt) {
    if (unroll == 1)
        launch_variant<P, 1>(update, nt, blocks, s, a, Prt);
    else
        launch_variant<P, 2>(update, nt, blocks, s, a, Prt);
}

void launch(int P, int unroll, bool update, bool nt, unsigned blocks, hipStream_t s, const RuArgs& a) {
    switch (P) {
        case 1: launch_unroll<1>(unroll, update, nt, blocks, s, a, P); break;
        case 2: launch_unroll<2>(unroll, update, nt, blocks, s, a, P); break;
        case 3: launch_unroll<3>(unroll, update, nt, blocks, s, a, P); break;
        case 4: launch_unroll<4>(unroll, update, nt, blocks, s, a, P); break;
        case 5: launch_unroll<5>(unroll, update, nt, blocks, s, a, P); break;
        case 6: launch_unroll<6>(unroll, update, nt, blocks, s, a, P); break;
        case 7: launch_unroll<7>(unroll, update, nt, blocks, s, a, P); break;
        case 8: launch_unroll<8>(unroll, update, nt, blocks, s, a, P); break;
        default: launch_unroll<0>(unroll, update, nt, blocks, s, a, P); break;
    }
}

// Shared by both entry points.  n_terms / do_update are null for the uniform call (every
// colour adds all P terms and updates).
//
// [r_lo, r_hi) restricts the call to a sub-range of the payload (a packet): every colour is
// intersected with it.  r_lo and r_hi are multiples of the colour alignment (r_hi may also be
// N), so every segment still starts on a 16-byte boundary.
int run_impl(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
             const int32_t* n_terms, const uint8_t* do_update, void* grad_out, void* weights,
             void* momentum, const mc::UpdateParams& up, int64_t r_lo, int64_t r_hi, void* stream) {
    if (!L || !contrib || P < 1 || P > MC_MAX_P) return MC_ERR_INVALID_ARG;
    if (up.hyper && !mc::aligned(up.hyper, 4)) return MC_ERR_ALIGN;
    if (r_lo < 0 || r_hi < r_lo || r_hi > L->N) return MC_ERR_INVALID_ARG;
    if (r_lo % MC_COLOUR_ALIGN_ELEMS != 0) return MC_ERR_INVALID_ARG;
    if (r_hi % MC_COLOUR_ALIGN_ELEMS != 0 && r_hi != L->N) return MC_ERR_INVALID_ARG;
    if ((n_terms == nullptr) != (do_update == nullptr)) return MC_ERR_INVALID_ARG;
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
    // What colour c contributes to this call: its range cut to [r_lo, r_hi).
    auto seg_lo = [&](int32_t c) { return std::max(L->bounds[c], r_lo); };
    auto seg_hi = [&](int32_t c) { return std::max(seg_lo(c), std::min(L->bounds[c + 1], r_hi)); };
    bool any_update = false, any_sum_only = false;
    for (int32_t c = 0; c < L->k; ++c) {
        if (n_terms && (n_terms[c] < 0 || n_terms[c] > P)) return MC_ERR_INVALID_ARG;
        if ((n_terms && n_terms[c] == 0) || seg_hi(c) == seg_lo(c)) continue;
        if (!do_update || do_update[c]) any_update = true; else any_sum_only = true;
    }
    if (!any_update && !any_sum_only) return MC_OK;  // nothing in range
    if (any_update && (!weights || !momentum)) return MC_ERR_INVALID_ARG;
    if (any_sum_only && !grad_out) return MC_ERR_INVALID_ARG;
    for (int32_t p = 0; p < P; ++p)
        if (!contrib[p]) return MC_ERR_INVALID_ARG;

    // Alignment and overlap over the whole list {contrib[0..P), weights, momentum, grad_out}.
    const void* bufs[MC_MAX_P + 3];
    int nb = 0;
    for (int32_t p = 0; p < P; ++p) bufs[nb++] = contrib[p];
    if (weights) bufs[nb++] = weights;
    if (momentum) bufs[nb++] = momentum;
    if (grad_out) bufs[nb++] = grad_out;
    for (int i = 0; i < nb; ++i)
        if (!mc::aligned(bufs[i], 16)) return MC_ERR_ALIGN;
    const uint64_t bytes = uint64_t(L->N) * 4;
    for (int i = 0; i < nb; ++i)
        for (int j = i + 1; j < nb; ++j)
            if (mc::overlaps(bufs[i], bytes, bufs[j], bytes)) return MC_ERR_OVERLAP;

    const int unroll = mc::unroll_for(r_hi - r_lo);
    const bool nt = mc::option(MC_OPT_RU_NONTEMPORAL) != 0;
    const int64_t tile = int64_t(kThreads) * 4 * unroll;
    hipStream_t s = static_cast<hipStream_t>(stream);

    RuArgs a;
    // Only the plain whole-payload step alternates: packets and role calls come several to a step.
    a.reverse = (!n_terms && r_lo == 0 && r_hi == L->N && mc::sweep_reversed(L)) ? 1 : 0;
    a.xcd_run = mc::option(MC_OPT_XCD_RUN);
    a.g = static_cast<float*>(grad_out);
    a.w = static_cast<float*>(weights);
    a.v = static_cast<float*>(momentum);
    a.up = up;

    // Colours that add the same number of terms and agree on updating share launches (a rank is
    // inner node or root for at most one colour, so there are at most two such classes in
    // practice; the uniform call has one).  `done` marks colours already launched.
    std::vector<uint8_t> done(size_t(L->k), 0);
    for (int32_t c0 = 0; c0 < L->k; ++c0) {
        if (done[c0]) continue;
        const int32_t cnt = n_terms ? n_terms[c0] : P;
        const bool upd = do_update ? do_update[c0] != 0 : true;
        if (cnt == 0 || seg_hi(c0) == seg_lo(c0)) {
            done[c0] = 1;
            continue;
        }
        const int segs_per_launch = std::min(kMaxSegs, kPtrSlots / cnt);
        int32_t c = c0;
        while (c < L->k) {
            int ns = 0;
            int64_t blocks = 0;
            a.first_block[0] = 0;
            for (; c < L->k && ns < segs_per_launch; ++c) {
                if (done[c]) continue;
                const int64_t lo = seg_lo(c), hi = seg_hi(c);
                const int32_t cc = n_terms ? n_terms[c] : P;
                const bool cu = do_update ? do_update[c] != 0 : true;
                if (cc == 0 || hi == lo) {
                    done[c] = 1;
                    continue;
                }
                if (cc != cnt || cu != upd) continue;  // another class: a later pass takes it
                const int64_t nblk = (hi - lo + tile - 1) / tile;
                if (blocks + nblk > 0x7fffffff) {
                    if (ns == 0) return MC_ERR_INVALID_ARG;
                    break;
                }
                a.lo[ns] = lo;
                a.hi[ns] = hi;
                for (int32_t q = 0; q < cnt; ++q) {
                    const int32_t src = order ? order[size_t(c) * P + q] : q;
                    a.x[ns * cnt + q] = static_cast<const float*>(contrib[src]);
                }
                blocks += nblk;
                a.first_block[ns + 1] = int32_t(blocks);
                done[c] = 1;
                ++ns;
            }
            if (ns == 0) break;
            for (int i = ns * cnt; i < kPtrSlots; ++i) a.x[i] = nullptr;
            for (int i = ns; i < kMaxSegs; ++i) {
                a.lo[i] = a.hi[i] = 0;
                a.first_block[i + 1] = a.first_block[ns];
            }
            a.n_segs = ns;
            launch(cnt, unroll, upd, nt, unsigned(blocks), s, a);
            MC_HIP_TRY(hipGetLastError());
        }
    }
    return MC_OK;
}

// No C++ exception may cross the C boundary.
int run(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
        const int32_t* n_terms, const uint8_t* do_update, void* grad_out, void* weights,
        void* momentum, const mc::UpdateParams& up, int64_t r_lo, int64_t r_hi, void* stream) {
    try {
        return run_impl(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, up,
                        r_lo, r_hi, stream);
    } catch (const std::bad_alloc&) {
        return MC_ERR_ALLOC;
    }
}

mc::UpdateParams immediate(float lr, float mu, float wd) {
    mc::UpdateParams up;
    up.lr = lr;
    up.mu = mu;
    up.wd = wd;
    up.hyper = nullptr;
    up.nesterov = 0;
    up.state_store_sc1 = mc::option(MC_OPT_STATE_STORE_SC1);
    return up;
}

}  // namespace

namespace mc {

int update_params(const mc_update_spec* spec, UpdateParams* out) {
    if (!spec || (spec->nesterov != 0 && spec->nesterov != 1)) return MC_ERR_INVALID_ARG;
    out->lr = spec->lr;
    out->mu = spec->mu;
    out->wd = spec->wd;
    out->hyper = spec->hyper_dev;
    out->nesterov = spec->nesterov;
    out->state_store_sc1 = mc::option(MC_OPT_STATE_STORE_SC1);
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
    mc::UpdateParams up;
    const int rc = mc::update_params(spec, &up);
    if (rc != MC_OK) return rc;
    return run(L, contrib, P, order, n_terms, do_update, grad_out, weights, momentum, up,
               elem_begin, elem_end < 0 ? L->N : elem_end, stream);
}

}  // extern "C"
