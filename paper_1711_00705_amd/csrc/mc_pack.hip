// a2 / a5: gather per-layer tensors into the flat payload (pack) and scatter it back (unpack).
//
// The flat side is always walked in 16-byte vectors aligned to the payload, so flat traffic is
// fully coalesced 128-bit accesses.  The tensor side is a 128-bit access when the four
// elements lie in one tensor and its address happens to be 16-byte aligned too (always the
// case for layouts whose tensor sizes are multiples of four elements and whose tensors are
// 16-byte aligned, like the CNN payloads), and four 32-bit accesses otherwise.
//
// Device pointers of the tensors travel in the kernel-argument block (no staging copy, no
// synchronisation); a layout with more tensors than fit is processed in several launches.  The
// `_set` forms read the pointers from a tensor set's device table instead: one launch whatever
// the number of tensors.  One wavefront per workgroup and one vector per thread: a tile is 256
// flat elements, the granularity of the layout's lookup table.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <utility>
#include <vector>

#include "mc_internal.h"
#include "mc_mem.h"
#include "mc_tiles.h"

namespace {

constexpr int kThreads = 64;
constexpr int kVecPerThread = int(mc::kPackTileElems / 4 / kThreads);  // 16-byte vectors per thread
static_assert(mc::kPackTileElems == int64_t(kThreads) * 4 * kVecPerThread, "tile shape");
static_assert(kVecPerThread == 1, "the launch code below instantiates V = 1");

struct PtrBatch {
    void* p[mc::kPackMaxPtrs];
};

typedef uint32_t native_u4 __attribute__((ext_vector_type(4)));
// Every buffer is device global memory.  Tensor pointers arrive through memory (the pointer batch
// or a tensor set's table) as generic pointers; dereferencing through global-address-space types
// lets the compiler emit global_ instead of flat_ instructions.
typedef __attribute__((address_space(1))) native_u4 global_u4;
typedef __attribute__((address_space(1))) uint32_t global_u1;

template <bool NT>
__device__ __forceinline__ uint4 ld4(const uint32_t* p) {
    const global_u4* gp = (const global_u4*)p;
    const native_u4 r = NT ? __builtin_nontemporal_load(gp) : *gp;
    return make_uint4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ uint32_t ld1(const uint32_t* p) { return *(const global_u1*)p; }
__device__ __forceinline__ void st1(uint32_t* p, uint32_t x) { *(global_u1*)p = x; }

// Streaming store: the agent-scope (write-through) bit measured faster than the non-temporal
// hint for copy-shaped kernels on this part.
template <bool STREAM>
__device__ __forceinline__ void st4(uint32_t* p, const uint4& q) {
    const native_u4 val = {q.x, q.y, q.z, q.w};
    if (STREAM)
        mc::store128_sc1(p, val);
    else
        *(global_u4*)p = val;
}

// One launch covers tensors [t0, t1), i.e. flat elements [off[t0], off[t1]), tile by tile.
// UNPACK = false: tensors -> flat.  UNPACK = true: flat -> tensors.
// NT_T / NT_F: streaming policy for the tensor side / the flat side (non-temporal loads,
// write-through stores).
// V: 16-byte vectors per thread; a workgroup covers a tile of kThreads * 4 * V flat elements.
// TABLE: tensor addresses come from a tensor set's device table instead of the argument block (a
// compile-time choice: a run-time one makes the compiler fetch the address with a per-lane load
// through a selected pointer).
template <bool UNPACK, bool NT_T, bool NT_F, int V, bool TABLE>
__global__ __launch_bounds__(kThreads) void gather_scatter_kernel(
    void* const* __restrict__ table, const int64_t* __restrict__ off, const int32_t* __restrict__ tile_first,
    uint32_t* flat, int64_t tile0, int64_t hi, int32_t t0, int32_t xcd_run, int64_t lo, PtrBatch ptrs) {
    // lo, hi: the launch's flat range [off[t0], off[t1]).  The scalars in front of lo are what a
    // tile needs before its first lookup; as leading arguments they arrive in registers when the
    // wavefront starts (kernel-argument preload).
    constexpr int64_t kTileElems = int64_t(kThreads) * 4 * V;
    static_assert(kTileElems % mc::kLookupElems == 0, "tiles start on lookup entries");
    const int64_t tile = tile0 + mc::xcd_tile(int(blockIdx.x), int(gridDim.x), xcd_run);
    const int64_t tile_base = tile * kTileElems;
    const int32_t t_tile = max(tile_first[tile_base / mc::kLookupElems], t0);
    __builtin_amdgcn_sched_barrier(0);

    // Whole tile inside one tensor (and inside this launch's range) with a 16-byte aligned
    // tensor side: nearly all bytes of a CNN payload.  Everything deciding it is uniform over
    // the workgroup, so the lookups are scalar loads; the tensor's bounds and its address are
    // fetched together and the decision is one expression over them (no fetch waits behind a
    // branch), and all V loads precede the first store.
    typedef long long ll2 __attribute__((ext_vector_type(2)));
    ll2 bounds;
    __builtin_memcpy(&bounds, off + t_tile, sizeof(bounds));
    uint32_t* const t_base = static_cast<uint32_t*>(TABLE ? table[t_tile] : ptrs.p[t_tile - t0]);
    __builtin_amdgcn_sched_barrier(0);
    uint32_t* const tens = t_base + (tile_base - bounds.x);
    const bool whole = (tile_base >= lo) & (tile_base + kTileElems <= hi) & (bounds.x <= tile_base) &
                       (tile_base + kTileElems <= bounds.y) & ((reinterpret_cast<uintptr_t>(tens) & 15) == 0);
    if (whole) {
        uint32_t* fl = flat + tile_base;
        uint4 q[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int e = (j * kThreads + int(threadIdx.x)) * 4;
            q[j] = UNPACK ? ld4<NT_F>(fl + e) : ld4<NT_T>(tens + e);
        }
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int e = (j * kThreads + int(threadIdx.x)) * 4;
            if (UNPACK)
                st4<NT_T>(tens + e, q[j]);
            else
                st4<NT_F>(fl + e, q[j]);
        }
        return;
    }

#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int64_t i = tile_base + (int64_t(j) * kThreads + threadIdx.x) * 4;
        if (i >= hi || i + 4 <= lo) continue;
        const int64_t first = i > lo ? i : lo;
        int32_t t = t_tile;
        while (off[t + 1] <= first) ++t;  // ends: first < hi == off[t1]

        const bool one_tensor = i >= lo && i + 4 <= off[t + 1];
        if (one_tensor) {
            uint32_t* src = static_cast<uint32_t*>(TABLE ? table[t] : ptrs.p[t - t0]) + (i - off[t]);
            if ((reinterpret_cast<uintptr_t>(src) & 15) == 0) {
                if (UNPACK)
                    st4<NT_T>(src, ld4<NT_F>(flat + i));
                else
                    st4<NT_F>(flat + i, ld4<NT_T>(src));
            } else if (UNPACK) {
                const uint4 q = ld4<NT_F>(flat + i);
                st1(src + 0, q.x);
                st1(src + 1, q.y);
                st1(src + 2, q.z);
                st1(src + 3, q.w);
            } else {
                uint4 q;
                q.x = ld1(src + 0);
                q.y = ld1(src + 1);
                q.z = ld1(src + 2);
                q.w = ld1(src + 3);
                st4<NT_F>(flat + i, q);
            }
            continue;
        }
        // The vector straddles a tensor boundary, the launch's range or the payload's end.
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t idx = i + e;
            if (idx < lo || idx >= hi) continue;
            while (off[t + 1] <= idx) ++t;
            uint32_t* elem = static_cast<uint32_t*>(TABLE ? table[t] : ptrs.p[t - t0]) + (idx - off[t]);
            if (UNPACK)
                st1(elem, ld1(flat + idx));
            else
                st1(flat + idx, ld1(elem));
        }
    }
}

// One launch over tensors [t0, t1): pointers from `batch` (kernel arguments) or, if given, from
// the device table of a tensor set.
template <bool UNPACK>
int launch_range(const mc_layout* L, const mc::DeviceTables* dt, const PtrBatch& batch, void* const* table,
                 void* flat, int32_t t0, int32_t t1, hipStream_t s) {
    const int64_t lo = L->off[t0], hi = L->off[t1];
    if (lo == hi) return MC_OK;
    const int nt = mc::option(MC_OPT_PACK_NONTEMPORAL);
    const int64_t tile_elems = mc::kPackTileElems;
    const bool small = L->N < (int64_t(1) << 24);
    const int64_t tile0 = lo / tile_elems;
    const int64_t tile_end = (hi + tile_elems - 1) / tile_elems;
    if (tile_end - tile0 > 0x7fffffff) return MC_ERR_INVALID_ARG;
    const dim3 grid(unsigned(tile_end - tile0)), block(kThreads);
    uint32_t* f = static_cast<uint32_t*>(flat);
    // Consecutive tiles per die.  Automatic: small payloads pack faster when neighbouring tiles share
    // an L2 (GoogLeNet-sized pack +14 %, extra fetches +4.6 % -> +1.1 %: its many small tensors leave
    // most tiles cutting through a cache line at a tensor boundary); large ones are indifferent,
    // and unpack, which often re-reads what an update has just written, loses with it.
    int xcd_run = mc::option(UNPACK ? MC_OPT_XCD_RUN_UNPACK : MC_OPT_XCD_RUN_PACK);
    if (xcd_run < 0) xcd_run = (!UNPACK && small) ? 16 : 0;
    const unsigned lds = mc::lds_reservation(MC_OPT_LDS_CAP_PACK, kThreads);
#define MC_GS_LAUNCH_V(NT_T, NT_F, V, TABLE)                                                                  \
    hipLaunchKernelGGL((gather_scatter_kernel<UNPACK, NT_T, NT_F, V, TABLE>), grid, block, lds, s, table, dt->off, \
                       dt->tile_first, f, tile0, hi, t0, xcd_run, lo, batch)
#define MC_GS_LAUNCH(NT_T, NT_F)                               \
    do {                                                       \
        if (table)                                             \
            MC_GS_LAUNCH_V(NT_T, NT_F, kVecPerThread, true);   \
        else                                                   \
            MC_GS_LAUNCH_V(NT_T, NT_F, kVecPerThread, false);  \
    } while (0)
    switch (nt & 3) {
        case 0: MC_GS_LAUNCH(false, false); break;
        case 1: MC_GS_LAUNCH(true, false); break;
        case 2: MC_GS_LAUNCH(false, true); break;
        default: MC_GS_LAUNCH(true, true); break;
    }
#undef MC_GS_LAUNCH_V
#undef MC_GS_LAUNCH
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

template <bool UNPACK>
int run(mc_layout* L, void* const* tensors, void* flat, void* stream) {
    if (!L || !tensors) return MC_ERR_INVALID_ARG;
    if (L->N == 0) return MC_OK;
    if (!flat) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(flat, 16)) return MC_ERR_ALIGN;
    const uint64_t flat_bytes = uint64_t(L->N) * 4;
    for (int32_t t = 0; t < L->n; ++t) {
        const int64_t cnt = L->off[t + 1] - L->off[t];
        if (cnt == 0) continue;
        if (!tensors[t]) return MC_ERR_INVALID_ARG;
        if (!mc::aligned(tensors[t], 4)) return MC_ERR_ALIGN;
        if (mc::overlaps(tensors[t], uint64_t(cnt) * 4, flat, flat_bytes)) return MC_ERR_OVERLAP;
    }
    if (UNPACK) {
        // destination tensors that overlap each other would be written by two workgroups at once
        std::vector<std::pair<uintptr_t, uintptr_t>> spans;
        for (int32_t t = 0; t < L->n; ++t) {
            const int64_t cnt = L->off[t + 1] - L->off[t];
            const uintptr_t b = reinterpret_cast<uintptr_t>(tensors[t]);
            if (cnt > 0) spans.emplace_back(b, b + uintptr_t(cnt) * 4);
        }
        std::sort(spans.begin(), spans.end());
        for (size_t i = 1; i < spans.size(); ++i)
            if (spans[i].first < spans[i - 1].second) return MC_ERR_OVERLAP;
    }
    const mc::DeviceTables* dt = nullptr;
    const int rc = mc::device_tables(L, &dt);
    if (rc != MC_OK) return rc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int32_t t0 = 0; t0 < L->n; t0 += mc::kPackMaxPtrs) {
        const int32_t t1 = std::min<int32_t>(L->n, t0 + mc::kPackMaxPtrs);
        PtrBatch batch;
        for (int32_t t = t0; t < t1; ++t) batch.p[t - t0] = tensors[t];
        for (int32_t t = t1 - t0; t < mc::kPackMaxPtrs; ++t) batch.p[t] = nullptr;
        const int lrc = launch_range<UNPACK>(L, dt, batch, nullptr, flat, t0, t1, s);
        if (lrc != MC_OK) return lrc;
    }
    return MC_OK;
}

template <bool UNPACK>
int run_set(mc_layout* L, const mc_tensor_set* S, void* flat, void* stream) {
    if (!L || !S || S->layout != L) return MC_ERR_INVALID_ARG;
    if (L->N == 0) return MC_OK;
    if (!flat) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(flat, 16)) return MC_ERR_ALIGN;
    const uintptr_t fb = reinterpret_cast<uintptr_t>(flat), fe = fb + uintptr_t(L->N) * 4;
    for (const auto& span : S->spans)
        if (span.first < fe && fb < span.second) return MC_ERR_OVERLAP;
    const mc::DeviceTables* dt = nullptr;
    const int rc = mc::device_tables(L, &dt);
    if (rc != MC_OK) return rc;
    int dev = -1;
    MC_HIP_TRY(hipGetDevice(&dev));
    if (S->device != dev) return MC_ERR_INVALID_ARG;
    PtrBatch none;
    for (int i = 0; i < mc::kPackMaxPtrs; ++i) none.p[i] = nullptr;
    return launch_range<UNPACK>(L, dt, none, S->d_ptrs, flat, 0, L->n, static_cast<hipStream_t>(stream));
}


// ---- mc_pack for callers that may not allocate ------------------------------------------------
// The gather kernel reads two tables (flat offsets, first tensor per 256 flat elements) that the
// other entry points keep in device memory allocated by mc_layout_prepare.  Here they live in a
// fixed array in the library's own device image and are rebuilt on the stream before every call.
constexpr int64_t kNoAllocMaxElems = int64_t(MC_NOALLOC_MAX_ELEMS);
constexpr size_t kScratchOffBytes = 4096;  // off[kPackMaxPtrs + 1] as int64, padded
constexpr size_t kScratchFirstEntries = size_t(kNoAllocMaxElems / mc::kLookupElems) + 1;
constexpr size_t kScratchBytes = (kScratchOffBytes + kScratchFirstEntries * sizeof(int32_t) + 255) / 256 * 256;
static_assert((mc::kPackMaxPtrs + 1) * sizeof(int64_t) <= kScratchOffBytes, "offsets fit their slot");

// Each GPU the library runs on holds its own copy of this array (about 4 MiB) until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress: the address that kernels
// and copies may use is the one that call returns, per device.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mu;
void* g_scratch_ptr[mc::kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int scratch_address(unsigned char** out) {
    int dev = -1;
    MC_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= mc::kMaxDevices) return MC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        MC_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return MC_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
    return MC_OK;
}

struct OffBatch {
    int64_t off[mc::kPackMaxPtrs + 1];
};

// Writes the n + 1 flat offsets and, for each of n_entries runs of kLookupElems flat elements, the
// first tensor whose range ends after the run's first element (n when there is none).
__global__ __launch_bounds__(kThreads) void noalloc_tables_kernel(OffBatch ob, int32_t n, int64_t* off_out,
                                                                  int32_t* first_out, int64_t n_entries) {
    __shared__ int64_t off[mc::kPackMaxPtrs + 1];
    for (int t = int(threadIdx.x); t <= n; t += kThreads) off[t] = ob.off[t];
    __syncthreads();
    if (blockIdx.x == 0)
        for (int t = int(threadIdx.x); t <= n; t += kThreads) off_out[t] = off[t];
    const int64_t j = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (j >= n_entries) return;
    const int64_t first = j * mc::kLookupElems;
    // smallest t in [0, n] with t == n or off[t + 1] > first (off is non-decreasing)
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (off[mid + 1] > first) hi = mid; else lo = mid + 1;
    }
    first_out[j] = lo;
}

int run_noalloc(const mc_layout* L, void* const* tensors, void* flat, void* stream) {
    if (!L || !tensors) return MC_ERR_INVALID_ARG;
    // the limits come first: nothing of the GPU is touched for a layout that cannot be served
    if (L->n > mc::kPackMaxPtrs || L->N > kNoAllocMaxElems) return MC_ERR_LIMIT;
    if (L->N == 0) return MC_OK;
    if (!flat) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(flat, 16)) return MC_ERR_ALIGN;
    const uint64_t flat_bytes = uint64_t(L->N) * 4;
    for (int32_t t = 0; t < L->n; ++t) {
        const int64_t cnt = L->off[t + 1] - L->off[t];
        if (cnt == 0) continue;
        if (!tensors[t]) return MC_ERR_INVALID_ARG;
        if (!mc::aligned(tensors[t], 4)) return MC_ERR_ALIGN;
        if (mc::overlaps(tensors[t], uint64_t(cnt) * 4, flat, flat_bytes)) return MC_ERR_OVERLAP;
    }
    unsigned char* base = nullptr;
    const int rc = scratch_address(&base);
    if (rc != MC_OK) return rc;

    mc::DeviceTables dt;
    dt.off = reinterpret_cast<int64_t*>(base);
    dt.tile_first = reinterpret_cast<int32_t*>(base + kScratchOffBytes);
    dt.ready = true;
    const int64_t n_entries = int64_t(L->tile_first.size());   // ceil(N / kLookupElems) + 1
    if (size_t(n_entries) > kScratchFirstEntries) return MC_ERR_LIMIT;

    hipStream_t s = static_cast<hipStream_t>(stream);
    OffBatch ob;
    for (int32_t t = 0; t <= L->n; ++t) ob.off[t] = L->off[t];
    for (int32_t t = L->n + 1; t <= mc::kPackMaxPtrs; ++t) ob.off[t] = L->N;
    const unsigned blocks = unsigned((n_entries + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(noalloc_tables_kernel, dim3(blocks), dim3(kThreads), 0, s, ob, L->n, dt.off, dt.tile_first,
                       n_entries);
    MC_HIP_TRY(hipGetLastError());

    PtrBatch batch;
    for (int32_t t = 0; t < L->n; ++t) batch.p[t] = tensors[t];
    for (int32_t t = L->n; t < mc::kPackMaxPtrs; ++t) batch.p[t] = nullptr;
    return launch_range<false>(L, &dt, batch, nullptr, flat, 0, L->n, s);
}

}  // namespace

namespace mc {

int device_tables(mc_layout* L, const DeviceTables** out) {
    int dev = 0;
    MC_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(L->mu);
    DeviceTables& d = L->dev[dev];
    if (!d.ready) {
        int64_t* off = nullptr;
        int32_t* tf = nullptr;
        const size_t off_bytes = L->off.size() * sizeof(int64_t);
        const size_t tf_bytes = L->tile_first.size() * sizeof(int32_t);
        MC_HIP_TRY(hipMalloc(reinterpret_cast<void**>(&off), off_bytes));
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&tf), tf_bytes);
        if (e == hipSuccess) e = hipMemcpy(off, L->off.data(), off_bytes, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(tf, L->tile_first.data(), tf_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(off);
            (void)hipFree(tf);
            return hip_fail(e);
        }
        int32_t *ut = nullptr, *uf = nullptr;
        if (!L->unit_tensor.empty()) {
            const size_t ut_bytes = L->unit_tensor.size() * sizeof(int32_t);
            const size_t uf_bytes = std::max<size_t>(L->unit_first.size(), 1) * sizeof(int32_t);
            e = hipMalloc(reinterpret_cast<void**>(&ut), ut_bytes);
            if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&uf), uf_bytes);
            if (e == hipSuccess) e = hipMemcpy(ut, L->unit_tensor.data(), ut_bytes, hipMemcpyHostToDevice);
            if (e == hipSuccess && !L->unit_first.empty())
                e = hipMemcpy(uf, L->unit_first.data(), L->unit_first.size() * sizeof(int32_t), hipMemcpyHostToDevice);
            if (e != hipSuccess) {
                (void)hipFree(off);
                (void)hipFree(tf);
                (void)hipFree(ut);
                (void)hipFree(uf);
                return hip_fail(e);
            }
        }
        d.off = off;
        d.tile_first = tf;
        d.unit_tensor = ut;
        d.unit_first = uf;
        d.ready = true;
    }
    *out = &d;
    return MC_OK;
}

}  // namespace mc

extern "C" {

int mc_layout_prepare(mc_layout* L) {
    if (!L) return MC_ERR_INVALID_ARG;
    const mc::DeviceTables* dt = nullptr;
    return mc::device_tables(L, &dt);
}

int mc_layout_destroy(mc_layout* L) {
    if (!L) return MC_OK;
    int rc = MC_OK;
    {
        std::lock_guard<std::mutex> lock(L->mu);
        int cur = -1;
        bool any = false;
        for (int d = 0; d < mc::kMaxDevices; ++d) any = any || L->dev[d].ready;
        if (any && hipGetDevice(&cur) != hipSuccess) cur = -1;
        for (int d = 0; d < mc::kMaxDevices; ++d) {
            mc::DeviceTables& t = L->dev[d];
            if (!t.ready) continue;
            hipError_t e = hipSetDevice(d);
            if (e == hipSuccess) e = hipFree(t.off);
            if (e == hipSuccess) e = hipFree(t.tile_first);
            if (e == hipSuccess && t.unit_tensor) e = hipFree(t.unit_tensor);
            if (e == hipSuccess && t.unit_first) e = hipFree(t.unit_first);
            if (e != hipSuccess) rc = mc::hip_fail(e);
            t.ready = false;
        }
        if (any && cur >= 0) (void)hipSetDevice(cur);
    }
    delete L;
    return rc;
}

int mc_pack(mc_layout* L, const void* const* tensors, void* flat, void* stream) {
    return run<false>(L, const_cast<void* const*>(tensors), flat, stream);
}

int mc_unpack(mc_layout* L, const void* flat, void* const* tensors, void* stream) {
    try {
        return run<true>(L, tensors, const_cast<void*>(flat), stream);
    } catch (const std::bad_alloc&) {   // the span list of the overlap check
        return MC_ERR_ALLOC;
    }
}

int mc_pack_noalloc(const mc_layout* L, const void* const* tensors, void* flat, void* stream) {
    return run_noalloc(L, const_cast<void* const*>(tensors), flat, stream);
}

int mc_pack_set(mc_layout* L, const mc_tensor_set* tensors, void* flat, void* stream) {
    return run_set<false>(L, tensors, flat, stream);
}

int mc_unpack_set(mc_layout* L, const void* flat, const mc_tensor_set* tensors, void* stream) {
    return run_set<true>(L, tensors, const_cast<void*>(flat), stream);
}

}  // extern "C"
