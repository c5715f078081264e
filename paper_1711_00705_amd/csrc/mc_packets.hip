// Packet-driven reduction: one resident kernel that sums and updates packets of the payload in
// their order of arrival, each as soon as a device-memory flag says that it has landed.
//
// Section 4.2 pipelines the k reductions: packets of every colour are in flight at once and a
// summing rank adds a packet when it arrives instead of waiting for whole chunks.  On the GPU the
// per-packet dependency must not go through the host or through stream events (each costs tens of
// microseconds, more than summing a packet takes), so the reducer polls the flags itself.  Whatever
// delivers a packet -- here a copy kernel followed by a one-thread kernel that raises the flag, on
// another stream -- writes
// the data first and the flag afterwards with release semantics; the reducer reads the flag with
// acquire semantics before it touches the packet.
//
// Every wait is bounded.  A workgroup that has polled `spin_limit` times in total without seeing
// the flag it needs stops, and so does every other one at its own pace; nothing is ever left
// half-done, because each workgroup records how many packets it has completed (progress[b]) and a
// later launch -- after the producer has finished -- resumes every workgroup from its own count.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "mc_internal.h"
#include "mc_ru_tile.h"
#include "mc_update.h"

#pragma clang fp contract(off)

namespace {

constexpr int kThreads = 256;
constexpr int64_t kTile = int64_t(kThreads) * 4;     // one 16-byte vector per thread
constexpr int kMaxColours = MC_PACKETS_MAX_COLOURS;
constexpr int kPtrSlots = 256;

struct PkArgs {
    const float* x[kPtrSlots];            // x[c * np + q]: q-th term of colour c
    int64_t bounds[kMaxColours + 1];      // colour bounds
    int32_t n_colours;
    int32_t np;
    int32_t n_packets;
    uint32_t arrivals;
    uint32_t spin_limit;
    int64_t N;
    const int64_t* packets;               // device: begin, end of each packet, in arrival order
    const uint32_t* ready;                // device: one flag per packet
    uint32_t* progress;                   // device: per workgroup, packets completed; then 2 status words
    float* g;
    float* w;
    float* v;
    mc::UpdateParams up;
};

template <int P, bool HAS_G, bool SS>
__global__ __launch_bounds__(kThreads) void packet_reducer_kernel(PkArgs a) {
    __shared__ int go;
    const mc::Hyper hp = mc::resolve(a.up);
    const int np = P > 0 ? P : a.np;
    const uint32_t G = gridDim.x;
    uint32_t polls_left = a.spin_limit;
    uint32_t j = a.progress[blockIdx.x];          // where an earlier launch of this step stopped
    bool gave_up = false;
    for (; j < uint32_t(a.n_packets); ++j) {
        // Packet j has landed when its flag equals arrivals x its length in elements: every delivery
        // adds the number of elements it wrote (mc_packet_deliver), or the producer writes the final
        // value at once (mc_packet_signal).  A malformed descriptor is not waited for.
        const int64_t lo = a.packets[2 * int64_t(j)];
        const int64_t hi = a.packets[2 * int64_t(j) + 1];
        const bool well_formed = lo >= 0 && lo < hi && hi <= a.N && lo % MC_COLOUR_ALIGN_ELEMS == 0;
        if (threadIdx.x == 0) {
            int ok = 0;
            int nap = 0;
            const uint32_t want = a.arrivals * uint32_t(hi - lo);
            for (;;) {
                if (!well_formed) {
                    ok = 1;
                    break;
                }
                // relaxed on purpose: an acquire here would invalidate the caches on every poll of
                // every workgroup; the one acquire that matters follows once the flag has been seen
                const uint32_t f = __hip_atomic_load(a.ready + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (f == want) {
                    ok = 1;
                    break;
                }
                if (polls_left == 0) break;
                --polls_left;
                // back off: a packet that is about to land is seen within a microsecond, a long wait
                // costs the memory system one request per workgroup every four microseconds
                if (nap == 0) __builtin_amdgcn_s_sleep(16);
                else if (nap == 1) __builtin_amdgcn_s_sleep(32);
                else if (nap == 2) __builtin_amdgcn_s_sleep(64);
                else __builtin_amdgcn_s_sleep(127);
                if (nap < 3) ++nap;
            }
            go = ok;
        }
        __syncthreads();
        const int ok = go;
        __syncthreads();                          // `go` is rewritten in the next round
        if (!ok) {
            gave_up = true;
            break;
        }
        // The flag was read (relaxed) by one thread; every wave now acquires at device scope, which
        // makes the packet's data, written before the flag was raised, visible to its loads.
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");

        int c = -1;
        if (well_formed) {
            for (int i = 0; i < a.n_colours; ++i)
                if (a.bounds[i] <= lo && hi <= a.bounds[i + 1]) c = i;
        }
        if (c < 0) {                              // not a range of one colour: skipped and reported
            if (threadIdx.x == 0) atomicOr(a.progress + G + 1, 1u);
        } else {
            const float* const* xs = a.x + c * np;
            const int64_t n_tiles = (hi - lo + kTile - 1) / kTile;
            // consecutive packets start on consecutive workgroups, so that small packets do not
            // all land on the first few
            const int64_t first = (int64_t(j) * n_tiles) % G;
            const int64_t mine = (int64_t(blockIdx.x) + G - first) % G;
            for (int64_t t = mine; t < n_tiles; t += G)
                mc::ru_tile<P, 1, kThreads, HAS_G, true, SS>(xs, np, lo + t * kTile, hi, a.g, a.w, a.v, hp);
        }
        if (threadIdx.x == 0) a.progress[blockIdx.x] = j + 1;
    }
    if (gave_up && threadIdx.x == 0) atomicAdd(a.progress + G, 1u);
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t value) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

__global__ void signal_kernel(uint32_t* flag, uint32_t value) {
    if (threadIdx.x == 0 && blockIdx.x == 0)
        __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// mc_packet_deliver: a copy of n elements, then -- as a launch of its own behind it in the stream, so
// that every store of the copy is complete -- one release-add of n to *flag.  (One add per workgroup
// of the copy, on the very word that the reducer's workgroups poll, serialised: about 22 ns each,
// 1 ms over the sixteen packets of a ResNet-50 step, and more the more workgroups polled.)
__global__ __launch_bounds__(kThreads) void deliver_kernel(float* dst, const float* src, int64_t n) {
    const int64_t base = int64_t(blockIdx.x) * kTile;
    const int64_t i = base + int64_t(threadIdx.x) * 4;
    if (i + 4 <= n) {
        *reinterpret_cast<float4*>(dst + i) = *reinterpret_cast<const float4*>(src + i);
    } else {
        for (int64_t e = i; e < n; ++e) dst[e] = src[e];
    }
}

__global__ void landed_kernel(uint32_t* flag, uint32_t n) {
    if (threadIdx.x == 0 && blockIdx.x == 0)
        __hip_atomic_fetch_add(flag, n, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Occupies one wavefront for about `us` microseconds (bounded by the caller): stands in for the time a
// packet spends on a wire.
__global__ void delay_kernel(uint32_t us) {
    const uint64_t t0 = wall_clock64();            // 100 MHz
    const uint64_t ticks = uint64_t(us) * 100;
    for (uint32_t i = 0; i < us * 4 + 16; ++i) {   // bounded whatever the clock does
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(16);
    }
}

template <int P>
void launch_p(bool has_g, bool ss, unsigned blocks, hipStream_t s, const PkArgs& a) {
    const dim3 grid(blocks), block(kThreads);
#define MC_PK_LAUNCH(G, SS) hipLaunchKernelGGL((packet_reducer_kernel<P, G, SS>), grid, block, 0, s, a)
    if (has_g) {
        if (ss) MC_PK_LAUNCH(true, true); else MC_PK_LAUNCH(true, false);
    } else {
        if (ss) MC_PK_LAUNCH(false, true); else MC_PK_LAUNCH(false, false);
    }
#undef MC_PK_LAUNCH
}

}  // namespace

extern "C" {

int mc_packets_reset(uint32_t* ready, int32_t n_packets, uint32_t* progress, int32_t n_blocks, void* stream) {
    if (n_packets < 0 || n_blocks < 0 || n_blocks > MC_PACKETS_MAX_BLOCKS) return MC_ERR_INVALID_ARG;
    if ((n_packets > 0 && !ready) || (n_blocks > 0 && !progress)) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(ready, 4) || !mc::aligned(progress, 4)) return MC_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_packets > 0) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(unsigned((n_packets + 255) / 256)), dim3(256), 0, s, ready,
                           int64_t(n_packets), 0u);
        MC_HIP_TRY(hipGetLastError());
    }
    if (n_blocks > 0) {
        const int64_t n = int64_t(n_blocks) + MC_PACKETS_STATUS_WORDS;
        hipLaunchKernelGGL(fill_u32_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, s, progress, n, 0u);
        MC_HIP_TRY(hipGetLastError());
    }
    return MC_OK;
}

int mc_packet_signal(uint32_t* ready, int32_t packet, uint32_t value, void* stream) {
    if (!ready || packet < 0) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(ready, 4)) return MC_ERR_ALIGN;
    hipLaunchKernelGGL(signal_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), ready + packet, value);
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

int mc_packet_deliver(void* dst, const void* src, int64_t n_elems, uint32_t* flag, void* stream) {
    if (n_elems < 0) return MC_ERR_INVALID_ARG;
    if (n_elems == 0) return MC_OK;
    if (!dst || !src || !flag) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(dst, 16) || !mc::aligned(src, 16) || !mc::aligned(flag, 4)) return MC_ERR_ALIGN;
    if (mc::overlaps(dst, uint64_t(n_elems) * 4, src, uint64_t(n_elems) * 4)) return MC_ERR_OVERLAP;
    const int64_t blocks = (n_elems + kTile - 1) / kTile;
    if (blocks > 0x7fffffff || n_elems > 0xffffffffll) return MC_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(deliver_kernel, dim3(unsigned(blocks)), dim3(kThreads), 0, s, static_cast<float*>(dst),
                       static_cast<const float*>(src), n_elems);
    MC_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(landed_kernel, dim3(1), dim3(64), 0, s, flag, uint32_t(n_elems));
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

int mc_delay(uint32_t microseconds, void* stream) {
    if (microseconds > 100000) return MC_ERR_INVALID_ARG;
    hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), microseconds);
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

int mc_reduce_update_packets(const mc_layout* L, const void* const* contrib, int32_t P, const int32_t* order,
                             void* grad_out, void* weights, void* momentum, const mc_update_spec* spec,
                             const int64_t* packets, int32_t n_packets, const uint32_t* ready,
                             uint32_t arrivals, uint32_t spin_limit, uint32_t* progress, int32_t n_blocks,
                             void* stream) {
    if (!L) return MC_ERR_INVALID_ARG;
    mc::UpdatePlan plan;
    int rc = mc::update_plan(spec, &plan);
    if (rc != MC_OK) return rc;
    if (n_packets < 0 || n_blocks < 1 || n_blocks > MC_PACKETS_MAX_BLOCKS || arrivals < 1) return MC_ERR_INVALID_ARG;
    if (L->k > kMaxColours || int64_t(L->k) * P > kPtrSlots) return MC_ERR_LIMIT;
    if (plan.up.hyper && !mc::aligned(plan.up.hyper, 4)) return MC_ERR_ALIGN;
    rc = mc::check_order(L, P, order);
    if (rc != MC_OK) return rc;
    rc = mc::check_flat_buffers(L, contrib, P, grad_out, weights, momentum, /*needs_state=*/true, /*needs_g=*/false);
    if (rc != MC_OK) return rc;
    if (n_packets == 0) return MC_OK;
    if (!packets || !ready || !progress) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(packets, 8) || !mc::aligned(ready, 4) || !mc::aligned(progress, 4)) return MC_ERR_ALIGN;
    // Every workgroup must be resident at once AND leave wave slots to whatever delivers the packets:
    // a grid that fills the device would wait for a producer that cannot start, until the poll budget
    // ends.  Two workgroups (8 of 32 wave slots) per compute unit is the most that is accepted.
    int dev = 0, cus = 0;
    MC_HIP_TRY(hipGetDevice(&dev));
    MC_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (n_blocks > 2 * cus) return MC_ERR_LIMIT;

    PkArgs a;
    for (int32_t c = 0; c < L->k; ++c)
        for (int32_t q = 0; q < P; ++q)
            a.x[c * P + q] = static_cast<const float*>(contrib[order ? order[size_t(c) * P + q] : q]);
    for (int i = L->k * P; i < kPtrSlots; ++i) a.x[i] = nullptr;
    for (int32_t c = 0; c <= L->k; ++c) a.bounds[c] = L->bounds[c];
    for (int c = L->k + 1; c <= kMaxColours; ++c) a.bounds[c] = L->N;
    a.n_colours = L->k;
    a.np = P;
    a.n_packets = n_packets;
    a.arrivals = arrivals;
    a.spin_limit = spin_limit;
    a.N = L->N;
    a.packets = packets;
    a.ready = ready;
    a.progress = progress;
    a.g = static_cast<float*>(grad_out);
    a.w = static_cast<float*>(weights);
    a.v = static_cast<float*>(momentum);
    a.up = plan.up;
    const bool ss = mc::stream_state(L, plan.state_policy);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned blocks = unsigned(n_blocks);
    switch (P) {
        case 1: launch_p<1>(a.g != nullptr, ss, blocks, s, a); break;
        case 2: launch_p<2>(a.g != nullptr, ss, blocks, s, a); break;
        case 4: launch_p<4>(a.g != nullptr, ss, blocks, s, a); break;
        case 8: launch_p<8>(a.g != nullptr, ss, blocks, s, a); break;
        default: launch_p<0>(a.g != nullptr, ss, blocks, s, a); break;
    }
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

}  // extern "C"
