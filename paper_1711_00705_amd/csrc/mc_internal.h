// Internal declarations shared by the translation units of libmc (never installed).
#pragma once

#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstdint>
#include <mutex>
#include <utility>
#include <vector>

#include "mc.h"

namespace mc {

// Elements of the flat payload that one workgroup of the pack / unpack kernels covers: one
// wavefront, one 16-byte vector per thread (as for the update kernels: against 256 threads x 2
// vectors, pack and unpack gain 4-5 % at ResNet-50 and VGG-16 size, 1 % at GoogLeNet size).
#ifndef MC_PACK_TILE_ELEMS
#define MC_PACK_TILE_ELEMS 256
#endif
constexpr int64_t kPackTileElems = MC_PACK_TILE_ELEMS;
// Granularity of the "first tensor" lookup table: one entry per this many flat elements.  It is
// the colour alignment, so every tile of every kernel (pack tiles, and reduce tiles, which
// start at colour bounds) begins on an entry.
constexpr int64_t kLookupElems = MC_COLOUR_ALIGN_ELEMS;
static_assert(kPackTileElems % kLookupElems == 0, "pack tiles must start on lookup entries");
// Device pointers that fit in one pack / unpack launch's kernel-argument block.
constexpr int kPackMaxPtrs = 256;
constexpr int kMaxDevices = 16;

struct DeviceTables {
    bool ready = false;
    int64_t* off = nullptr;         // n+1 flat offsets
    int32_t* tile_first = nullptr;  // per kLookupElems flat elements: first tensor that may intersect them
    int32_t* unit_tensor = nullptr; // per unit slot: its tensor, -1 for padding (null when the layout has no unit table)
    int32_t* unit_first = nullptr;  // at c + t: index in colour c of the first unit of tensor t
};

}  // namespace mc

struct mc_layout {
    int32_t n = 0;
    int32_t k = 0;
    int64_t N = 0;
    int64_t chunk = 0;                // colour chunk length C (a multiple of 256; 0 when N == 0)
    std::vector<int64_t> off;         // n+1
    std::vector<int64_t> bounds;      // k+1
    std::vector<int32_t> tile_first;  // ceil(N / kLookupElems) + 1
    // Tensor-aligned units (the fused step's work items): inside colour c, tensor t is cut into
    // runs of 256 elements counted from the TENSOR's first element, so that a unit's accesses to
    // the per-layer tensors start on a 1 KiB boundary of the tensor whatever its flat offset is
    // (a tile grid laid over the flat index instead leaves every tensor-side access of a tile
    // straddling cache lines, shared with the neighbouring tile, once an earlier tensor's length
    // is not a multiple of 32).  A run cut by a colour bound or by the tensor's end is a shorter
    // unit.  Every colour owns units_per_colour slots (the largest count; unused slots hold -1),
    // so a slot's colour is its index divided by that number.  Empty when k > 32 or the slot count
    // does not fit 31 bits.
    std::vector<int32_t> unit_tensor;  // k * units_per_colour
    // Index in colour c of the first unit of tensor t, at position c + t (colours and tensors both
    // advance along the payload, so c + t names the pair uniquely): n + k entries.
    std::vector<int32_t> unit_first;
    int32_t units_per_colour = 0;
    // Parity of the next whole-payload update call with automatic sweep direction (see
    // sweep_reversed()): the one member that changes after prepare; it never affects a result.
    mutable std::atomic<uint32_t> sweep{0};
    std::mutex mu;                    // guards dev[] during prepare / destroy
    mc::DeviceTables dev[mc::kMaxDevices];
};

// The device-resident list of one tensor pointer per layer of a layout.
struct mc_tensor_set {
    const mc_layout* layout = nullptr;
    int device = -1;
    void** d_ptrs = nullptr;                             // device: n pointers
    std::vector<const void*> ptrs;                       // host copy
    std::vector<std::pair<uintptr_t, uintptr_t>> spans;  // non-empty tensors' [begin, end), sorted
};

namespace mc {

// Records a failed HIP call for mc_last_hip_error() and returns MC_ERR_HIP.
int hip_fail(hipError_t e);

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Do the byte ranges [a, a+na) and [b, b+nb) intersect?  Empty ranges never do.
inline bool overlaps(const void* a, uint64_t na, const void* b, uint64_t nb) {
    if (na == 0 || nb == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

// Returns the device tables of L for the current device, uploading them on first use.
int device_tables(mc_layout* L, const DeviceTables** out);

constexpr int kNoSuchOption = -1000;
int option(int which);   // kNoSuchOption for an unknown option

// Workgroup shape of the reduce_update / fused_step kernels for one launch.
struct Shape {
    int threads;   // 64 or 256
    int vectors;   // 16-byte vectors per thread per tile: 1 or 2
    int64_t tile() const { return int64_t(threads) * 4 * vectors; }
};
// 64 threads x 1 vector (one wavefront per workgroup, a tile of exactly one colour-alignment unit)
// measured fastest or within noise on every configuration: against 256 threads x 2 vectors the fused
// step gains 1 % on the back-to-back ResNet-50 step, 2 % with eight contributions, 3-4 % on
// GoogLeNet- and VGG-16-sized steps and 2-4 % when nothing is cache-resident; 128 x 1 and 256 x 1
// are within 1 % of it.  So it is the default for every launch; MC_OPT_RU_SHAPE = 2 forces 256 x 2.
Shape shape_for(int64_t elems, int n_terms, bool stream_state);

// Bytes of (unused) dynamic LDS to reserve per workgroup, which caps how many workgroups a compute
// unit holds at once.  These kernels need no LDS; the reservation is a throttle.  With every wave
// slot filled (32 per compute unit) a streaming kernel keeps about 50 MB of loads in flight across
// the chip, spread over a 5-6 MB window of each of its streams, far more than the 12-16 MB that
// cover HBM's latency -- and the wider the window, the fewer requests find their DRAM row still open.
// A bare loop with this access mix (64-thread workgroups, one 16-byte vector per thread and stream)
// is fastest at 8 wavefronts per compute unit: +3-5 % on a cold ResNet-50-sized step, +6-7 % at
// VGG-16 size, +2-3 % warm.  How few wavefronts a real kernel tolerates depends on how long each
// one sits on lookups before its first load (two batches of scalar loads in the fused step, one in
// reduce_update) and on where the traffic comes from, so the automatic setting of the update
// kernels (update_lds_reservation) goes by the cache regime of the call.  Measured on the fused
// step (% of the 8 TB/s peak; wavefronts per compute unit 32 / 16 / 14 / 12 / 10 / 8):
//   ResNet-50, P = 4, back to back (state cache-resident)  89.3 / 89.0 / 87.2 / 84.7 / 82.6 / 80.7
//   ResNet-50, P = 4, cold                                 79.4 / 80.2 / 80.9 / 79.1 / 76.7 / 74.2
//   ResNet-50, P = 8, cold                                 75.7 / 74.5 / 75.9 / 78.0 / 78.5 / 78.7
//   GoogLeNet, P = 4, cold                                 74.4 / 74.9 / 75.2 / 72.9 / 71.9 / 69.4
//   VGG-16, P = 4 (state larger than the cache)            79.3 / 80.9 / 81.8 / 82.3 / 81.2 / 79.7
// i.e. nothing to gain while the state is cached, and otherwise a constant amount of loads in flight:
// 14 wavefronts x 6 KB, 8 x 10 KB, 12 x 6 KB.
// lds_reservation serves the copy-shaped kernels (MC_OPT_LDS_CAP_PACK; they only lose with a cap:
// default none) and returns an explicit MC_OPT_LDS_CAP_UPDATE setting as it is; `threads` per
// workgroup of the launch.
unsigned lds_reservation(int which, int threads);
// state_cached: every colour of the call updates, with the resident policy; terms: contributions per
// colour, 0 for a launch whose colours differ in term count or update flag.
unsigned update_lds_reservation(const mc_layout* L, int threads, bool state_cached, int terms, bool per_layer);

// Cache treatment of weights and momentum for a call on layout L: `policy` is the caller's
// MC_STATE_* value (MC_STATE_DEFAULT defers to MC_OPT_STATE_POLICY).  The library cannot know
// whether anything ran between two steps, so the default is the policy that suits steps run back to
// back (resident: +15 % on the ResNet-50-sized step, and with alternating sweeps still +3 % on the
// VGG-16-sized one whose state is four times the cache); a caller whose steps are separated by a
// forward / backward pass asks for streaming (+6 % when the state is cold).
bool stream_state(const mc_layout* L, int policy);

// Should this whole-payload update call walk the payload backwards?  `sweep` is the caller's
// MC_SWEEP_* value.  Automatic: weights and momentum are the only data that come back every step;
// when they exceed the memory-side cache and are kept resident, sweeping in the same direction every
// step evicts each line long before it is needed again, while alternating the direction makes the
// most recently written part the first to be read (measured on a bare loop: 480 MB of state
// 5.8 -> 6.7 TB/s, 1.1 GB 5.4 -> 5.8 TB/s; no gain when the state fits or is streamed).  The layout
// keeps the parity of its automatic calls in one relaxed atomic counter -- the only thing in a
// layout that changes after mc_layout_prepare, and it affects the order of the tiles, never a result.
bool sweep_reversed(const mc_layout* L, int sweep, bool stream_state);

// Argument checks shared by the entry points that work on flat buffers.
// check_order: P in range and every row of the order table a permutation of 0..P-1.
// check_flat_buffers: null / alignment / overlap of {contrib[0..P), grad_out, weights, momentum}:
// nothing that is written may overlap anything else; contributions are only read and may repeat.
// needs_state: weights and momentum are required; needs_g: grad_out is.
int check_order(const mc_layout* L, int32_t P, const int32_t* order);
int check_flat_buffers(const mc_layout* L, const void* const* contrib, int32_t P, const void* grad_out,
                       const void* weights, const void* momentum, bool needs_state, bool needs_g);

struct UpdateParams;
// A validated mc_update_spec: the kernels' argument form plus the host-side launch choices.
struct UpdatePlan;
int update_plan(const mc_update_spec* spec, UpdatePlan* out);

}  // namespace mc

#define MC_HIP_TRY(expr)                                  \
    do {                                                  \
        hipError_t mc_e_ = (expr);                        \
        if (mc_e_ != hipSuccess) return mc::hip_fail(mc_e_); \
    } while (0)
