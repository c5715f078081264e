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

// Elements of the flat payload that one workgroup of the pack / unpack kernels covers.
#ifndef MC_PACK_TILE_ELEMS
#define MC_PACK_TILE_ELEMS 2048
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
};

}  // namespace mc

struct mc_layout {
    int32_t n = 0;
    int32_t k = 0;
    int64_t N = 0;
    std::vector<int64_t> off;         // n+1
    std::vector<int64_t> bounds;      // k+1
    std::vector<int32_t> tile_first;  // ceil(N / kLookupElems) + 1
    // Parity of the next whole-payload update call: successive steps sweep the payload in opposite
    // directions (see sweep_reversed()).
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

int option(int which);
// Should this whole-payload update call walk the payload backwards?  Weights and momentum are the
// only data that come back every step.  When they exceed the 256 MB memory-side cache, sweeping
// the payload in the same direction every step evicts each line long before it is needed again;
// alternating the direction makes the most recently written part the first to be read.  Measured on
// a bare loop: 480 MB of state 5.8 -> 6.7 TB/s, 1.1 GB (VGG-16) 5.4 -> 5.8 TB/s; no gain when the
// state fits, so smaller payloads keep one direction.  The result does not depend on the direction
// (the step is elementwise).
bool sweep_reversed(const mc_layout* L);
// Vectors per thread per tile for a launch over `elems` elements (honours MC_OPT_RU_UNROLL).
int unroll_for(int64_t elems);

struct UpdateParams;
// Validates a caller's spec and converts it to the kernels' argument form.
int update_params(const mc_update_spec* spec, UpdateParams* out);

}  // namespace mc

#define MC_HIP_TRY(expr)                                  \
    do {                                                  \
        hipError_t mc_e_ = (expr);                        \
        if (mc_e_ != hipSuccess) return mc::hip_fail(mc_e_); \
    } while (0)
