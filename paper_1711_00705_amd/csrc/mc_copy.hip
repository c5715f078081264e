// A plain 128-bit device-to-device copy: the yardstick the other kernels are measured
// against (achievable HBM bandwidth) and the known-size traffic used to calibrate hardware
// counters.  One 16-byte vector per thread, non-temporal load and write-through (agent-scope)
// store: the fastest of the plain copies measured on this part.
#include <hip/hip_runtime.h>

#include "mc_internal.h"
#include "mc_mem.h"

namespace {

constexpr int kThreads = 64;   // one wavefront per workgroup measured fastest for every streaming kernel here
constexpr int kVecPerThread = 1;

__global__ __launch_bounds__(kThreads) void copy_kernel(uint4* __restrict__ dst,
                                                        const uint4* __restrict__ src, int64_t n_vec) {
    const int64_t base = int64_t(blockIdx.x) * (kThreads * kVecPerThread) + threadIdx.x;
    uint4 r[kVecPerThread];
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t i = base + int64_t(j) * kThreads;
        if (i < n_vec) {
            typedef uint32_t native4 __attribute__((ext_vector_type(4)));
            const native4 t = __builtin_nontemporal_load(reinterpret_cast<const native4*>(src + i));
            r[j] = make_uint4(t.x, t.y, t.z, t.w);
        }
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t i = base + int64_t(j) * kThreads;
        if (i < n_vec) {
            typedef uint32_t native4 __attribute__((ext_vector_type(4)));
            const native4 val = {r[j].x, r[j].y, r[j].z, r[j].w};
            mc::store128_sc1(dst + i, val);
        }
    }
}

}  // namespace

extern "C" int mc_copy(void* dst, const void* src, int64_t n_bytes, void* stream) {
    if (n_bytes < 0 || (n_bytes & 15) != 0) return MC_ERR_INVALID_ARG;
    if (n_bytes == 0) return MC_OK;
    if (!dst || !src) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(dst, 16) || !mc::aligned(src, 16)) return MC_ERR_ALIGN;
    if (mc::overlaps(dst, uint64_t(n_bytes), src, uint64_t(n_bytes))) return MC_ERR_OVERLAP;
    const int64_t n_vec = n_bytes / 16;
    const int64_t per_block = int64_t(kThreads) * kVecPerThread;
    const int64_t blocks = (n_vec + per_block - 1) / per_block;
    if (blocks > 0x7fffffff) return MC_ERR_INVALID_ARG;
    hipLaunchKernelGGL(copy_kernel, dim3(unsigned(blocks)), dim3(kThreads), mc::lds_reservation(MC_OPT_LDS_CAP_PACK, kThreads),
                       static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), n_vec);
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}
