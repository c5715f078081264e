// The learning-rate schedule of Section 5 (host arithmetic) and the device-side scalar triple
// {lr, mu, wd} that lets a captured step be replayed with a new rate.
#include <hip/hip_runtime.h>

#include <cmath>

#include "mc_internal.h"

namespace {

__global__ void hyper_write_kernel(float* hyper, float lr, float mu, float wd) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        hyper[0] = lr;
        hyper[1] = mu;
        hyper[2] = wd;
    }
}

}  // namespace

extern "C" {

int mc_hyper_write(float* hyper_dev, float lr, float mu, float wd, void* stream) {
    if (!hyper_dev) return MC_ERR_INVALID_ARG;
    if (!mc::aligned(hyper_dev, 4)) return MC_ERR_ALIGN;
    hipLaunchKernelGGL(hyper_write_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       hyper_dev, lr, mu, wd);
    MC_HIP_TRY(hipGetLastError());
    return MC_OK;
}

int mc_lr_schedule(float base_lr, int32_t batch_per_gpu, int32_t n_workers, float warmup_epochs,
                   float drop_every_epochs, float epoch, float* lr_out) {
    if (!lr_out) return MC_ERR_INVALID_ARG;
    if (!std::isfinite(base_lr) || base_lr <= 0.0f || batch_per_gpu < 1 || n_workers < 1)
        return MC_ERR_INVALID_ARG;
    if (!(warmup_epochs >= 0.0f) || !std::isfinite(warmup_epochs)) return MC_ERR_INVALID_ARG;
    if (!(drop_every_epochs > 0.0f) || !std::isfinite(drop_every_epochs)) return MC_ERR_INVALID_ARG;
    if (!(epoch >= 0.0f) || !std::isfinite(epoch)) return MC_ERR_INVALID_ARG;
    const double target = double(base_lr) * double(batch_per_gpu) * double(n_workers) / 256.0;
    double lr;
    if (double(epoch) < double(warmup_epochs)) {
        lr = double(base_lr) + (target - double(base_lr)) * double(epoch) / double(warmup_epochs);
    } else {
        const double drops = std::floor(double(epoch) / double(drop_every_epochs));
        lr = target / std::pow(10.0, drops);
    }
    *lr_out = float(lr);
    return MC_OK;
}

}  // extern "C"
