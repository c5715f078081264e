// The SGD step of one element, shared by the reduce_update and fused_step kernels.
//
// Section 3, Algorithm 1 ends with "perform SGD"; the paper gives no formula.  Implemented:
// heavy-ball momentum with L2 decay folded into the gradient,
//     d = g + wd*w;  v' = mu*v + d;  w' = w - lr*v'
// and, with the Nesterov flag (the look-ahead form used by the Torch ResNet recipe the paper
// builds on),
//     d = g + wd*w;  v' = mu*v + d;  w' = w - lr*(d + mu*v').
// Every multiply and add is rounded once to binary32; files that include this header are
// compiled with floating-point contraction off.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace mc {

// As passed in kernel arguments: immediate values, or a device pointer to {lr, mu, wd} that the
// kernel reads when it runs (so that a captured graph can be replayed with a new learning rate).
struct UpdateParams {
    float lr, mu, wd;
    const float* hyper;  // device, 3 floats, or null
    int32_t nesterov;
};

struct Hyper {
    float lr, mu, wd;
    bool nesterov;
};

__device__ __forceinline__ Hyper resolve(const UpdateParams& p) {
    Hyper h;
    if (p.hyper) {
        h.lr = p.hyper[0];
        h.mu = p.hyper[1];
        h.wd = p.hyper[2];
    } else {
        h.lr = p.lr;
        h.mu = p.mu;
        h.wd = p.wd;
    }
    h.nesterov = p.nesterov != 0;
    return h;
}

// Each line is one rounding.
__device__ __forceinline__ void sgd(float g, float& w, float& v, const Hyper& h) {
    const float decay = h.wd * w;
    const float d = g + decay;
    const float mv = h.mu * v;
    const float vn = mv + d;
    float dir = vn;
    if (h.nesterov) {
        const float look = h.mu * vn;
        dir = d + look;
    }
    const float step = h.lr * dir;
    w = w - step;
    v = vn;
}

}  // namespace mc
