// The SGD step of one element, shared by the reduce_update and fused_step kernels.
//
// Section 3, Algorithm 1 ends with an SGD step on every GPU; the paper gives no formula.  Implemented:
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

#include "mc_mem.h"

namespace mc {

// As passed in kernel arguments: immediate values, or a device pointer to {lr, mu, wd} that the
// kernel reads when it runs (so that a captured graph can be replayed with a new learning rate).
struct UpdateParams {
    float lr, mu, wd;
    const float* hyper;  // device, 3 floats, or null
    int32_t nesterov;
    int32_t state_store_sc1;  // store policy of weights and momentum, see store_state()
};

// Host side: what a call asked for.
struct UpdatePlan {
    UpdateParams up;
    int32_t state_policy;  // MC_STATE_*
    int32_t sweep;         // MC_SWEEP_*
};

struct Hyper {
    float lr, mu, wd;
    bool nesterov;
    bool state_store_sc1;
};

// The immediate values sit in the kernel's argument block and arrive through scalar loads.  The
// device triple is read through a volatile pointer on purpose: with two plain loads the compiler
// turns "argument block or device memory" into ONE vector load through a selected address, and that
// load -- issued by every wavefront, from an argument block that may live in host memory -- is then
// in front of every tile even when no device triple is in use.
__device__ __forceinline__ Hyper resolve(const UpdateParams& p) {
    Hyper h;
    h.lr = p.lr;
    h.mu = p.mu;
    h.wd = p.wd;
    if (p.hyper) {
        const volatile float* dev = p.hyper;
        h.lr = dev[0];
        h.mu = dev[1];
        h.wd = dev[2];
    }
    h.nesterov = p.nesterov != 0;
    h.state_store_sc1 = p.state_store_sc1 != 0;
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

// How a kernel treats weights and momentum in the caches (a compile-time choice of the launch).
//   resident : plain loads, stores written through with the agent-scope bit (`sc1`, or plain when
//              the store_sc1 flag is off).  Back-to-back steps on a model whose state fits the
//              256 MB memory-side cache find it there: +20 % on the ResNet-50-sized step.
//   streaming: non-temporal loads and stores, like the contributions.  When the state cannot be
//              in the cache anyway (a forward / backward pass ran since the last step, or the state
//              is larger than the cache) this is 3-5 % faster, because the state no longer
//              displaces anything and is not kept dirty in L2.
template <bool STREAM>
__device__ __forceinline__ float4 load_state(const float* p) {
    typedef float native4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) native4 global4;  // device global memory
    const global4* gp = (const global4*)p;
    const native4 r = STREAM ? __builtin_nontemporal_load(gp) : *gp;
    return make_float4(r.x, r.y, r.z, r.w);
}

template <bool STREAM>
__device__ __forceinline__ void store_state(float* p, const float4& q, bool sc1) {
    typedef float native4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) native4 global4;
    const native4 val = {q.x, q.y, q.z, q.w};
    if (STREAM) {
        __builtin_nontemporal_store(val, (global4*)p);
    } else if (sc1) {
        store128_sc1(p, val);
    } else {
        *(global4*)p = val;
    }
}

}  // namespace mc
