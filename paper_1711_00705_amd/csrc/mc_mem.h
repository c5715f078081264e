// Device-side memory access helpers shared by every kernel of the library.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace mc {

// 128-bit store to global memory with the agent-scope bit (`sc1`): the line is written through
// instead of lingering dirty in the die's L2.  Measured faster than both the default and the
// non-temporal store for data that is not read again soon (updated weights / momentum: +3 % on the
// ResNet-50-sized step; copy-shaped kernels: +15 % at 28 MB, +2 % at 100 MB, equal at 550 MB).
//
// There is no C++ spelling for a 128-bit store with that bit, hence the one-instruction asm; this is
// the only place in the library that issues it.  The compiler still orders the asm after the
// instructions that produce its operands.  The `s_nop 1` is required: a store of more than 64 bits
// keeps reading its data registers for two wait states after issue, the compiler's hazard
// recogniser cannot see into the asm, and a VALU write to one of those registers in the very next
// instruction corrupts the stored value (seen as 8688 wrong words in a 25 M-word pack before the
// nop was added).
//
// V: any 16-byte vector type (ext_vector_type(4) of float or uint32_t).
template <typename V>
__device__ __forceinline__ void store128_sc1(void* p, const V& val) {
    static_assert(sizeof(V) == 16, "a 128-bit store");
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(val) : "memory");
}

}  // namespace mc
