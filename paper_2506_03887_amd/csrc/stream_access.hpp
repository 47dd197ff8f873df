// Non-temporal 16-byte accesses to the logits and the mask rows, shared by the kernels that stream them.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace pre3 {

// 16-byte accesses marked non-temporal: the logits pass through once, and lines marked this way
// are the first to leave L2, so the automaton's tables survive the pass for the next kernel.
typedef unsigned int NativeUint4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load(const uint16_t *p) {
    const NativeUint4 x = __builtin_nontemporal_load(reinterpret_cast<const NativeUint4 *>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void stream_store(uint4 v, uint16_t *p) {
    const NativeUint4 x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<NativeUint4 *>(p));
}

// The same store for a mask row: the row is read once, by the kernel that masks the logits, and
// lines that linger dirty in the writer's L2 slow that kernel down (B = 2,048: 232 us per step with
// plain stores of the mask rows against 209 us; B = 256: 35.0 against 34.6 us).
__device__ __forceinline__ void stream_store(uint4 v, uint4 *p) {
    const NativeUint4 x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<NativeUint4 *>(p));
}

constexpr uint32_t kNegInfPair = 0xFF80FF80u;   // two bf16 -inf

}  // namespace pre3
