// The greedy choice among allowed bf16 logits: order keys, the candidate word that lanes, waves and
// blocks are combined through, and the exact float-compare pass for the rows the keys cannot decide.
// Shared by the sampler kernel and the one-launch greedy step kernel.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace pre3 {

namespace {

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    const uint32_t lo = __shfl_xor((uint32_t)v, mask), hi = __shfl_xor((uint32_t)(v >> 32), mask);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = shfl_xor_u64(v, off);
        v = o > v ? o : v;
    }
    return v;
}

// Signed order key of a bf16 pattern: for non-NaN patterns a larger key is a larger value.  Valid
// values map to kOrderNegInf .. kOrderPosInf (-0 to -1, +0 to 0), negative NaN patterns below
// kOrderNegInf, positive NaN patterns above kOrderPosInf.
constexpr int kOrderNegInf = -32641, kOrderPosInf = 32640;
__device__ __forceinline__ int bf16_order(uint32_t h) {
    const int v = (int)(int16_t)h;
    return v ^ ((v >> 15) & 0x7FFF);
}
typedef short PackedS16 __attribute__((ext_vector_type(2)));
// The same for the two patterns of one register; halves the AND mask `allow` clears get the lowest key.
__device__ __forceinline__ uint32_t bf16_order_keys(uint32_t x) {                     // the two keys, nothing masked
    const uint32_t negative = __builtin_bit_cast(uint32_t, __builtin_bit_cast(PackedS16, x) >> 15);
    return x ^ (negative & 0x7FFF7FFFu);
}
__device__ __forceinline__ uint32_t mask_order_keys(uint32_t key, uint32_t allow) { // halves that `allow` clears get the lowest key
    return (key & allow) | (~allow & 0x80008000u);
}
__device__ __forceinline__ uint32_t bf16_order_pair(uint32_t x, uint32_t allow) {
    return mask_order_keys(bf16_order_keys(x), allow);
}
__device__ __forceinline__ uint32_t packed_max_s16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(PackedS16, a), __builtin_bit_cast(PackedS16, b)));
}
// A lane's or a block's candidate: order key (with -0 counted as +0) above the complement of the id,
// so that the largest word is the largest value and, among equal values, the smallest id; 0 = none.
__device__ __forceinline__ unsigned long long argmax_word(int order, int id) {
    if (order == -1) order = 0;
    return ((unsigned long long)(uint32_t)(order + 32768) << 32) | (0xFFFFFFFFu - (uint32_t)id);
}

// Half a mask byte -> the AND masks of two registers of packed 16-bit pairs (bit i of the nibble allows half i).
// Sixteen entries of 8 bytes: lanes that read the same entry are served together and different entries lie in
// different LDS banks, where a table of whole bytes (256 entries of 16 bytes) puts every sixteenth entry on the
// same banks.  mask_nibble_table_init: by the first sixteen threads, followed by a barrier of the caller.
__device__ __forceinline__ void mask_nibble_table_init(uint2 *table, int tid) {
    if (tid < 16) {
        uint32_t a[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) a[q] = (((tid >> (2 * q)) & 1) ? 0x0000FFFFu : 0u) | (((tid >> (2 * q + 1)) & 1) ? 0xFFFF0000u : 0u);
        table[tid] = make_uint2(a[0], a[1]);
    }
}
__device__ __forceinline__ uint4 expand_mask_byte(const uint2 *table, uint32_t mask_byte) {
    const uint2 lo = table[mask_byte & 15u], hi = table[mask_byte >> 4];
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
}

constexpr int kArgBlock = 1024;

__device__ __forceinline__ unsigned long long argmax_block_max(unsigned long long mine, unsigned long long *s_part, int tid) {
    mine = wave_max_u64(mine);
    __syncthreads();                                    // s_part may still be read from an earlier round
    if ((tid & 63) == 0) s_part[tid >> 6] = mine;
    __syncthreads();
    if (tid < 64) {
        mine = wave_max_u64(tid < kArgBlock / 64 ? s_part[tid] : 0ull);
        if (tid == 0) s_part[kArgBlock / 64] = mine;
    }
    __syncthreads();
    return s_part[kArgBlock / 64];
}

// The segment's candidate with one float compare per token: a lane keeps the largest value it has
// seen among allowed entries and its id (ids ascend within a lane, so `>` keeps the first of equal
// values, -0 and +0 are equal, a NaN never compares greater); an allowed -inf, which can only win if
// nothing else is allowed, is remembered separately by lanes that have seen nothing larger.  Used
// for the rare rows on which the packed keys of masked_argmax_kernel cannot decide.
__device__ __forceinline__ unsigned long long argmax_segment_by_compare_inline(const uint16_t *__restrict__ lrow,
                                                                                const uint8_t *__restrict__ mrow, int g_lo,
                                                                                int g_hi, int vocab, int tid) {
    float best_v = -INFINITY;
    int best_t = -1, ninf_t = -1;
    for (int g = g_lo + tid; g < g_hi; g += kArgBlock) {
        const uint32_t mu = mrow[g];
        if (mu == 0u) continue;
        for (int k = 0; k < 8 && g * 8 + k < vocab; ++k) {
            if (!((mu >> k) & 1u)) continue;
            const uint32_t h = lrow[g * 8 + k];
            const float f = __uint_as_float(h << 16);
            if (f > best_v) { best_v = f; best_t = g * 8 + k; }
            if (best_t < 0 && ninf_t < 0 && h == 0xFF80u) ninf_t = g * 8 + k;
        }
    }
    if (best_t >= 0) return argmax_word(bf16_order(__float_as_uint(best_v) >> 16), best_t);
    if (ninf_t >= 0) return argmax_word(kOrderNegInf, ninf_t);
    return 0ull;
}
// The same as a call (keeps the register count of a kernel's main loop apart from this pass's).
__device__ __noinline__ unsigned long long argmax_segment_by_compare(const uint16_t *__restrict__ lrow,
                                                                     const uint8_t *__restrict__ mrow, int g_lo, int g_hi,
                                                                     int vocab, int tid) {
    return argmax_segment_by_compare_inline(lrow, mrow, g_lo, g_hi, vocab, tid);
}

}  // namespace

}  // namespace pre3
