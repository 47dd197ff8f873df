// Where the (condition node, token) -> stack-effect table keeps a key: two candidate buckets of
// kEffectBucketSlots 16-byte slots each.  One definition for the host builder and the kernels.
#pragma once
#include <cstdint>

#if defined(__HIP__)
#define PRE3_HOST_DEVICE __host__ __device__
#else
#define PRE3_HOST_DEVICE
#endif

namespace pre3 {

constexpr int kEffectBucketSlots = 4;

PRE3_HOST_DEVICE inline void effect_buckets(uint32_t node, uint32_t tok, uint32_t mask, uint32_t *b1, uint32_t *b2) {
    uint32_t x = node * 0x9E3779B1u + tok * 0x85EBCA77u;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    *b1 = x & mask;
    uint32_t y = (x * 0x846CA68Bu) ^ (x >> 13);
    y ^= y >> 16;
    *b2 = y & mask;
    if (*b2 == *b1) *b2 = (*b1 + 1) & mask;
}

// A slot of the table, four 32-bit words:
//   w0 = condition node
//   w1 = token | k << 21 | c << 29        c = number of pushed states if they are inline (1 or 2), else 0
//   w2 = (peak + 32768) << 16 | (second inline state >> 12) << 8 | n_push
//   w3 = first inline state | (second inline state & 0xFFF) << 20        (c > 0; states below 2^20)
//      = offset of the pushed states in the pool                        (c == 0)
// w0 = -1 marks an empty slot.  Tokens are below 2^21, k and n_push at most 255.
constexpr int kEffectInlineStateBits = 20;

struct EffectFields {
    int k, peak, np, inline_count, x0, x1;     // x0, x1: inline states; x0: pool offset when inline_count == 0
};

PRE3_HOST_DEVICE inline bool effect_slot_matches(uint32_t w0, uint32_t w1, uint32_t node, uint32_t tok) {
    return w0 == node && (w1 & 0x1FFFFFu) == tok;
}

PRE3_HOST_DEVICE inline EffectFields effect_unpack(uint32_t w1, uint32_t w2, uint32_t w3) {
    EffectFields f;
    f.k = (int)((w1 >> 21) & 0xFFu);
    f.inline_count = (int)((w1 >> 29) & 3u);
    f.peak = (int)(w2 >> 16) - 32768;
    f.np = (int)(w2 & 0xFFu);
    if (f.inline_count > 0) {
        f.x0 = (int)(w3 & 0xFFFFFu);
        f.x1 = (int)((w3 >> 20) | (((w2 >> 8) & 0xFFu) << 12));
    } else {
        f.x0 = (int)w3;
        f.x1 = 0;
    }
    return f;
}

}  // namespace pre3
