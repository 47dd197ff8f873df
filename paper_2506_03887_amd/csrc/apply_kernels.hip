// gfx950 kernel that masks the logits in place: one pass over the [batch, vocab] bf16 logits,
// bound by HBM bandwidth.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.hpp"
#include "stream_access.hpp"

namespace pre3 {

namespace {

constexpr int kApplyBlock = 256;
constexpr int kApplySpan = kApplyBlock * 8;            // logits per block
constexpr int64_t kMaskBytesInL2 = 16 << 20;            // masks up to this size are read where they were written (half of the L2s)

// One block per span of kApplySpan logits of one row.  kRowsByXcd = false: blockIdx.y = row,
// blockIdx.x = span.  kRowsByXcd = true (one-dimensional grid): workgroups go round-robin to the
// chip's eight XCDs in the order of their linear id, and the kernels that write the mask run row b
// in block b, that is on XCD b % 8 -- so block L takes a row of XCD L % 8's, and the mask bytes it
// reads are still in that XCD's L2 (B = 256: 34.8 -> 33.7 us per step, B = 1,024: 111.5 -> 109.0;
// a mask beyond the L2s gains nothing and the scattered rows cost 2 %, so large batches keep the
// two-dimensional grid).  A lane owns one group of 8 consecutive
// logits (16 bytes), so that every access of a wave is one contiguous 1 KiB.  Fully allowed groups
// are not touched, fully masked groups are overwritten without being read, mixed groups are read,
// patched and written back: the mask byte's bits become the AND masks of the group's four registers
// (sign-extending bit extracts, a byte permute), and one bit-select per register puts -inf where a
// bit is clear.  The kernel is bound by the turnover of its waves (a mask byte, then the logits,
// then the store) as much as by HBM: the fewer instructions a wave issues, the faster it runs, and
// variants that give a lane several groups -- 4 KiB apart or side by side -- were slower (26.6 us
// and 52.8 us against 23.6 us at B = 256, V = 128,256).
constexpr int kXcds = 8;
template <bool kRowsByXcd>
__global__ __launch_bounds__(kApplyBlock) void apply_mask_vec8_kernel(uint16_t *__restrict__ logits,
                                                                     const uint32_t *__restrict__ bitmask,
                                                                     int vocab, int64_t row_stride, int n_words,
                                                                     int batch, int spans) {
    int b = blockIdx.y, span = blockIdx.x;
    if (kRowsByXcd) {
        const int xcd = blockIdx.x % kXcds, at = blockIdx.x / kXcds;
        b = (at / spans) * kXcds + xcd;
        span = at % spans;
        if (b >= batch) return;
    }
    const int groups = (vocab + 7) >> 3;
    const int g = span * kApplyBlock + threadIdx.x;
    uint32_t mu = 0xFFu;
    if (g < groups) mu = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words)[g];   // little endian: byte g of the row = bits of group g
    // a 128-byte line (the groups of eight consecutive lanes) is written whole or not at all: lines
    // written in part cost the memory system far more than the bytes saved
    const unsigned long long changed = __ballot(mu != 0xFFu);
    if (g >= groups || !((changed >> (threadIdx.x & 56)) & 0xFFull)) return;
    uint16_t *p = logits + (size_t)b * row_stride + (size_t)g * 8;
    if (g * 8 + 8 <= vocab) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (mu != 0u) v = stream_load(p);
        uint32_t *x = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)mu, 2 * k, 1);        // all ones if the token is allowed
            const uint32_t hi = (uint32_t)__builtin_amdgcn_sbfe((int)mu, 2 * k + 1, 1);
            const uint32_t allow = __builtin_amdgcn_perm(hi, lo, 0x05040100u);              // low half from lo, high half from hi
            x[k] = (x[k] & allow) | (~allow & kNegInfPair);
        }
        stream_store(v, p);
    } else {
        for (int k = 0; g * 8 + k < vocab; ++k)
            if (!((mu >> k) & 1u)) p[k] = 0xFF80;
    }
}

// Fallback for rows that are not 16-byte aligned: one lane per logit.
__global__ __launch_bounds__(256) void apply_mask_scalar_kernel(uint16_t *__restrict__ logits,
                                                                 const uint32_t *__restrict__ bitmask, int batch,
                                                                 int vocab, int64_t row_stride, int n_words) {
    const int64_t total = (int64_t)batch * vocab;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(i / vocab), t = (int)(i - (int64_t)b * vocab);
        if (!((bitmask[(size_t)b * n_words + (t >> 5)] >> (t & 31)) & 1u))
            logits[(size_t)b * row_stride + t] = 0xFF80;
    }
}

__global__ void timestamp_kernel(int64_t *out) { *out = (int64_t)wall_clock64(); }

}  // namespace

hipError_t launch_timestamp(int64_t *out, hipStream_t stream) {
    hipLaunchKernelGGL(timestamp_kernel, dim3(1), dim3(1), 0, stream, out);
    return hipGetLastError();
}

hipError_t launch_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                             hipStream_t stream) {
    if (batch == 0 || vocab == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32;
    const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    if (aligned && batch <= 65535) {
        const int spans = (vocab + kApplySpan - 1) / kApplySpan;
        const int64_t by_xcd = (int64_t)spans * kXcds * ((batch + kXcds - 1) / kXcds);
        if ((int64_t)batch * n_words * 4 <= kMaskBytesInL2 && by_xcd <= 0x7FFFFFFF)
            hipLaunchKernelGGL(apply_mask_vec8_kernel<true>, dim3((unsigned)by_xcd), dim3(kApplyBlock), 0, stream, logits, bitmask,
                               vocab, row_stride, n_words, batch, spans);
        else
            hipLaunchKernelGGL(apply_mask_vec8_kernel<false>, dim3(spans, batch), dim3(kApplyBlock), 0, stream, logits, bitmask,
                               vocab, row_stride, n_words, batch, spans);
    } else {
        const int64_t total = (int64_t)batch * vocab;
        const int64_t want = (total + 255) / 256;
        const int grid = (int)(want < 65536 ? want : 65536);
        hipLaunchKernelGGL(apply_mask_scalar_kernel, dim3(grid), dim3(256), 0, stream, logits, bitmask, batch, vocab,
                           row_stride, n_words);
    }
    return hipGetLastError();
}

}  // namespace pre3
