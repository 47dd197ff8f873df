// gfx950 kernel that masks the logits in place: one pass over the [batch, vocab] bf16 logits,
// bound by HBM bandwidth.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.hpp"
#include "stream_access.hpp"

namespace pre3 {

namespace {

constexpr int kApplyBlock = 256;
constexpr int kApplyUnroll = 1;        // 16-byte groups per lane (measured: more waves beat more loads per lane)
constexpr int kApplySpan = kApplyBlock * kApplyUnroll * 8;   // logits per block

// blockIdx.y = row, blockIdx.x = span of kApplySpan logits.  A lane owns kApplyUnroll groups of 8
// consecutive logits (16 bytes), one per pass, so that every pass of a wave is one contiguous
// 1 KiB access.  Fully allowed groups are not touched, fully masked groups are overwritten
// without being read, mixed groups are read, patched and written back.  In-place
// read-modify-write of the logits streams at about 5.4 TB/s on MI355X whatever the unroll or
// block size; one group per lane was the fastest.
__global__ __launch_bounds__(kApplyBlock) void apply_mask_vec8_kernel(uint16_t *__restrict__ logits,
                                                                     const uint32_t *__restrict__ bitmask,
                                                                     int vocab, int64_t row_stride, int n_words) {
    const int b = blockIdx.y;
    const int groups = (vocab + 7) >> 3;
    const int g0 = blockIdx.x * (kApplyBlock * kApplyUnroll) + threadIdx.x;
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    uint16_t *lrow = logits + (size_t)b * row_stride;
    uint32_t m[kApplyUnroll];
    uint4 v[kApplyUnroll];
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {
        const int g = g0 + u * kApplyBlock;
        m[u] = g < groups ? mrow[g] : 0xFFu;            // little endian: byte g of the row = bits of group g
    }
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {                // all loads of the lane are in flight together
        const int g = g0 + u * kApplyBlock;
        if (m[u] != 0xFFu && m[u] != 0u && g * 8 + 8 <= vocab) v[u] = stream_load(lrow + (size_t)g * 8);
    }
#pragma unroll
    for (int u = 0; u < kApplyUnroll; ++u) {
        const int g = g0 + u * kApplyBlock;
        const uint32_t mu = m[u];
        if (mu == 0xFFu) continue;
        uint16_t *p = lrow + (size_t)g * 8;
        if (g * 8 + 8 <= vocab) {
            if (mu == 0u) {
                stream_store(make_uint4(kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair), p);
            } else {
                uint32_t *x = reinterpret_cast<uint32_t *>(&v[u]);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (!((mu >> (2 * k)) & 1u)) x[k] = (x[k] & 0xFFFF0000u) | 0xFF80u;
                    if (!((mu >> (2 * k + 1)) & 1u)) x[k] = (x[k] & 0x0000FFFFu) | 0xFF800000u;
                }
                stream_store(v[u], p);
            }
        } else {
            for (int k = 0; g * 8 + k < vocab; ++k)
                if (!((mu >> k) & 1u)) p[k] = 0xFF80;
        }
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

}  // namespace

hipError_t launch_apply_mask(uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                             hipStream_t stream) {
    if (batch == 0 || vocab == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32;
    const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    if (aligned && batch <= 65535) {
        const dim3 grid((vocab + kApplySpan - 1) / kApplySpan, batch);
        hipLaunchKernelGGL(apply_mask_vec8_kernel, grid, dim3(kApplyBlock), 0, stream, logits, bitmask, vocab, row_stride,
                           n_words);
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
