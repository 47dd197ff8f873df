// gfx950 kernels over the logits: masking in place, and the greedy choice among allowed tokens.
// Both stream the [batch, vocab] bf16 logits once and are bound by HBM bandwidth.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.hpp"

namespace pre3 {

namespace {

constexpr uint32_t kNegInfPair = 0xFF80FF80u;   // two bf16 -inf

// ---------------------------------------------------------------------------- apply

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


// ------------------------------------------------------------------- masked argmax

// Order-preserving map of a non-NaN binary32 pattern to an unsigned key (-0 counts as +0).
__device__ __forceinline__ uint32_t float_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

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

// Greedy choice among the allowed tokens without writing the masked logits back: a row's logits
// are read once (groups of 8 whose mask byte is zero are not read at all).  blockIdx.x = row,
// blockIdx.y = segment of the row.  A lane keeps the largest value it has seen among allowed
// entries and its id (ids ascend within a lane, so `>` keeps the first of equal values; a NaN
// never compares greater; an allowed -inf, which can only win if nothing else is allowed, is
// remembered separately by lanes that have seen nothing larger); lanes and waves are then
// combined through the packed word
//   key(value) << 32 | ~id,
// whose maximum is the largest value and, among equal values, the smallest id; 0 = no candidate.  With one segment
// per row the block writes out[b] itself; otherwise it stores its word in partial[b][segment]
// and masked_argmax_finish_kernel combines the segments.  (Combining them inside this kernel
// with device-scope atomics and a last-arrival counter was measured: rows that finish early
// then cost tens of microseconds per launch.)  The mask bytes of the next pass are fetched
// while the logits of the current one are in flight.
constexpr int kArgBlock = 1024;
constexpr int kArgUnroll = 4;
__global__ __launch_bounds__(kArgBlock) void masked_argmax_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int groups_per_seg, int vec_ok, unsigned long long *__restrict__ partial, int32_t *__restrict__ out) {
    __shared__ unsigned long long s_part[kArgBlock / 64];
    const int b = blockIdx.x, seg = blockIdx.y, n_seg = gridDim.y, tid = threadIdx.x;
    const int groups = (vocab + 7) >> 3;
    const int g_lo = seg * groups_per_seg, g_hi = min(groups, g_lo + groups_per_seg);
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    float best_v = -INFINITY;
    int best_t = -1, ninf_t = -1;                       // ninf_t: first allowed entry that is exactly -inf
    uint32_t m[kArgUnroll], m_next[kArgUnroll];
#pragma unroll
    for (int u = 0; u < kArgUnroll; ++u) {
        const int g = g_lo + tid + u * kArgBlock;
        m[u] = g < g_hi ? mrow[g] : 0u;
    }
    for (int g0 = g_lo + tid; g0 < g_hi; g0 += kArgBlock * kArgUnroll) {
        uint4 v[kArgUnroll];
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const int g = g0 + u * kArgBlock;
            if (m[u] != 0u && vec_ok && g * 8 + 8 <= vocab) v[u] = stream_load(lrow + (size_t)g * 8);
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const int g = g0 + kArgBlock * kArgUnroll + u * kArgBlock;
            m_next[u] = g < g_hi ? mrow[g] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) {
            const uint32_t mu = m[u];
            if (mu == 0u) continue;
            const int t0 = (g0 + u * kArgBlock) * 8;
            if (vec_ok && t0 + 8 <= vocab) {
                const uint32_t x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float f0 = (mu >> (2 * k)) & 1u ? __uint_as_float(x[k] << 16) : -INFINITY;
                    const float f1 = (mu >> (2 * k + 1)) & 1u ? __uint_as_float(x[k] & 0xFFFF0000u) : -INFINITY;
                    if (f0 > best_v) { best_v = f0; best_t = t0 + 2 * k; }
                    if (f1 > best_v) { best_v = f1; best_t = t0 + 2 * k + 1; }
                }
                if (best_t < 0 && ninf_t < 0) {
#pragma unroll
                    for (int k = 7; k >= 0; --k) {     // descending: the smallest k is assigned last
                        const uint32_t h = (k & 1) ? (x[k >> 1] >> 16) : (x[k >> 1] & 0xFFFFu);
                        if (((mu >> k) & 1u) && h == 0xFF80u) ninf_t = t0 + k;
                    }
                }
            } else {                                   // ragged tail or unaligned rows: one logit at a time
                for (int k = 0; k < 8 && t0 + k < vocab; ++k) {
                    const uint32_t h = lrow[t0 + k];
                    const float f = (mu >> k) & 1u ? __uint_as_float(h << 16) : -INFINITY;
                    if (f > best_v) { best_v = f; best_t = t0 + k; }
                    if (best_t < 0 && ninf_t < 0 && ((mu >> k) & 1u) && h == 0xFF80u) ninf_t = t0 + k;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) m[u] = m_next[u];
    }
    unsigned long long mine = 0ull;
    if (best_t >= 0) mine = ((unsigned long long)float_key(best_v) << 32) | (0xFFFFFFFFu - (uint32_t)best_t);
    else if (ninf_t >= 0) mine = ((unsigned long long)float_key(-INFINITY) << 32) | (0xFFFFFFFFu - (uint32_t)ninf_t);
    mine = wave_max_u64(mine);
    if ((tid & 63) == 0) s_part[tid >> 6] = mine;
    __syncthreads();
    if (tid < 64) {
        mine = wave_max_u64(tid < kArgBlock / 64 ? s_part[tid] : 0ull);
        if (tid == 0) s_part[0] = mine;
    }
    __syncthreads();
    mine = s_part[0];
    if (n_seg > 1) {
        if (tid == 0) partial[(size_t)b * n_seg + seg] = mine;
        return;
    }
    if (tid == 0) out[b] = mine != 0ull ? (int32_t)(0xFFFFFFFFu - (uint32_t)mine) : -1;
}

// One wave per row: combines the row's segments.
constexpr int kArgFinishRows = 4;
__global__ __launch_bounds__(64 * kArgFinishRows) void masked_argmax_finish_kernel(
    int batch, int n_seg, const unsigned long long *__restrict__ partial, int32_t *__restrict__ out) {
    const int lane = threadIdx.x & 63, b = blockIdx.x * kArgFinishRows + (threadIdx.x >> 6);
    if (b >= batch) return;
    unsigned long long mine = 0ull;
    for (int i = lane; i < n_seg; i += 64) {
        const unsigned long long p = partial[(size_t)b * n_seg + i];
        mine = p > mine ? p : mine;
    }
    mine = wave_max_u64(mine);
    if (lane == 0) out[b] = mine != 0ull ? (int32_t)(0xFFFFFFFFu - (uint32_t)mine) : -1;
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

// blocks per row of the argmax kernel: enough blocks to fill the chip, and every block at least
// one full pass wide
static int masked_argmax_segments(int batch, int vocab, int n_compute_units) {
    const int groups = (vocab + 7) / 8;
    const int max_seg = (groups + kArgBlock * kArgUnroll - 1) / (kArgBlock * kArgUnroll);
    int n_seg = batch > 0 ? (n_compute_units + batch - 1) / batch : 1;
    n_seg = n_seg > max_seg ? max_seg : n_seg;
    return n_seg < 1 ? 1 : n_seg;
}

size_t masked_argmax_workspace_bytes(int batch, int vocab, int n_compute_units) {
    return (size_t)batch * masked_argmax_segments(batch, vocab, n_compute_units) * sizeof(unsigned long long);
}

hipError_t launch_masked_argmax(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                                int n_compute_units, unsigned long long *workspace, int32_t *out, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32, groups = (vocab + 7) / 8;
    const int n_seg = masked_argmax_segments(batch, vocab, n_compute_units);
    const int groups_per_seg = (groups + n_seg - 1) / n_seg;
    const int vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    hipLaunchKernelGGL(masked_argmax_kernel, dim3(batch, n_seg), dim3(kArgBlock), 0, stream, logits, bitmask, vocab,
                       row_stride, n_words, groups_per_seg, vec_ok, workspace, out);
    if (n_seg > 1)
        hipLaunchKernelGGL(masked_argmax_finish_kernel, dim3((batch + kArgFinishRows - 1) / kArgFinishRows),
                           dim3(64 * kArgFinishRows), 0, stream, batch, n_seg, workspace, out);
    return hipGetLastError();
}

}  // namespace pre3
