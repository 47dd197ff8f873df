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


// ------------------------------------------------------------------- masked top-k

// Order-preserving 16-bit key of a non-NaN bf16 pattern (-0 counts as +0).  Valid values map to
// 0x007F (-inf) .. 0xFF80 (+inf); 0 is never produced and marks "no candidate".
__device__ __forceinline__ uint32_t bf16_key(uint32_t h) {
    if (h == 0x8000u) h = 0u;
    return (h & 0x8000u) ? (~h & 0xFFFFu) : (h | 0x8000u);
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// The k best candidates of one segment of one row (blockIdx.x = row, blockIdx.y = segment of
// kTopkSeg tokens): every thread keeps the keys of its 16 tokens in registers (0 = masked, NaN or
// beyond the vocabulary), so the logits are read once.  The block then finds by bisection on the
// 16-bit key the largest threshold T that at least kk = min(k, candidates) keys reach, takes every
// key above T and, of the keys equal to T, the first kk - (number above) in id order (an ordered
// block scan of the per-thread counts gives each its rank).  The chosen ones are written as
//   key << 32 | ~id     (distinct words; larger = better value, then smaller id; 0 = empty slot)
// to out[(row * n_seg + segment) * k ..], in no particular order.
constexpr int kTopkBlock = 1024;
constexpr int kTopkSeg = 16 * kTopkBlock;
__global__ __launch_bounds__(kTopkBlock) void masked_topk_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int vec_ok, int k, unsigned long long *__restrict__ out) {
    __shared__ int s_cnt[kTopkBlock / 64];
    __shared__ unsigned long long s_out[kTopkMax];
    __shared__ int s_n;
    const int b = blockIdx.x, seg = blockIdx.y, n_seg = gridDim.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    const int n_mask_bytes = n_words * 4;
    uint32_t key[16];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int t0 = seg * kTopkSeg + (tid + half * kTopkBlock) * 8;
        const uint32_t m = (t0 < vocab && (t0 >> 3) < n_mask_bytes) ? mrow[t0 >> 3] : 0u;
        uint32_t h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = 0x7FC0u;           // NaN: no candidate
        if (m != 0u) {
            if (vec_ok && t0 + 8 <= vocab) {
                const uint4 v = stream_load(lrow + (size_t)t0);
                const uint32_t x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) { h[2 * j] = x[j] & 0xFFFFu; h[2 * j + 1] = x[j] >> 16; }
            } else {
                for (int j = 0; j < 8 && t0 + j < vocab; ++j) h[j] = lrow[t0 + j];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = ((m >> j) & 1u) && (h[j] & 0x7FFFu) <= 0x7F80u;
            key[half * 8 + j] = ok ? bf16_key(h[j]) : 0u;
        }
    }
    if (tid == 0) s_n = 0;
    if (tid < kTopkMax) s_out[tid] = 0ull;
    auto count_ge = [&](uint32_t T) -> int {                  // keys >= T over the whole block
        int c = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) c += key[i] >= T ? 1 : 0;
        c = wave_sum(c);
        if (lane == 0) s_cnt[wave] = c;
        __syncthreads();
        int total = 0;
#pragma unroll
        for (int w = 0; w < kTopkBlock / 64; ++w) total += s_cnt[w];
        __syncthreads();
        return total;
    };
    const int candidates = count_ge(1u);
    const int kk = candidates < k ? candidates : k;
    unsigned long long *dst = out + ((size_t)b * n_seg + seg) * (size_t)k;
    if (kk == 0) {
        if (tid < k) dst[tid] = 0ull;
        return;
    }
    uint32_t lo = 1u, hi = 0x10000u;                          // count_ge(lo) >= kk > count_ge(hi) = above
    int above = 0;
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        const int c = count_ge(mid);
        if (c >= kk) lo = mid;
        else { hi = mid; above = c; }
    }
    const uint32_t T = lo;
    const int need_equal = kk - above;                        // >= 1, and at least that many keys equal T
    // rank of every key equal to T in id order: the first halves of all threads come before the second halves
    int e0 = 0, e1 = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { e0 += key[i] == T ? 1 : 0; e1 += key[8 + i] == T ? 1 : 0; }
    int packed = e0 | (e1 << 16), incl = packed;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (lane == 63) s_cnt[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kTopkBlock / 64; ++w) {
        const int c = s_cnt[w];
        if (w < wave) before += c;
        all += c;
    }
    const int excl = before + incl - packed;
    int rank0 = excl & 0xFFFF, rank1 = (all & 0xFFFF) + (excl >> 16);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t kv = key[i];
        bool take = kv > T;
        if (kv == T) {
            int &rank = i < 8 ? rank0 : rank1;
            take = rank < need_equal;
            ++rank;
        }
        if (take) {
            const uint32_t id = (uint32_t)(seg * kTopkSeg + (tid + (i >> 3) * kTopkBlock) * 8 + (i & 7));
            const int slot = atomicAdd(&s_n, 1);
            if (slot < kTopkMax) s_out[slot] = ((unsigned long long)kv << 32) | (0xFFFFFFFFu - id);
        }
    }
    __syncthreads();
    if (tid < k) dst[tid] = s_out[tid];
}

// Merges the segments' candidates of one row (n_cand words, 0 = empty) and writes the k best in
// order: a word's rank is the number of larger words (all non-zero words are distinct).
__global__ __launch_bounds__(256) void masked_topk_finish_kernel(
    const unsigned long long *__restrict__ cand, int n_cand, int k, const uint16_t *__restrict__ logits,
    int64_t row_stride, int32_t *__restrict__ out_ids, uint16_t *__restrict__ out_vals) {
    extern __shared__ unsigned long long s_cand[];
    __shared__ int s_valid;
    const int b = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) s_valid = 0;
    __syncthreads();
    int mine = 0;
    for (int i = tid; i < n_cand; i += 256) {
        const unsigned long long c = cand[(size_t)b * n_cand + i];
        s_cand[i] = c;
        mine += c != 0ull ? 1 : 0;
    }
    if (mine) atomicAdd(&s_valid, mine);
    __syncthreads();
    const int n_valid = s_valid;
    for (int i = tid; i < n_cand; i += 256) {
        const unsigned long long c = s_cand[i];
        if (c == 0ull) continue;
        int rank = 0;
        for (int j = 0; j < n_cand; ++j) rank += s_cand[j] > c ? 1 : 0;
        if (rank < k) {
            const uint32_t id = 0xFFFFFFFFu - (uint32_t)c;
            out_ids[(size_t)b * k + rank] = (int32_t)id;
            if (out_vals) out_vals[(size_t)b * k + rank] = logits[(size_t)b * row_stride + id];
        }
    }
    for (int j = (n_valid < k ? n_valid : k) + tid; j < k; j += 256) {
        out_ids[(size_t)b * k + j] = -1;
        if (out_vals) out_vals[(size_t)b * k + j] = 0xFF80u;
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

static int masked_topk_segments(int vocab) { return (vocab + kTopkSeg - 1) / kTopkSeg; }

size_t masked_topk_workspace_bytes(int batch, int vocab) {
    return (size_t)batch * masked_topk_segments(vocab) * kTopkMax * sizeof(unsigned long long);
}

hipError_t launch_masked_topk(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                              int k, unsigned long long *workspace, int32_t *out_ids, uint16_t *out_vals,
                              hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    const int n_words = (vocab + 31) / 32, n_seg = masked_topk_segments(vocab);
    const int n_cand = n_seg * k;
    if (k < 1 || k > kTopkMax || n_seg > 65535 || (size_t)n_cand * sizeof(unsigned long long) > 65536) return hipErrorInvalidValue;
    const int vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    hipLaunchKernelGGL(masked_topk_kernel, dim3(batch, n_seg), dim3(kTopkBlock), 0, stream, logits, bitmask, vocab, row_stride,
                       n_words, vec_ok, k, workspace);
    hipLaunchKernelGGL(masked_topk_finish_kernel, dim3(batch), dim3(256), (size_t)n_cand * sizeof(unsigned long long), stream,
                       workspace, n_cand, k, logits, row_stride, out_ids, out_vals);
    return hipGetLastError();
}

}  // namespace pre3
