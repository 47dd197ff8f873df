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
// 0x007F (-inf) .. 0xFF80 (+inf); 0 is never produced.
__device__ __forceinline__ uint32_t bf16_key(uint32_t h) {
    if (h == 0x8000u) h = 0u;
    return (h & 0x8000u) ? (~h & 0xFFFFu) : (h | 0x8000u);
}

// A candidate travels between the stages as the word  key << 21 | (0x1FFFFF - id)  (id < 2^21):
// distinct words, larger = better value, then smaller id; 0 = no candidate.
constexpr int kTopkIdBits = 21;
constexpr int kTopkWordBits = 16 + kTopkIdBits;
constexpr uint32_t kTopkIdMask = (1u << kTopkIdBits) - 1u;
__device__ __forceinline__ unsigned long long topk_word(uint32_t key, uint32_t id) {
    return ((unsigned long long)key << kTopkIdBits) | (unsigned long long)(kTopkIdMask - id);
}

// Number of (lane, element) pairs for which pred(i) holds, by ballots (scalar population counts: no
// LDS, no cross-lane data movement).
template <int kPer, class Pred>
__device__ __forceinline__ int wave_count(Pred pred) {
    int c = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) c += __popcll(__ballot(pred(i)));
    return c;
}

// The largest threshold t (16 bits, found bit by bit from the top) that at least `want` of the
// wave's keys reach; *reached = how many do.  want >= 1 and at least `want` keys are non-zero.
template <int kPer, class KeyAt>
__device__ __forceinline__ uint32_t wave_key_threshold(KeyAt key_at, int n_nonzero, int want, int *reached) {
    uint32_t T = 0u;
    int at_T = n_nonzero;
    for (int bit = 15; bit >= 0 && at_T != want; --bit) {
        const uint32_t t = T | (1u << bit);
        const int c = wave_count<kPer>([&](int i) { return key_at(i) >= t; });
        if (c >= want) { T = t; at_T = c; }
    }
    *reached = at_T;
    return T == 0u ? 1u : T;                                  // want == n_nonzero: every candidate
}

// Selection of the kk = min(k, candidates) best of the elements a wave holds, kPer per lane:
// key_at(i) (0 = no candidate, else the 16-bit value key) and pref_at(i) (distinct among equal keys,
// 1 .. 2^pref_bits - 1, larger = preferred, i.e. smaller id).  First the largest key threshold T
// that at least kk keys reach; then, if more keys equal T than are still needed, the largest
// preference threshold P that enough of them reach.  Selected: key > T, or key == T and pref >= P.
// All lanes run in lockstep and obtain the same T, P, kk.
template <int kPer, class KeyAt, class PrefAt>
__device__ __forceinline__ void wave_select(KeyAt key_at, PrefAt pref_at, int pref_bits, int k, uint32_t *T_out,
                                            uint32_t *P_out, int *kk_out) {
    const int nz = wave_count<kPer>([&](int i) { return key_at(i) != 0u; });
    const int kk = nz < k ? nz : k;
    *kk_out = kk;
    *T_out = 0x10000u;                                        // nothing selected
    *P_out = 0u;
    if (kk == 0) return;
    int at_T;
    const uint32_t T = wave_key_threshold<kPer>(key_at, nz, kk, &at_T);
    *T_out = T;
    if (at_T == kk) return;                                   // every key >= T is selected (P = 0)
    const int above = wave_count<kPer>([&](int i) { return key_at(i) > T; });
    const int need = kk - above;                              // of the keys equal to T, the `need` most preferred
    uint32_t P = 0u;
    int at_P = at_T - above;                                  // count(key == T && pref >= P)
    for (int bit = pref_bits - 1; bit >= 0 && at_P != need; --bit) {
        const uint32_t t = P | (1u << bit);
        const int c = wave_count<kPer>([&](int i) { return key_at(i) == T && pref_at(i) >= t; });
        if (c >= need) { P = t; at_P = c; }
    }
    *P_out = P;
}

// The kk-th largest of the S distinct non-zero words of an LDS list (1 <= kk <= S), found bit by bit
// from the top by one wave; lane l looks at the words l, l + 64, ... (kept in registers when there
// are at most 256 of them).  Words >= the result are the kk largest.
__device__ __forceinline__ unsigned long long wave_kth_largest(const unsigned long long *list, int S, int kk, int lane) {
    if (kk >= S) return 1ull;
    constexpr int kRegs = 4;
    unsigned long long r[kRegs];
#pragma unroll
    for (int i = 0; i < kRegs; ++i) r[i] = i * 64 + lane < S ? list[i * 64 + lane] : 0ull;
    const bool in_regs = S <= 64 * kRegs;
    unsigned long long prefix = 0ull;
    for (int bit = kTopkWordBits - 1; bit >= 0; --bit) {
        const unsigned long long t = prefix | (1ull << bit);
        int c = 0;
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < kRegs; ++i)
                if (i * 64 < S) c += __popcll(__ballot(r[i] >= t));
        } else {
            for (int r0 = 0; r0 < S; r0 += 64) c += __popcll(__ballot(r0 + lane < S && list[r0 + lane] >= t));
        }
        if (c >= kk) {
            prefix = t;
            if (c == kk) break;
        }
    }
    return prefix;
}

// The k best candidates of one segment of one row (blockIdx.x = row, blockIdx.y = segment of
// kTopkSeg tokens).  Every thread keeps the 16-bit keys of its 32 tokens in registers, two per
// register (0 = masked, NaN or beyond the vocabulary), so the logits are read once.
//   Fast path: from the per-thread maxima the block derives a lower bound M of the segment's k-th
//   largest key (at least k threads hold a key >= M), so only keys >= M can be among the k best:
//   usually a few times k of them.  They are collected in an LDS list; with at most one per thread
//   every thread ranks its word against the list, otherwise wave 0 selects the k best bit by bit.
//   If the list overflows -- only possible when thousands of keys tie with M -- every wave selects
//   the k best of its own 2,048 tokens (ties by id) and wave 0 merges the waves' lists.
// The k words are written, in no particular order, to out[(row * n_seg + segment) * k ..], 0-padded.
// The phases after the load cost about a microsecond per block whatever its size, so a block covers
// as many tokens as its registers hold.
constexpr int kTopkBlock = 512;
constexpr int kTopkWaves = kTopkBlock / 64;
constexpr int kTopkPerThread = 32;
constexpr int kTopkSeg = kTopkPerThread * kTopkBlock;
constexpr int kTopkList = 2048;
__global__ __launch_bounds__(kTopkBlock) void masked_topk_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int vec_ok, int k, unsigned long long *__restrict__ out) {
    __shared__ unsigned long long s_list[kTopkList];
    __shared__ unsigned long long s_sel[kTopkWaves][kTopkMax];
    __shared__ int s_nz[kTopkWaves];
    __shared__ uint32_t s_wbound[kTopkWaves];
    __shared__ int s_n[kTopkWaves];
    __shared__ int s_count;
    const int b = blockIdx.x, seg = blockIdx.y, n_seg = gridDim.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    const int n_mask_bytes = n_words * 4;
    unsigned long long *dst = out + ((size_t)b * n_seg + seg) * (size_t)k;
    // element e of a thread (0 .. 31) is token  seg * kTopkSeg + rel(e); its key is half (e & 1) of kp[e >> 1]
    auto rel = [&](int e) { return (tid + (e >> 3) * kTopkBlock) * 8 + (e & 7); };
    uint32_t kp[kTopkPerThread / 2];
    auto key_at = [&](int e) { return (kp[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu; };
    uint32_t m[kTopkPerThread / 8];
    uint4 v[kTopkPerThread / 8];
#pragma unroll
    for (int g = 0; g < kTopkPerThread / 8; ++g) {
        const int t0 = seg * kTopkSeg + (tid + g * kTopkBlock) * 8;
        m[g] = (t0 < vocab && (t0 >> 3) < n_mask_bytes) ? mrow[t0 >> 3] : 0u;
    }
#pragma unroll
    for (int g = 0; g < kTopkPerThread / 8; ++g) {
        const int t0 = seg * kTopkSeg + (tid + g * kTopkBlock) * 8;
        v[g] = make_uint4(0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u);   // NaN: no candidate
        if (m[g] != 0u) {
            if (vec_ok && t0 + 8 <= vocab) {
                v[g] = stream_load(lrow + (size_t)t0);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = t0 + j < vocab ? (uint32_t)lrow[t0 + j] : 0x7FC0u;
                v[g] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            }
        }
    }
#pragma unroll
    for (int g = 0; g < kTopkPerThread / 8; ++g) {
        const uint32_t x[4] = {v[g].x, v[g].y, v[g].z, v[g].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = x[j] & 0xFFFFu, hi = x[j] >> 16;
            const bool ok_lo = ((m[g] >> (2 * j)) & 1u) && (lo & 0x7FFFu) <= 0x7F80u;
            const bool ok_hi = ((m[g] >> (2 * j + 1)) & 1u) && (hi & 0x7FFFu) <= 0x7F80u;
            kp[g * 4 + j] = (ok_lo ? bf16_key(lo) : 0u) | ((ok_hi ? bf16_key(hi) : 0u) << 16);
        }
    }
    uint32_t best = 0u;
#pragma unroll
    for (int e = 0; e < kTopkPerThread; ++e) best = key_at(e) > best ? key_at(e) : best;
    // A lower bound of the segment's k-th largest key from the threads' maxima: wave w takes the
    // q_w-th largest of its 64 maxima, q_w = min(j, threads of w that hold a candidate), with the
    // smallest j for which the q_w add up to k; the smallest of these is reached by at least k keys.
    const int nz_wave = __popcll(__ballot(best != 0u));
    if (lane == 0) s_nz[wave] = nz_wave;
    if (tid == 0) s_count = 0;
    if (lane == 0) s_n[wave] = 0;
    s_sel[wave][lane] = 0ull;
    __syncthreads();
    int quota = 0, holders = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) holders += s_nz[w];
    if (holders >= k) {
        for (quota = 1; quota < 64; ++quota) {
            int sum = 0;
#pragma unroll
            for (int w = 0; w < kTopkWaves; ++w) sum += s_nz[w] < quota ? s_nz[w] : quota;
            if (sum >= k) break;
        }
    }
    {
        uint32_t mine = 0x10000u;                             // no candidate in this wave
        if (nz_wave > 0) {
            mine = 1u;                                        // fewer than k holders in the block: every candidate
            if (quota > 0) {
                int reached;
                mine = wave_key_threshold<1>([&](int) { return best; }, nz_wave, nz_wave < quota ? nz_wave : quota, &reached);
            }
        }
        if (lane == 0) s_wbound[wave] = mine;
    }
    __syncthreads();
    uint32_t bound = 0x10000u;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) bound = s_wbound[w] < bound ? s_wbound[w] : bound;
    if (bound == 0x10000u) {                                  // no candidate in the segment
        if (tid < k) dst[tid] = 0ull;
        return;
    }
    if (best >= bound) {
#pragma unroll
        for (int e = 0; e < kTopkPerThread; ++e)
            if (key_at(e) >= bound) {
                const int slot = atomicAdd(&s_count, 1);
                if (slot < kTopkList) s_list[slot] = topk_word(key_at(e), (uint32_t)(seg * kTopkSeg + rel(e)));
            }
    }
    __syncthreads();
    const int S = s_count;
    if (S <= kTopkBlock) {
        // the usual case: one listed word per thread, its rank = number of larger words (every thread
        // reads the same LDS word at a time: a broadcast), the k best write themselves in order
        if (tid < S) {
            const unsigned long long w = s_list[tid];
            int rank = 0;
#pragma unroll 8
            for (int j = 0; j < S; ++j) rank += s_list[j] > w ? 1 : 0;
            if (rank < k) dst[rank] = w;
        }
        if (tid >= S && tid < k) dst[tid] = 0ull;
        return;
    }
    if (S <= kTopkList) {
        if (wave != 0) return;
        const int kk = S < k ? S : k;
        const unsigned long long thr = wave_kth_largest(s_list, S, kk, lane);
        int base = 0;
        for (int r0 = 0; r0 < S; r0 += 64) {
            const unsigned long long w = r0 + lane < S ? s_list[r0 + lane] : 0ull;
            const bool take = w >= thr && w != 0ull;
            const unsigned long long mm = __ballot(take);
            if (take) dst[base + __popcll(mm & ((1ull << lane) - 1ull))] = w;
            base += __popcll(mm);
        }
        if (lane >= kk && lane < k) dst[lane] = 0ull;
        return;
    }
    // thousands of ties: exact selection per wave, then a merge by wave 0
    auto pref_at = [&](int e) { return (uint32_t)(kTopkSeg - rel(e)); };     // 1 .. kTopkSeg, larger = smaller id
    uint32_t T, P;
    int kk;
    wave_select<kTopkPerThread>(key_at, pref_at, 15, k, &T, &P, &kk);
#pragma unroll
    for (int e = 0; e < kTopkPerThread; ++e)
        if (key_at(e) > T || (key_at(e) == T && pref_at(e) >= P)) {
            const int slot = atomicAdd(&s_n[wave], 1);
            if (slot < kTopkMax) s_sel[wave][slot] = topk_word(key_at(e), (uint32_t)(seg * kTopkSeg + rel(e)));
        }
    __syncthreads();
    if (wave != 0) return;
    unsigned long long c[kTopkWaves];
#pragma unroll
    for (int i = 0; i < kTopkWaves; ++i) c[i] = s_sel[i][lane];      // slot `lane` of every wave (empty slots are 0)
    auto ckey_at = [&](int i) { return (uint32_t)(c[i] >> kTopkIdBits); };
    auto cpref_at = [&](int i) { return c[i] != 0ull ? ((uint32_t)c[i] & kTopkIdMask) + 1u : 0u; };
    wave_select<kTopkWaves>(ckey_at, cpref_at, kTopkIdBits + 1, k, &T, &P, &kk);
    int base = 0;                                             // compact the selected words into dst[0 .. kk)
#pragma unroll
    for (int i = 0; i < kTopkWaves; ++i) {
        const bool take = c[i] != 0ull && (ckey_at(i) > T || (ckey_at(i) == T && cpref_at(i) >= P));
        const unsigned long long mm = __ballot(take);
        if (take) dst[base + __popcll(mm & ((1ull << lane) - 1ull))] = c[i];
        base += __popcll(mm);
    }
    if (lane >= kk && lane < k) dst[lane] = 0ull;
}

// Merges the segments' candidates of one row with one wave: n_cand words (0 = empty), at most
// kTopkFinishPer per lane.  As above, the k-th largest of the 64 per-lane maxima bounds the k-th
// largest word from below; the words that reach it go to an LDS list.  Up to 256 listed words are
// ranked directly (a word's rank = number of larger words) and those ranked below k written in
// order; a longer list is first cut to its k best bit by bit.
constexpr int kTopkFinishPer = 16;
__global__ __launch_bounds__(64) void masked_topk_finish_kernel(
    const unsigned long long *__restrict__ cand, int n_cand, int k, const uint16_t *__restrict__ logits,
    int64_t row_stride, int32_t *__restrict__ out_ids, uint16_t *__restrict__ out_vals) {
    __shared__ unsigned long long s_list[64 * kTopkFinishPer];
    __shared__ unsigned long long s_best[kTopkMax];
    const int b = blockIdx.x, lane = threadIdx.x;
    unsigned long long c[kTopkFinishPer], top = 0ull;
#pragma unroll
    for (int i = 0; i < kTopkFinishPer; ++i) {
        const int at = i * 64 + lane;
        c[i] = at < n_cand ? cand[(size_t)b * n_cand + at] : 0ull;
        top = c[i] > top ? c[i] : top;
    }
    // lower bound: the min(k, lanes with a candidate)-th largest of the lanes' best words
    const int nz = __popcll(__ballot(top != 0ull));
    const int kq = nz < k ? nz : k;
    unsigned long long bound = 1ull;
    if (kq < nz) {
        unsigned long long prefix = 0ull;
        for (int bit = kTopkWordBits - 1; bit >= 0; --bit) {
            const unsigned long long t = prefix | (1ull << bit);
            const int n = __popcll(__ballot(top >= t));
            if (n >= kq) {
                prefix = t;
                if (n == kq) break;
            }
        }
        bound = prefix;
    }
    int S = 0;
#pragma unroll
    for (int i = 0; i < kTopkFinishPer; ++i) {
        const bool keep = c[i] != 0ull && c[i] >= bound;
        const unsigned long long m = __ballot(keep);
        if (keep) s_list[S + __popcll(m & ((1ull << lane) - 1ull))] = c[i];
        S += __popcll(m);
    }
    __builtin_amdgcn_wave_barrier();
    const int kk = S < k ? S : k;
    auto emit = [&](unsigned long long w, int rank) {
        const uint32_t id = kTopkIdMask - ((uint32_t)w & kTopkIdMask);
        out_ids[(size_t)b * k + rank] = (int32_t)id;
        if (out_vals) out_vals[(size_t)b * k + rank] = logits[(size_t)b * row_stride + id];
    };
    if (S <= 256) {
        // the usual case: every listed word is ranked directly (rank = number of larger words; all
        // lanes read the same LDS word at a time)
        unsigned long long w[4];
        int rank[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = i * 64 + lane < S ? s_list[i * 64 + lane] : ~0ull;
#pragma unroll 8
        for (int j = 0; j < S; ++j) {
            const unsigned long long o = s_list[j];
#pragma unroll
            for (int i = 0; i < 4; ++i) rank[i] += o > w[i] ? 1 : 0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i * 64 + lane < S && rank[i] < k) emit(w[i], rank[i]);
    } else {
        s_best[lane] = 0ull;
        __builtin_amdgcn_wave_barrier();
        const unsigned long long thr = kk > 0 ? wave_kth_largest(s_list, S, kk, lane) : ~0ull;
        int base = 0;
        for (int r0 = 0; r0 < S; r0 += 64) {
            const unsigned long long w = r0 + lane < S ? s_list[r0 + lane] : 0ull;
            const bool take = w >= thr && w != 0ull;
            const unsigned long long m = __ballot(take);
            if (take) s_best[base + __popcll(m & ((1ull << lane) - 1ull))] = w;
            base += __popcll(m);
        }
        __builtin_amdgcn_wave_barrier();
        const unsigned long long mine = s_best[lane];         // kk <= 64 selected words, one per lane
        int rank = 0;
        for (int j = 0; j < kk; ++j) rank += s_best[j] > mine ? 1 : 0;
        if (mine != 0ull) emit(mine, rank);
    }
    if (lane >= kk && lane < k) {
        out_ids[(size_t)b * k + lane] = -1;
        if (out_vals) out_vals[(size_t)b * k + lane] = 0xFF80u;
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

bool masked_topk_fits(int vocab, int k) {
    return k >= 1 && k <= kTopkMax && vocab >= 1 && vocab <= (1 << kTopkIdBits) &&
           masked_topk_segments(vocab) * k <= 64 * kTopkFinishPer;
}

size_t masked_topk_workspace_bytes(int batch, int vocab) {
    return (size_t)batch * masked_topk_segments(vocab) * kTopkMax * sizeof(unsigned long long);
}

hipError_t launch_masked_topk(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                              int k, unsigned long long *workspace, int32_t *out_ids, uint16_t *out_vals,
                              hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    if (!masked_topk_fits(vocab, k)) return hipErrorInvalidValue;
    const int n_words = (vocab + 31) / 32, n_seg = masked_topk_segments(vocab);
    const int vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    hipLaunchKernelGGL(masked_topk_kernel, dim3(batch, n_seg), dim3(kTopkBlock), 0, stream, logits, bitmask, vocab, row_stride,
                       n_words, vec_ok, k, workspace);
    hipLaunchKernelGGL(masked_topk_finish_kernel, dim3(batch), dim3(64), 0, stream, workspace, n_seg * k, k, logits, row_stride,
                       out_ids, out_vals);
    return hipGetLastError();
}

}  // namespace pre3
