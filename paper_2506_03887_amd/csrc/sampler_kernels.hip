// gfx950 kernels that sample behind the mask: the greedy choice and the k best among the allowed
// tokens.  Both read the [batch, vocab] bf16 logits once and write nothing back.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "argmax.hpp"
#include "launch.hpp"
#include "stream_access.hpp"

namespace pre3 {

namespace {

// ------------------------------------------------------------------- masked argmax

constexpr int kArgUnroll = 4;

// Greedy choice among the allowed tokens without writing the masked logits back: a row's logits
// are read once (groups of 8 whose mask byte is zero are not read at all).  blockIdx.x = row,
// blockIdx.y = segment of the row.  The stream is bound by instruction issue as much as by HBM, so
// the inner loop does as little as it can per token: the two bf16 patterns of a register become
// two signed 16-bit order keys with packed arithmetic (masked halves get the lowest key; the mask
// byte of a group expands to its four AND masks through a 4 KB table in LDS), packed maxima fold a
// group of 8 into its largest key, and only when that beats the lane's best so far (strictly: the
// first of equal values stays) the lane keeps the key, the group's index, registers and mask byte.
// At the end a lane finds its winner's position inside the kept group; lanes, waves and segments
// are combined through argmax_word.  Two cases the keys cannot decide are left to
// argmax_segment_by_compare, for the whole segment: a positive NaN pattern has a key above +inf's
// (the block's best key shows it), and -0 and +0 have different keys but are equal values (the
// block's best value is zero).  With one segment per row the block writes out[b] itself; otherwise
// it stores its word in partial[b][segment] and masked_argmax_finish_kernel combines the segments.
// (Combining them inside this kernel with device-scope atomics and a last-arrival counter was
// measured: rows that finish early then cost tens of microseconds per launch.)  The mask bytes of
// the next pass are fetched while the logits of the current one are in flight.
__global__ __launch_bounds__(kArgBlock) void masked_argmax_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int groups_per_seg, int vec_ok, unsigned long long *__restrict__ partial, int32_t *__restrict__ out) {
    __shared__ unsigned long long s_part[kArgBlock / 64 + 1];
    __shared__ uint2 s_expand[16];                      // half a mask byte -> AND masks of two of the group's registers
    const int b = blockIdx.x, seg = blockIdx.y, n_seg = gridDim.y, tid = threadIdx.x;
    const int groups = (vocab + 7) >> 3;
    const int g_lo = seg * groups_per_seg, g_hi = min(groups, g_lo + groups_per_seg);
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    mask_nibble_table_init(s_expand, tid);
    int best = kOrderNegInf - 1, best_g = -1;           // only a valid value (or a positive NaN pattern) beats the start
    uint4 best_x = make_uint4(0, 0, 0, 0);
    uint32_t best_m = 0u;
    uint32_t m[kArgUnroll], m_next[kArgUnroll];
#pragma unroll
    for (int u = 0; u < kArgUnroll; ++u) {
        const int g = g_lo + tid + u * kArgBlock;
        m[u] = g < g_hi ? mrow[g] : 0u;
    }
    __syncthreads();                                    // s_expand
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
            uint32_t mu = m[u];
            if (mu == 0u) continue;
            const int g = g0 + u * kArgBlock, t0 = g * 8;
            if (!(vec_ok && t0 + 8 <= vocab)) {        // ragged tail or unaligned rows: one logit at a time
                uint32_t x[4] = {0u, 0u, 0u, 0u};
                if (t0 + 8 > vocab) mu &= (1u << (vocab - t0)) - 1u;
                for (int k = 0; k < 8 && t0 + k < vocab; ++k) x[k >> 1] |= (uint32_t)lrow[t0 + k] << (16 * (k & 1));
                v[u] = make_uint4(x[0], x[1], x[2], x[3]);
                if (mu == 0u) continue;
            }
            const uint4 allow = expand_mask_byte(s_expand, mu);
            const uint32_t k01 = packed_max_s16(bf16_order_pair(v[u].x, allow.x), bf16_order_pair(v[u].y, allow.y));
            const uint32_t k23 = packed_max_s16(bf16_order_pair(v[u].z, allow.z), bf16_order_pair(v[u].w, allow.w));
            const uint32_t k = packed_max_s16(k01, k23);
            const int group_best = max((int)(int16_t)(k & 0xFFFFu), (int)k >> 16);
            if (group_best > best) {
                best = group_best;
                best_g = g;
                best_x = v[u];
                best_m = mu;
            }
        }
#pragma unroll
        for (int u = 0; u < kArgUnroll; ++u) m[u] = m_next[u];
    }
    unsigned long long mine = 0ull;
    if (best_g >= 0) {
        const uint32_t x[4] = {best_x.x, best_x.y, best_x.z, best_x.w};
        int first = 0;
#pragma unroll
        for (int k = 7; k >= 0; --k) {                  // descending: the smallest k is assigned last
            const uint32_t h = (k & 1) ? (x[k >> 1] >> 16) : (x[k >> 1] & 0xFFFFu);
            if (((best_m >> k) & 1u) && bf16_order(h) == best) first = k;
        }
        mine = argmax_word(best, best_g * 8 + first);
    }
    mine = argmax_block_max(mine, s_part, tid);
    const int order = (int)(uint32_t)(mine >> 32) - 32768;
    if (mine != 0ull && (order > kOrderPosInf || order == 0))
        mine = argmax_block_max(argmax_segment_by_compare(lrow, mrow, g_lo, g_hi, vocab, tid), s_part, tid);
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

// Order-preserving 16-bit key of a non-NaN bf16 pattern: a negative value's pattern is negated
// (two's complement), a non-negative one gets its top bit set (so -0 and +0 share a key), and 0x7F
// is subtracted with saturation.  Valid values map to 0x0001 (-inf) .. 0xFF01 (+inf); negative NaN
// patterns map to 0 (no candidate), positive NaN patterns to keys above 0xFF01.
constexpr uint32_t kTopkKeyMax = 0xFF01u;
__device__ __forceinline__ uint32_t bf16_key(uint32_t h) {
    const uint32_t folded = (h & 0x8000u) ? ((0u - h) & 0xFFFFu) : (h | 0x8000u);
    return folded > 0x7Fu ? folded - 0x7Fu : 0u;
}

// The same for two patterns in one register, with packed 16-bit arithmetic.
typedef unsigned short PackedU16 __attribute__((ext_vector_type(2)));
typedef short PackedI16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t packed_sub_sat_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(PackedU16, a), __builtin_bit_cast(PackedU16, b)));
}
__device__ __forceinline__ uint32_t bf16_key_pair(uint32_t x) {
    const PackedU16 h = __builtin_bit_cast(PackedU16, x);
    const uint32_t negative = __builtin_bit_cast(uint32_t, __builtin_bit_cast(PackedI16, x) >> 15);   // 0xFFFF per negative half
    const uint32_t neg = __builtin_bit_cast(uint32_t, (PackedU16)(PackedU16{0, 0} - h));
    const uint32_t pos = x | 0x80008000u;
    return packed_sub_sat_u16((neg & negative) | (pos & ~negative), 0x007F007Fu);
}
__device__ __forceinline__ uint32_t packed_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(PackedU16, a), __builtin_bit_cast(PackedU16, b)));
}
__device__ __forceinline__ uint32_t packed_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(PackedU16, a), __builtin_bit_cast(PackedU16, b)));
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

// The kk-th largest of the S distinct non-zero words of an LDS list (1 <= kk <= S), found bit by bit
// from the top by one wave; lane l looks at the words l, l + 64, ... (kept in registers when there
// are at most 512 of them).  Words >= the result are the kk largest.
__device__ __forceinline__ unsigned long long wave_kth_largest(const unsigned long long *list, int S, int kk, int lane) {
    if (kk >= S) return 1ull;
    constexpr int kRegs = 8;
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

// The k best candidates of one segment of one row (blockIdx.x = row, blockIdx.y = segment: a run of
// chunks_per_seg chunks of kTopkChunk tokens, taken in order).  Of each chunk every thread keeps the
// 16-bit keys of its 32 tokens in registers, two per register (0 = masked, NaN or beyond the
// vocabulary), so the logits are read once; the loads of the next chunk are in flight meanwhile.
//   From the per-thread maxima of the first chunk that holds candidates the block derives a lower
//   bound M of the k-th largest key (at least k threads hold a key >= M), so only keys >= M can be
//   among the k best: of every chunk a little more than k.  From then on the waves do not meet again
//   until the end: each appends its keys >= M to a list of its own (kTopkRegion words of LDS).  A wave
//   whose list runs full cuts it to its k best and from then on uses the key of its k-th as its bound
//   (a wave's k-th best is a lower bound of the block's); after a chunk in which that happened the
//   bound rises by one more, because later chunks hold larger ids, which lose every tie.
//   At the end every thread ranks the words of its wave's list that fall to it (rank = number of
//   larger words in all lists) and the k best write themselves in order.
// The k words are written to out[(row * n_seg + segment) * k ..], best first, 0-padded; with one
// segment per row the kernel writes the row's ids and bf16 patterns itself (out_ids, out_vals).
constexpr int kTopkBlock = 512;                    // threads per block; kTopkBlockWide when a row has a compute unit to itself
constexpr int kTopkBlockWide = 1024;
constexpr int kTopkPerThread = 32;
constexpr int kTopkChunk = kTopkPerThread * kTopkBlock;   // tokens per chunk (twice as many for the wide block)
constexpr int kTopkRegion = 256;

// Eight logits from t0 on, one 2-byte load each (rows that are not 16-byte aligned, and the group
// that straddles the end of the vocabulary); tokens beyond the vocabulary read as NaN.  A loop that
// is not unrolled: the path is rare and must not cost the kernel registers.
__device__ __forceinline__ uint4 topk_load_group_unaligned(const uint16_t *__restrict__ lrow, int t0, int vocab) {
    unsigned long long lo = 0x7FC07FC07FC07FC0ull, hi = lo;
#pragma unroll 1
    for (int j = 0; j < 8; ++j) {
        if (t0 + j >= vocab) break;
        const unsigned long long h = lrow[t0 + j];
        const int sh = (j & 3) * 16;
        if (j < 4) lo = (lo & ~(0xFFFFull << sh)) | (h << sh);
        else hi = (hi & ~(0xFFFFull << sh)) | (h << sh);
    }
    return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

// Block barrier for data exchanged through LDS: waits for the wave's own LDS operations only, so
// that global loads issued ahead stay in flight across it (__syncthreads would wait for them).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Cuts a wave's list (n > k words) to its k best, moved to the front; returns the key of the k-th.
__device__ __noinline__ uint32_t topk_cut_list(unsigned long long *list, int n, int k, int lane) {
    const unsigned long long thr = wave_kth_largest(list, n, k, lane);
    int base = 0;
    for (int r0 = 0; r0 < n; r0 += 64) {                      // all lanes read, then write: the ranges may overlap
        const unsigned long long w = r0 + lane < n ? list[r0 + lane] : 0ull;
        const bool take = w >= thr;
        const unsigned long long mm = __ballot(take);
        __builtin_amdgcn_wave_barrier();
        if (take) list[base + __popcll(mm & ((1ull << lane) - 1ull))] = w;
        base += __popcll(mm);
    }
    __builtin_amdgcn_wave_barrier();
    return (uint32_t)(thr >> kTopkIdBits);
}

template <int kBlock>
__device__ __forceinline__ void masked_topk_chunked(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int vec_ok, int k, int chunks_per_seg, unsigned long long *__restrict__ out,
    int32_t *__restrict__ out_ids, uint16_t *__restrict__ out_vals, int b, int seg, int n_seg) {
    constexpr int kWaves = kBlock / 64, kChunk = kTopkPerThread * kBlock;
    __shared__ unsigned long long s_list[kWaves * kTopkRegion];
    __shared__ int s_nz[kWaves];
    __shared__ uint32_t s_wbound[kWaves];
    __shared__ int s_n[kWaves];
    __shared__ uint2 s_expand[16];                            // half a mask byte -> AND masks of two of the group's registers
    __shared__ unsigned long long s_short[kBlock];        // the few words left at the end, one per thread
    __shared__ int s_total;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    mask_nibble_table_init(s_expand, tid);
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    const int n_mask_bytes = n_words * 4;
    unsigned long long *dst = out + ((size_t)b * n_seg + seg) * (size_t)k;
    // with one segment per row (out_ids given) the ranked words are the row's result and go out as ids and patterns
    auto emit = [&](int rank, unsigned long long word) {
        if (out_ids == nullptr) {
            dst[rank] = word;
        } else if (word != 0ull) {
            const uint32_t id = kTopkIdMask - ((uint32_t)word & kTopkIdMask);
            out_ids[(size_t)b * k + rank] = (int32_t)id;
            if (out_vals) out_vals[(size_t)b * k + rank] = lrow[id];
        } else {
            out_ids[(size_t)b * k + rank] = -1;
            if (out_vals) out_vals[(size_t)b * k + rank] = 0xFF80u;
        }
    };
    const int n_chunks = (vocab + kChunk - 1) / kChunk;
    const int c_begin = seg * chunks_per_seg;
    const int c_end = c_begin + chunks_per_seg < n_chunks ? c_begin + chunks_per_seg : n_chunks;
    // element e of a thread (0 .. 31) is token  chunk * kChunk + rel(e); its key is half (e & 1) of kp[e >> 1]
    auto rel = [&](int e) { return (tid + (e >> 3) * kBlock) * 8 + (e & 7); };
    unsigned long long *mylist = s_list + wave * kTopkRegion;
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    int n_mine = 0;                                           // length of the wave's list
    uint32_t block_bound = 0u;                                // 0: no candidate seen yet; 1: every candidate (same in all waves)
    uint32_t wave_bound = 0u;                                 // what the wave's own list has proved since
    // The loads run ahead of the selection: while a chunk is worked on, the logits of the next one and
    // the mask bytes of the one after it are in flight (a group's logits are only read when its mask
    // byte is not 0, so the mask has to arrive one stage earlier).
    auto load_mask = [&](int chunk, uint32_t (&m)[kTopkPerThread / 8]) {
#pragma unroll
        for (int g = 0; g < kTopkPerThread / 8; ++g) {
            const int t0 = chunk * kChunk + (tid + g * kBlock) * 8;
            m[g] = (chunk < c_end && t0 < vocab && (t0 >> 3) < n_mask_bytes) ? mrow[t0 >> 3] : 0u;
        }
    };
    auto load_logits = [&](int chunk, const uint32_t (&m)[kTopkPerThread / 8], uint4 (&v)[kTopkPerThread / 8]) {
        const uint16_t *p = lrow + (size_t)chunk * kChunk + (size_t)tid * 8;
        if (vec_ok && (chunk + 1) * kChunk <= vocab) {       // a whole chunk of an aligned row
#pragma unroll
            for (int g = 0; g < kTopkPerThread / 8; ++g) {
                v[g] = make_uint4(0u, 0u, 0u, 0u);               // its mask zeroes the keys anyway
                if (m[g] != 0u) v[g] = stream_load(p + g * kBlock * 8);
            }
            return;
        }
#pragma unroll
        for (int g = 0; g < kTopkPerThread / 8; ++g) {
            const int t0 = chunk * kChunk + (tid + g * kBlock) * 8;
            v[g] = make_uint4(0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u);   // NaN: no candidate
            if (m[g] != 0u) {
                if (vec_ok && t0 + 8 <= vocab) v[g] = stream_load(lrow + (size_t)t0);
                else v[g] = topk_load_group_unaligned(lrow, t0, vocab);
            }
        }
    };
    uint32_t m[kTopkPerThread / 8], m_ahead[kTopkPerThread / 8];
    uint4 v[kTopkPerThread / 8];
    load_mask(c_begin, m);
    load_mask(c_begin + 1, m_ahead);
    load_logits(c_begin, m, v);
    lds_barrier();                                            // s_expand
    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        uint32_t kp[kTopkPerThread / 2];
        // two keys per register with packed 16-bit arithmetic; the mask byte of a group expands to the
        // four AND masks of its registers through a table in LDS
        uint32_t best2 = 0u;
#pragma unroll
        for (int g = 0; g < kTopkPerThread / 8; ++g) {
            const uint4 allow = expand_mask_byte(s_expand, m[g]);
            const uint32_t x[4] = {v[g].x, v[g].y, v[g].z, v[g].w}, a[4] = {allow.x, allow.y, allow.z, allow.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                kp[g * 4 + j] = bf16_key_pair(x[j]) & a[j];
                best2 = packed_max_u16(best2, kp[g * 4 + j]);
            }
        }
        if ((best2 & 0xFFFFu) > kTopkKeyMax || (best2 >> 16) > kTopkKeyMax) {      // an allowed NaN: one half at a time
            best2 = 0u;
#pragma unroll
            for (int g = 0; g < kTopkPerThread / 8; ++g) {
                const uint32_t x[4] = {v[g].x, v[g].y, v[g].z, v[g].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t lo = x[j] & 0xFFFFu, hi = x[j] >> 16;
                    const bool ok_lo = ((m[g] >> (2 * j)) & 1u) && (lo & 0x7FFFu) <= 0x7F80u;
                    const bool ok_hi = ((m[g] >> (2 * j + 1)) & 1u) && (hi & 0x7FFFu) <= 0x7F80u;
                    kp[g * 4 + j] = (ok_lo ? bf16_key(lo) : 0u) | ((ok_hi ? bf16_key(hi) : 0u) << 16);
                    best2 = packed_max_u16(best2, kp[g * 4 + j]);
                }
            }
        }
        const uint32_t best = (best2 & 0xFFFFu) > (best2 >> 16) ? (best2 & 0xFFFFu) : (best2 >> 16);
#pragma unroll
        for (int g = 0; g < kTopkPerThread / 8; ++g) m[g] = m_ahead[g];
        if (chunk + 1 < c_end) load_logits(chunk + 1, m, v);
        load_mask(chunk + 2, m_ahead);
        if (block_bound <= 1u) {
            // A lower bound of the k-th largest key from the threads' maxima: wave w takes the q_w-th
            // largest of its 64 maxima, q_w = min(j, threads of w that hold a candidate), with the
            // smallest j for which the q_w add up to k; the smallest of these is reached by at least k keys.
            const int nz_wave = __popcll(__ballot(best != 0u));
            if (lane == 0) s_nz[wave] = nz_wave;
            lds_barrier();
            int quota = 0, holders = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) holders += s_nz[w];
            if (holders >= k) {
                for (quota = 1; quota < 64; ++quota) {
                    int sum = 0;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) sum += s_nz[w] < quota ? s_nz[w] : quota;
                    if (sum >= k) break;
                }
            }
            uint32_t mine = 0x10000u;                         // no candidate in this wave
            if (nz_wave > 0) {
                mine = 1u;                                    // fewer than k holders in the block: every candidate
                if (quota > 0) {
                    int reached;
                    mine = wave_key_threshold<1>([&](int) { return best; }, nz_wave, nz_wave < quota ? nz_wave : quota, &reached);
                }
            }
            if (lane == 0) s_wbound[wave] = mine;
            lds_barrier();
            uint32_t cb = 0x10000u;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) cb = s_wbound[w] < cb ? s_wbound[w] : cb;
            if (cb != 0x10000u && cb > block_bound) block_bound = cb;
        }
        uint32_t bound = block_bound > wave_bound ? block_bound : wave_bound;
        if (bound == 0u || !__any(best >= bound)) continue;
        // The keys that reach the bound (few): every thread counts its own -- a saturating packed
        // subtraction leaves a non-zero half where a key reaches it -- and notes in which register.
        const uint32_t below = (bound - 1u) * 0x10001u;
        uint32_t count2 = 0u, where2 = 0u;                    // per half: how many reach it, and the sum of their register numbers
#pragma unroll
        for (int i = 0; i < kTopkPerThread / 2; ++i) {
            const uint32_t one = packed_min_u16(packed_sub_sat_u16(kp[i], below), 0x00010001u);
            count2 += one;
            where2 += one * (uint32_t)i;
        }
        const int mine = (int)((count2 & 0xFFFFu) + (count2 >> 16));      // 0 .. 32
        const unsigned long long holders = __ballot(mine > 0);
        int before = __popcll(holders & lanes_below), total = __popcll(holders);   // right when no thread holds several
        if (__ballot(mine > 1) != 0ull) {
            before = 0;
            total = 0;
#pragma unroll
            for (int bit = 0; bit < 6; ++bit) {
                const unsigned long long has = __ballot((mine >> bit) & 1);
                before += __popcll(has & lanes_below) << bit;
                total += __popcll(has) << bit;
            }
        }
        if (n_mine + total <= kTopkRegion) {
            int slot = n_mine + before;
            if (mine == 1) {
                // the usual case: the key is the thread's maximum, and the sum is its register
                const int e = (count2 & 0xFFFFu) ? 2 * (int)(where2 & 0xFFFFu) : 2 * (int)(where2 >> 16) + 1;
                mylist[slot] = topk_word(best, (uint32_t)(chunk * kChunk + rel(e)));
            } else if (mine > 1) {
#pragma unroll
                for (int i = 0; i < kTopkPerThread / 2; ++i) {
                    const uint32_t reach = packed_sub_sat_u16(kp[i], below);
                    if (reach & 0xFFFFu) mylist[slot++] = topk_word(kp[i] & 0xFFFFu, (uint32_t)(chunk * kChunk + rel(2 * i)));
                    if (reach >> 16) mylist[slot++] = topk_word(kp[i] >> 16, (uint32_t)(chunk * kChunk + rel(2 * i + 1)));
                }
            }
            n_mine += total;
            continue;
        }
        // the list may run full: element by element, with room made when it is needed
        bool cut = false;
        uint32_t last_kth = 0u;                               // key of the k-th word after the latest cut
#pragma unroll
        for (int e = 0; e < kTopkPerThread; ++e) {
            const uint32_t key = (kp[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
            bool take = key >= bound;
            unsigned long long mm = __ballot(take);
            if (mm == 0ull) continue;
            if (n_mine + __popcll(mm) > kTopkRegion) {        // n_mine > k here: the cut leaves k words
                last_kth = topk_cut_list(mylist, n_mine, k, lane);
                n_mine = k;
                wave_bound = last_kth > wave_bound ? last_kth : wave_bound;
                bound = block_bound > wave_bound ? block_bound : wave_bound;
                cut = true;
                take = key >= bound;
                mm = __ballot(take);
            }
            if (take) mylist[n_mine + __popcll(mm & lanes_below)] = topk_word(key, (uint32_t)(chunk * kChunk + rel(e)));
            n_mine += __popcll(mm);
        }
        if (cut) {                                            // from the next chunk on ties with the k-th can be left out
            if (n_mine > k) {
                last_kth = topk_cut_list(mylist, n_mine, k, lane);
                n_mine = k;
            }
            wave_bound = last_kth + 1u > wave_bound ? last_kth + 1u : wave_bound;
        }
    }
    // The lists are complete.  If they hold many words, the same bound as above -- now from the
    // maxima of the listed words each thread holds -- leaves little more than k of them, and every
    // wave drops the rest of its list.  Then every thread ranks the words of its wave's list that fall
    // to it against all lists (rank = number of larger words) and the k best write themselves in order.
    if (lane == 0) s_n[wave] = n_mine;
    lds_barrier();
    int S = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) S += s_n[w];
    if (tid >= S && tid < k) emit(tid, 0ull);
    unsigned long long w[kTopkRegion / 64];
#pragma unroll
    for (int r = 0; r < kTopkRegion / 64; ++r) w[r] = r * 64 + lane < n_mine ? mylist[r * 64 + lane] : 0ull;
    uint32_t cb = 1u;                                         // every listed word
    if (S > 2 * k + 32) {                                     // the same in every thread
        unsigned long long top = 0ull;
#pragma unroll
        for (int r = 0; r < kTopkRegion / 64; ++r) top = w[r] > top ? w[r] : top;
        const uint32_t best = (uint32_t)(top >> kTopkIdBits);
        const int nz_wave = __popcll(__ballot(best != 0u));
        if (lane == 0) s_nz[wave] = nz_wave;
        lds_barrier();
        int quota = 0, holders = 0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) holders += s_nz[ww];
        if (holders >= k) {
            for (quota = 1; quota < 64; ++quota) {
                int sum = 0;
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) sum += s_nz[ww] < quota ? s_nz[ww] : quota;
                if (sum >= k) break;
            }
        }
        uint32_t mine = 0x10000u;
        if (nz_wave > 0) {
            mine = 1u;
            if (quota > 0) {
                int reached;
                mine = wave_key_threshold<1>([&](int) { return best; }, nz_wave, nz_wave < quota ? nz_wave : quota, &reached);
            }
        }
        if (lane == 0) s_wbound[wave] = mine;
        lds_barrier();
        cb = 0x10000u;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) cb = s_wbound[ww] < cb ? s_wbound[ww] : cb;
    }
    {
        // the words that reach it: counted, and if there are few, gathered in one short list, one word per thread
        bool keep[kTopkRegion / 64];
        int kept = 0;
#pragma unroll
        for (int r = 0; r < kTopkRegion / 64; ++r) {
            keep[r] = w[r] != 0ull && (uint32_t)(w[r] >> kTopkIdBits) >= cb;
            kept += __popcll(__ballot(keep[r]));
        }
        if (tid == 0) s_total = 0;
        if (lane == 0) s_nz[wave] = kept;                     // (every wave has read the old values before the last barrier)
        lds_barrier();
        int S2 = 0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) S2 += s_nz[ww];
        if (S2 <= kBlock) {
            int at = 0;
            if (lane == 0 && kept > 0) at = atomicAdd(&s_total, kept);
            at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
            for (int r = 0; r < kTopkRegion / 64; ++r) {
                const unsigned long long mm = __ballot(keep[r]);
                if (keep[r]) s_short[at + __popcll(mm & lanes_below)] = w[r];
                at += __popcll(mm);
            }
            lds_barrier();
            if (wave * 64 >= S2) return;
            const unsigned long long mine = tid < S2 ? s_short[tid] : ~0ull;
            int rank = 0;
#pragma unroll 8
            for (int j = 0; j < S2; ++j) rank += s_short[j] > mine ? 1 : 0;
            if (tid < S2 && rank < k) emit(rank, mine);
            return;
        }
        // many ties with the bound: the words stay where they are, every wave drops the others from its list
        kept = 0;
#pragma unroll
        for (int r = 0; r < kTopkRegion / 64; ++r) {
            const unsigned long long mm = __ballot(keep[r]);
            if (keep[r]) mylist[kept + __popcll(mm & lanes_below)] = w[r];   // every word of the list is in a register by now
            kept += __popcll(mm);
        }
        n_mine = kept;
        if (lane == 0) s_n[wave] = n_mine;
        lds_barrier();
#pragma unroll
        for (int r = 0; r < kTopkRegion / 64; ++r) w[r] = r * 64 + lane < n_mine ? mylist[r * 64 + lane] : 0ull;
    }
    if (n_mine == 0) return;
    int rank[kTopkRegion / 64];
#pragma unroll
    for (int r = 0; r < kTopkRegion / 64; ++r) rank[r] = 0;
    for (int ww = 0; ww < kWaves; ++ww) {
        const unsigned long long *other = s_list + ww * kTopkRegion;
        const int n_other = s_n[ww];
        if (n_mine <= 64) {
#pragma unroll 8
            for (int j = 0; j < n_other; ++j) rank[0] += other[j] > w[0] ? 1 : 0;
        } else {
#pragma unroll 2
            for (int j = 0; j < n_other; ++j) {
                const unsigned long long o = other[j];
#pragma unroll
                for (int r = 0; r < kTopkRegion / 64; ++r) rank[r] += o > w[r] ? 1 : 0;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kTopkRegion / 64; ++r)
        if (r * 64 + lane < n_mine && rank[r] < k) emit(rank[r], w[r]);
}

template <int kBlock>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4))) void masked_topk_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int vec_ok, int k, int chunks_per_seg, unsigned long long *__restrict__ out,
    int32_t *__restrict__ out_ids, uint16_t *__restrict__ out_vals) {
    masked_topk_chunked<kBlock>(logits, bitmask, vocab, row_stride, n_words, vec_ok, k, chunks_per_seg, out, out_ids, out_vals,
                                blockIdx.x, blockIdx.y, gridDim.y);
}

// The stored bf16 pattern behind a key of bf16_key, or -1 for the key of zero, which -0 and +0 share.
__device__ __forceinline__ int bf16_pattern_of_key(uint32_t key) {
    const uint32_t folded = key + 0x7Fu;
    if (folded == 0x8000u) return -1;
    return (folded & 0x8000u) ? (int)(folded & 0x7FFFu) : (int)((0x10000u - folded) & 0xFFFFu);
}

// The k best of a whole row by one block of 1,024 threads that keeps the row in registers: rows of at
// most kTopkRowGroups * 1,024 groups of 8 tokens (131,072 tokens), 16-byte aligned.  Every thread
// issues the loads of its mask bytes and of its up to 16 groups of logits at once (a group is read
// whatever its mask byte says: no load waits for another one) and turns them into 64 registers of
// packed 16-bit keys (0 = masked, NaN or beyond the vocabulary), with the packed maximum of every
// group and the thread's maximum.  What follows the stream is short:
//   (1) a lower bound M of the k-th largest key: every wave takes the q-th largest of its 64 thread
//       maxima (q = ceil(k / 16); a wave with fewer holders its smallest); if these quotas add up to
//       k, at least k keys reach the smallest of the waves' values (one barrier);
//   (2) the few threads whose maximum reaches M look through the groups whose maximum does and
//       append those keys, as words, to one list in LDS;
//   (3) the list (little more than k words) is ranked by all threads together -- a word's rank is the
//       number of larger words, counted in slices by several threads and added up in LDS -- and the
//       k best write their id and pattern (rebuilt from the key, read back only for a zero) in order.
// A list that would pass kTopkRowList words (thousands of ties with the bound, or quotas that do not
// add up to k on a dense row) is given up: the block then takes the row chunk by chunk with
// masked_topk_chunked, which has no such limit.
// (Measured and dropped: taking the bound from half of the row while the other half is still in
// flight, with the second half filtered as it arrives -- the waves of a block finish their halves
// microseconds apart, so the barrier gains nothing, and the looser bound doubles the list.)
constexpr int kTopkRowGroups = 16;
constexpr int kTopkRowList = 512;
__global__ __launch_bounds__(kTopkBlockWide) __attribute__((amdgpu_waves_per_eu(4))) void masked_topk_row_kernel(
    const uint16_t *__restrict__ logits, const uint32_t *__restrict__ bitmask, int vocab, int64_t row_stride,
    int n_words, int k, unsigned long long *__restrict__ workspace, int32_t *__restrict__ out_ids,
    uint16_t *__restrict__ out_vals) {
    constexpr int kBlock = kTopkBlockWide, kWaves = kBlock / 64, kG = kTopkRowGroups;
    __shared__ uint2 s_expand[16];                            // half a mask byte -> AND masks of two of the group's registers
    __shared__ unsigned long long s_cand[kTopkRowList];
    __shared__ int s_rank[kTopkRowList];
    __shared__ int s_nz[kWaves];
    __shared__ uint32_t s_wbound[kWaves];
    __shared__ int s_count;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    mask_nibble_table_init(s_expand, tid);
    if (tid < kTopkRowList) s_rank[tid] = 0;                  // (the list has fewer entries than the block has threads)
    if (tid == 0) s_count = 0;
    const uint8_t *mrow = reinterpret_cast<const uint8_t *>(bitmask + (size_t)b * n_words);
    const uint16_t *lrow = logits + (size_t)b * row_stride;
    const int groups = (vocab + 7) >> 3, n_mask_bytes = n_words * 4;
    uint32_t m[kG];
    uint4 v[kG];
#pragma unroll
    for (int u = 0; u < kG; ++u) {
        const int g = tid + u * kBlock;
        m[u] = (g < groups && g < n_mask_bytes) ? mrow[g] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kG; ++u) {
        const int g = tid + u * kBlock;
        v[u] = make_uint4(0u, 0u, 0u, 0u);
        if (g * 8 + 8 <= vocab) v[u] = stream_load(lrow + (size_t)g * 8);
        else if (g < groups) v[u] = topk_load_group_unaligned(lrow, g * 8, vocab);   // the group the vocabulary ends in
    }
    lds_barrier();                                            // s_expand, s_rank, s_count
    uint32_t kp[kG * 4], gmax2[kG];
    uint32_t best2 = 0u;
#pragma unroll
    for (int u = 0; u < kG; ++u) {
        const uint4 allow = expand_mask_byte(s_expand, m[u]);
        const uint32_t x[4] = {v[u].x, v[u].y, v[u].z, v[u].w}, a[4] = {allow.x, allow.y, allow.z, allow.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) kp[u * 4 + j] = bf16_key_pair(x[j]) & a[j];
        gmax2[u] = packed_max_u16(packed_max_u16(kp[u * 4], kp[u * 4 + 1]), packed_max_u16(kp[u * 4 + 2], kp[u * 4 + 3]));
        best2 = packed_max_u16(best2, gmax2[u]);
    }
    if ((best2 & 0xFFFFu) > kTopkKeyMax || (best2 >> 16) > kTopkKeyMax) {          // an allowed NaN: its key goes
        best2 = 0u;
#pragma unroll
        for (int u = 0; u < kG; ++u) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = kp[u * 4 + j] & 0xFFFFu, hi = kp[u * 4 + j] >> 16;
                kp[u * 4 + j] = (lo > kTopkKeyMax ? 0u : lo) | ((hi > kTopkKeyMax ? 0u : hi) << 16);
            }
            gmax2[u] = packed_max_u16(packed_max_u16(kp[u * 4], kp[u * 4 + 1]), packed_max_u16(kp[u * 4 + 2], kp[u * 4 + 3]));
            best2 = packed_max_u16(best2, gmax2[u]);
        }
    }
    const uint32_t best = (best2 & 0xFFFFu) > (best2 >> 16) ? (best2 & 0xFFFFu) : (best2 >> 16);
    // (1) the bound
    const int quota = (k + kWaves - 1) / kWaves;
    const int nz_wave = __popcll(__ballot(best != 0u));
    uint32_t wave_m = 0x10000u;                                // no candidate in this wave
    if (nz_wave > 0) {
        int reached;
        wave_m = wave_key_threshold<1>([&](int) { return best; }, nz_wave, nz_wave < quota ? nz_wave : quota, &reached);
    }
    if (lane == 0) { s_nz[wave] = nz_wave; s_wbound[wave] = wave_m; }
    lds_barrier();
    uint32_t bound = 0x10000u;
    int reach_bound = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        bound = s_wbound[w] < bound ? s_wbound[w] : bound;
        reach_bound += s_nz[w] < quota ? s_nz[w] : quota;
    }
    auto emit = [&](int rank, unsigned long long word) {
        if (word != 0ull) {
            const uint32_t id = kTopkIdMask - ((uint32_t)word & kTopkIdMask);
            out_ids[(size_t)b * k + rank] = (int32_t)id;
            if (out_vals) {
                const int pattern = bf16_pattern_of_key((uint32_t)(word >> kTopkIdBits));
                out_vals[(size_t)b * k + rank] = pattern >= 0 ? (uint16_t)pattern : lrow[id];
            }
        } else {
            out_ids[(size_t)b * k + rank] = -1;
            if (out_vals) out_vals[(size_t)b * k + rank] = 0xFF80u;
        }
    };
    if (bound == 0x10000u) {                                  // nothing is allowed (or only NaN)
        if (tid < k) emit(tid, 0ull);
        return;
    }
    if (reach_bound < k) bound = 1u;                          // the quotas do not add up: every candidate
    // (2) the list
    if (__any(best >= bound)) {
        const uint32_t below = (bound - 1u) * 0x10001u;
#pragma unroll
        for (int u = 0; u < kG; ++u) {
            if (packed_sub_sat_u16(gmax2[u], below) == 0u) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t reach = packed_sub_sat_u16(kp[u * 4 + j], below);
                const uint32_t t0 = (uint32_t)(tid + u * kBlock) * 8u + (uint32_t)j * 2u;
                if (reach & 0xFFFFu) {
                    const int slot = atomicAdd(&s_count, 1);
                    if (slot < kTopkRowList) s_cand[slot] = topk_word(kp[u * 4 + j] & 0xFFFFu, t0);
                }
                if (reach >> 16) {
                    const int slot = atomicAdd(&s_count, 1);
                    if (slot < kTopkRowList) s_cand[slot] = topk_word(kp[u * 4 + j] >> 16, t0 + 1u);
                }
            }
        }
    }
    __syncthreads();
    const int n = s_count;
    if (n > kTopkRowList) {                                   // same in every thread
        masked_topk_chunked<kBlock>(logits, bitmask, vocab, row_stride, n_words, 1, k,
                                    (vocab + kTopkPerThread * kBlock - 1) / (kTopkPerThread * kBlock), workspace, out_ids, out_vals,
                                    b, 0, 1);
        return;
    }
    // (3) ranks: thread (slice, word) counts the larger words of its slice of the list
    if (tid >= n && tid < k) emit(tid, 0ull);
    if (n == 0) return;
    const int slices = kBlock / n > 0 ? kBlock / n : 1, per = (n + slices - 1) / slices;
    const int word_at = tid % n, slice = tid / n;
    if (slice < slices) {
        const unsigned long long mine = s_cand[word_at];
        const int j_end = (slice + 1) * per < n ? (slice + 1) * per : n;
        int larger = 0;
#pragma unroll 4
        for (int j = slice * per; j < j_end; ++j) larger += s_cand[j] > mine ? 1 : 0;
        if (larger) atomicAdd(&s_rank[word_at], larger);
    }
    __syncthreads();
    if (tid < n && s_rank[tid] < k) emit(s_rank[tid], s_cand[tid]);
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

static int masked_topk_chunks(int vocab, int chunk = kTopkChunk) { return (vocab + chunk - 1) / chunk; }

// Chunks per block: the whole row once there is a row per compute unit (the block then writes the
// result itself and no second kernel runs); below that as many as still leave two blocks per compute
// unit, so that small batches are spread over the chip.
static int masked_topk_chunks_per_segment(int batch, int vocab, int n_compute_units) {
    const int n_chunks = masked_topk_chunks(vocab);
    if (batch >= n_compute_units) return n_chunks;
    int per = 1;
    while (per < n_chunks && (int64_t)batch * ((n_chunks + 2 * per - 1) / (2 * per)) >= 2 * (int64_t)n_compute_units) per *= 2;
    return per < n_chunks ? per : n_chunks;
}

bool masked_topk_fits(int vocab, int k) {
    return k >= 1 && k <= kTopkMax && vocab >= 1 && vocab <= (1 << kTopkIdBits) &&
           masked_topk_chunks(vocab) * k <= 64 * kTopkFinishPer;
}

size_t masked_topk_workspace_bytes(int batch, int vocab) {
    return (size_t)batch * masked_topk_chunks(vocab) * kTopkMax * sizeof(unsigned long long);
}

hipError_t launch_masked_topk(const uint16_t *logits, const uint32_t *bitmask, int batch, int vocab, int64_t row_stride,
                              int k, int n_compute_units, unsigned long long *workspace, int32_t *out_ids,
                              uint16_t *out_vals, hipStream_t stream) {
    if (batch == 0) return hipSuccess;
    if (!masked_topk_fits(vocab, k)) return hipErrorInvalidValue;
    const int n_words = (vocab + 31) / 32;
    const int vec_ok = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 8 == 0);
    if (batch >= n_compute_units && vec_ok && (vocab + 7) / 8 <= kTopkRowGroups * kTopkBlockWide) {
        // a block per row that keeps the whole row in registers
        hipLaunchKernelGGL(masked_topk_row_kernel, dim3(batch), dim3(kTopkBlockWide), 0, stream, logits, bitmask, vocab,
                           row_stride, n_words, k, workspace, out_ids, out_vals);
        return hipGetLastError();
    }
    if (batch >= n_compute_units && batch < 2 * n_compute_units) {
        // a row per compute unit and no second block beside it: sixteen waves take the row
        hipLaunchKernelGGL(masked_topk_kernel<kTopkBlockWide>, dim3(batch, 1), dim3(kTopkBlockWide), 0, stream, logits, bitmask,
                           vocab, row_stride, n_words, vec_ok, k, masked_topk_chunks(vocab, kTopkPerThread * kTopkBlockWide),
                           workspace, out_ids, out_vals);
        return hipGetLastError();
    }
    const int per = masked_topk_chunks_per_segment(batch, vocab, n_compute_units);
    const int n_seg = (masked_topk_chunks(vocab) + per - 1) / per;
    if (n_seg == 1) {
        hipLaunchKernelGGL(masked_topk_kernel<kTopkBlock>, dim3(batch, 1), dim3(kTopkBlock), 0, stream, logits, bitmask, vocab,
                           row_stride, n_words, vec_ok, k, per, workspace, out_ids, out_vals);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(masked_topk_kernel<kTopkBlock>, dim3(batch, n_seg), dim3(kTopkBlock), 0, stream, logits, bitmask, vocab,
                       row_stride, n_words, vec_ok, k, per, workspace, (int32_t *)nullptr, (uint16_t *)nullptr);
    hipLaunchKernelGGL(masked_topk_finish_kernel, dim3(batch), dim3(64), 0, stream, workspace, n_seg * k, k, logits, row_stride,
                       out_ids, out_vals);
    return hipGetLastError();
}

}  // namespace pre3
