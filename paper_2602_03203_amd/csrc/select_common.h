// Device helpers of the selection kernels: order-preserving score keys, a workgroup scan and the
// most-significant-digit-first radix select over a workgroup (used by fk_select_keep,
// fk_select_keep_sampled and the Golden Eviction trace).
#ifndef FK_SELECT_COMMON_H
#define FK_SELECT_COMMON_H
#include "fk_common.h"

namespace fk {

static constexpr int kSelThreads = 1024;
static constexpr int kSelWaves = kSelThreads / kWave;

__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN: below everything
    if (u == 0x80000000u) u = 0u;                     // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves (a handful of cycles per
// step; the same scan through LDS permutes costs about a hundred per step): shifts by 1, 2, 4, 8 inside each row of 16
// lanes, then the last lane of rows 0 / 2 is added to rows 1 / 3, then lane 31 to the upper half.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);  // lanes without a source get 0
}
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t v) {
    v += dpp_u32<0x111, 0xF>(v);  // row_shr:1
    v += dpp_u32<0x112, 0xF>(v);  // row_shr:2
    v += dpp_u32<0x114, 0xF>(v);  // row_shr:4
    v += dpp_u32<0x118, 0xF>(v);  // row_shr:8
    v += dpp_u32<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_u32<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// inclusive scan of a 64-bit value over the workgroup, in thread order; returns the inclusive
// value and the workgroup total.  s_part must hold kSelWaves entries.
__device__ __forceinline__ unsigned long long block_scan_incl(unsigned long long v,
                                                              unsigned long long* s_part,
                                                              unsigned long long* total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const unsigned long long o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    __syncthreads();  // s_part free for reuse
    if (lane == kWave - 1) s_part[wave] = v;
    __syncthreads();
    unsigned long long before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const unsigned long long x = s_part[w];
        if (w < wave) before += x;
        tot += x;
    }
    *total = tot;
    return v + before;
}

// MSB-first radix select over slots [0, nslots): finds T and `want` such that the k best valid
// slots are those with key > T plus the first `want` (in slot order) with key == T.  k >= 1 and at
// least k valid slots.  key_of(i, valid) returns the slot's key and whether it takes part.
template <typename KeyFn>
__device__ __forceinline__ void radix_threshold(int nslots, uint32_t k, KeyFn key_of, uint32_t* s_hist,
                                                uint32_t* s_sel, uint32_t* T, uint32_t* want_out) {
    uint32_t prefix = 0, mask = 0, want = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = threadIdx.x; i < 256; i += kSelThreads) s_hist[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < nslots; i += kSelThreads) {
            bool valid;
            const uint32_t key = key_of(i, valid);
            if (valid && (key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 0xffu], 1u);
        }
        __syncthreads();
        if (threadIdx.x < kWave) {
            const int lane = threadIdx.x;
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = s_hist[255 - 4 * lane - j];
                tot += c[j];
            }
            uint32_t incl = tot;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            const uint32_t excl = incl - tot;
            if (excl < want && want <= incl) {
                uint32_t run = excl;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (run < want && want <= run + c[j]) {
                        s_sel[0] = 255 - 4 * lane - j;
                        s_sel[1] = run;
                    }
                    run += c[j];
                }
            }
        }
        __syncthreads();
        prefix |= s_sel[0] << shift;
        mask |= 0xffu << shift;
        want -= s_sel[1];
        __syncthreads();
    }
    *T = prefix;
    *want_out = want;
}

// OR over the wavefront (result in every lane).
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
    v |= dpp_u32<0x111, 0xF>(v);  // row_shr:1
    v |= dpp_u32<0x112, 0xF>(v);  // row_shr:2
    v |= dpp_u32<0x114, 0xF>(v);  // row_shr:4
    v |= dpp_u32<0x118, 0xF>(v);  // row_shr:8
    v |= dpp_u32<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
    v |= dpp_u32<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1);
}

// Most-significant-digit-first passes (8-bit digits, at most four) over the slots [0, nslots) whose key_of(i, valid)
// reports valid: finds the key T of the k-th best valid slot and the number `want` of valid slots equal to T that
// still belong to the k best (1 <= k <= number of valid slots).  hist: [4][256] in LDS, zero on entry, dirty on return
// (one histogram per pass, one barrier per pass).  U keys per thread are fetched before the first of them is used.
// Every thread of the workgroup must call this, with the same arguments.
//
// base, diff: what the caller knows about the keys' spread: every valid key agrees with `base` in every bit that is
// clear in `diff` (base = any valid key, diff = OR over the valid keys of key ^ base; base 0, diff ~0 if unknown).  The
// first digit starts at the highest bit set in diff: scores of one row share their sign and most of their exponent,
// so that the 256 bins of the first pass divide the range the keys really cover, not the whole float range.
//
// Early finish: once the digit's bin holds at most 64 slots, no further histogram is built.  One sweep appends the
// remaining bits of those slots to a list (in the last pass's histogram, which is then never needed), and every
// wavefront ranks the list by itself, one entry per lane: entries are made distinct by their list index, the entry of
// rank want - 1 carries the threshold.  The list's order depends on the order of the atomics; the threshold and the
// count above it do not.  With the spread known, 2000 distinct scores mostly take one histogram and the list; rows of
// equal scores take none (diff 0) or, if a few differ, up to four.
template <int THREADS, int U, typename KeyFn>
__device__ __forceinline__ void msd_select(KeyFn key_of, int nslots, uint32_t k, uint32_t* hist4, uint32_t base,
                                           uint32_t diff, uint32_t* T_out, uint32_t* want_out) {
    const int lane = threadIdx.x & (kWave - 1);
    if (diff == 0) {   // every valid key is `base`
        *T_out = base;
        *want_out = k;
        return;
    }
    int open = 32 - __clz(diff);   // bits [0, open) are still undecided
    uint32_t mask = open >= 32 ? 0u : ~0u << open, prefix = base & mask, want = k;
    for (int pass = 0; pass < 4; ++pass) {   // open <= 32 - 8 * pass
        const int shift = max(open - 8, 0);
        const uint32_t dmask = (1u << (open - shift)) - 1u;   // eight bits; fewer in a last, short digit
        uint32_t* hist = hist4 + pass * 256;
        for (int i0 = 0; i0 < nslots; i0 += U * THREADS) {   // uniform trip count: the wavefront votes below
            uint32_t kv[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) kv[u] = key_of(min(i0 + u * THREADS + (int)threadIdx.x, nslots - 1), ok[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool todo = ok[u] && i0 + u * THREADS + (int)threadIdx.x < nslots && (kv[u] & mask) == prefix;
                const uint32_t dg = (kv[u] >> shift) & dmask;
                // Scores of one row share their sign and most of their exponent: in the first pass a wavefront's keys
                // usually all carry one digit, and atomics of many lanes on one LDS word are served one per cycle (2000
                // keys on one word: 2000 cycles).  One vote: if every pending lane has the first one's digit, one lane
                // adds the count; otherwise one atomic per lane.  (Measured and dropped: counting the first lane's digit
                // by vote also when the wavefront is not unanimous, and peeling several digits off it one vote each;
                // the votes' scalar round trips cost what the shorter queues save, or more.)
                const unsigned long long act = __ballot(todo);
                if (act != 0) {
                    const int first = __ffsll((long long)act) - 1;
                    const uint32_t lead = __builtin_amdgcn_readlane(dg, first);
                    if (__ballot(todo && dg == lead) == act) {
                        if (lane == first) atomicAdd(&hist[lead], (uint32_t)__popcll(act));
                    } else if (todo) {
                        atomicAdd(&hist[dg], 1u);
                    }
                }
            }
        }
        __syncthreads();
        // Every wavefront finds the digit for itself (no broadcast through LDS, one barrier per pass): lane l owns
        // digits 255-4l .. 252-4l (descending); the digit where the running count from the top reaches `want`.
        const uint4 h4 = *reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);
        const uint32_t c[4] = {h4.w, h4.z, h4.y, h4.x};
        const uint32_t tot = c[0] + c[1] + c[2] + c[3];
        const uint32_t incl = wave_scan_incl(tot), excl = incl - tot;
        uint32_t digit = 0, above = 0, inbin = 0;
        const bool mine = excl < want && want <= incl;  // exactly one lane
        if (mine) {
            uint32_t run = excl;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (run < want && want <= run + c[j]) {
                    digit = 255 - 4 * lane - j;
                    above = run;
                    inbin = c[j];
                }
                run += c[j];
            }
        }
        const int src = __ffsll((long long)__ballot(mine)) - 1;
        digit = __builtin_amdgcn_readlane(digit, src);
        above = __builtin_amdgcn_readlane(above, src);
        inbin = __builtin_amdgcn_readlane(inbin, src);
        prefix |= digit << shift;
        mask |= dmask << shift;
        want -= above;   // 1 <= want <= inbin
        open = shift;
        if (open == 0) break;   // every bit is decided (after the fourth pass at the latest)
        if (inbin <= (uint32_t)kWave) {   // the same for every wavefront: all read the same histogram; pass <= 2 here
            // the last pass's histogram, still zero: [0] entries so far, [4 + i] entry i as a tag: the open bits of the
            // key above six bits that tell equal keys apart, plus one (0 = no entry)
            uint32_t* fill = hist4 + 3 * 256;
            for (int i0 = 0; i0 < nslots; i0 += U * THREADS) {
                uint32_t kv[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) kv[u] = key_of(min(i0 + u * THREADS + (int)threadIdx.x, nslots - 1), ok[u]);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (ok[u] && i0 + u * THREADS + (int)threadIdx.x < nslots && (kv[u] & mask) == prefix) {
                        const uint32_t idx = atomicAdd(fill, 1u);
                        fill[4 + idx] = (((kv[u] & ~mask) << 6) | (63u - idx)) + 1u;   // at most 24 open bits
                    }
                }
            }
            __syncthreads();
            const bool have = (uint32_t)lane < inbin;
            const uint32_t tag = fill[4 + lane];   // 0 beyond the list
            const uint32_t low = (tag - 1u) >> 6;
            // rank = entries with a larger tag; the list is read 16 entries at a time, every lane the same words
            uint32_t rank = 0;
            for (uint32_t c = 0; c < inbin; c += 16) {
                uint4 e[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) e[q] = *reinterpret_cast<const uint4*>(fill + 4 + c + 4 * q);
#pragma unroll
                for (int q = 0; q < 4; ++q) rank += (e[q].x > tag) + (e[q].y > tag) + (e[q].z > tag) + (e[q].w > tag);
            }
            const int at = __ffsll((long long)__ballot(have && rank == want - 1)) - 1;   // exactly one lane
            const uint32_t tlow = __builtin_amdgcn_readlane(low, at);
            *T_out = prefix | tlow;
            *want_out = want - (uint32_t)__popcll(__ballot(have && low > tlow));
            return;
        }
    }
    *T_out = prefix;
    *want_out = want;
}

}  // namespace fk
#endif
