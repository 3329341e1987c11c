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

}  // namespace fk
#endif
