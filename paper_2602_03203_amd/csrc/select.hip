// fk_select_keep: deterministic per-row top-k by radix select (Section 3.1: the most recent
// L pairs stay, the others are pruned to the B - L most important; Top-K form of the
// sampling ablation).
//
// One workgroup per row.  Scores are mapped to order-preserving 32-bit keys (larger key =
// more important; -0 -> +0; NaN -> 0, below -inf).  Four most-significant-digit-first passes
// over 8-bit digits find the key T of the k-th best candidate and the number `take` of
// candidates equal to T that still fit.  One ordered pass then writes the kept slots
// ascending: every candidate above T, the first `take` candidates equal to T in slot order
// (slot order is position order, so ties go to the lower position), and the protected tail.
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

__global__ __launch_bounds__(kSelThreads) void select_keep_kernel(const float* __restrict__ scores,
                                                                  const int32_t* __restrict__ len,
                                                                  int cap, int budget, int recent,
                                                                  int32_t* __restrict__ keep) {
    const int row = blockIdx.x;
    const int n = min(len[row], cap);
    int32_t* out = keep + (size_t)row * budget;
    if (n <= budget) {
        for (int j = threadIdx.x; j < n; j += kSelThreads) out[j] = j;
        return;
    }
    const float* sc = scores + (size_t)row * cap;
    const int ncand = n - recent;   // candidates: slots [0, ncand)
    const int k = budget - recent;  // how many of them stay (0 <= k < ncand)

    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_sel[2];  // chosen digit, candidates above it
    __shared__ unsigned long long s_part[kSelWaves];

    uint32_t prefix = 0, mask = 0;
    uint32_t want = (uint32_t)k;   // how many still to take among keys matching the prefix
    if (k > 0) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (int i = threadIdx.x; i < 256; i += kSelThreads) s_hist[i] = 0;
            __syncthreads();
            for (int i = threadIdx.x; i < ncand; i += kSelThreads) {
                const uint32_t key = score_key(sc[i]);
                if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 0xffu], 1u);
            }
            __syncthreads();
            if (threadIdx.x < kWave) {
                // lane l owns digits 255-4l .. 252-4l (descending); find the digit where the
                // running count from the top reaches `want`
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
                if (excl < want && want <= incl) {  // exactly one lane
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
    }
    // now: keep key > prefix, and the first `want` keys == prefix (k == 0: keep no candidate)
    const uint32_t T = prefix;
    uint32_t gt_base = 0, eq_base = 0;
    for (int base = 0; base < ncand; base += kSelThreads) {
        const int i = base + threadIdx.x;
        uint32_t gt = 0, eq = 0;
        if (i < ncand && k > 0) {
            const uint32_t key = score_key(sc[i]);
            gt = key > T;
            eq = key == T;
        }
        unsigned long long tot;
        const unsigned long long incl =
            block_scan_incl(((unsigned long long)gt << 32) | eq, s_part, &tot);
        const uint32_t gt_before = gt_base + (uint32_t)(incl >> 32) - gt;
        const uint32_t eq_before = eq_base + (uint32_t)(incl & 0xffffffffu) - eq;
        if (gt || (eq && eq_before < want)) out[gt_before + min(eq_before, want)] = i;
        gt_base += (uint32_t)(tot >> 32);
        eq_base += (uint32_t)(tot & 0xffffffffu);
    }
    for (int j = threadIdx.x; j < recent; j += kSelThreads) out[k + j] = ncand + j;
}

}  // namespace fk

using namespace fk;

extern "C" fk_status fk_select_keep(const fk_cache_desc* desc, const float* scores, const int32_t* pos,
                                    const int32_t* len, int32_t max_len, int32_t budget,
                                    int32_t protect_recent, int32_t* keep_idx, void* stream) {
    (void)pos;  // slot order stands for position order (cache precondition)
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!scores || !len || !keep_idx) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || budget > desc->capacity || protect_recent < 0 || protect_recent > budget)
        return FK_ERR_INVALID_ARG;
    const int rows = desc->batch * desc->n_kv_heads;
    hipLaunchKernelGGL(select_keep_kernel, dim3(rows), dim3(kSelThreads), 0, (hipStream_t)stream, scores,
                       len, desc->capacity, budget, protect_recent, keep_idx);
    return launch_status();
}
