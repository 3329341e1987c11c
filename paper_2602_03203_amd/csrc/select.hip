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
#include "select_common.h"

namespace fk {

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

// ---------------------------------------------------------------------------------------
// Sampled selection: Top-K multinomial eviction (Section 3.1 Eq. 2, Appendix B.2).
// The n_cand lowest-scored non-recent pairs are candidates; of them E = len - budget are evicted,
// drawn without replacement with probabilities softmax(-score).  The draw is taken in its
// Gumbel-top-k form on noise supplied by the caller: the E candidates with the smallest fp32
// t = score - noise go.  Two radix selects per row: (1) the others - n_cand most important pairs
// are safe; a bitmap in LDS marks the candidates; (2) among the candidates the n_cand - E largest t
// stay (ties to the lower slot).  One ordered pass writes the kept slots ascending.
// ---------------------------------------------------------------------------------------
static constexpr int kSampledMaxLen = 131072;  // bitmap of candidates: 16 KB of LDS

__global__ __launch_bounds__(kSelThreads) void select_keep_sampled_kernel(const float* __restrict__ scores,
                                                                          const float* __restrict__ noise,
                                                                          const int32_t* __restrict__ len, int cap,
                                                                          int budget, int recent, int n_cand,
                                                                          int32_t* __restrict__ keep) {
    const int row = blockIdx.x;
    const int n = min(min(len[row], cap), kSampledMaxLen);
    int32_t* out = keep + (size_t)row * budget;
    if (n <= budget) {
        for (int j = threadIdx.x; j < n; j += kSelThreads) out[j] = j;
        return;
    }
    const float* sc = scores + (size_t)row * cap;
    const float* nz = noise + (size_t)row * cap;
    const int others = n - recent;  // slots [0, others) are not protected
    const int E = n - budget;       // pairs to evict (1 <= E <= others)
    const int K = min(max(n_cand, E), others);  // candidates
    const int k_safe = others - K;  // most important pairs, never evicted
    const int k2 = K - E;           // candidates that stay

    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_sel[2];
    __shared__ unsigned long long s_part[kSelWaves];
    __shared__ unsigned long long s_cand[kSampledMaxLen / 64];  // bit i: slot i is a candidate
    const int lane = threadIdx.x & (kWave - 1);

    // (1) safe set
    uint32_t T1 = 0, want1 = 0;
    if (k_safe > 0)
        radix_threshold(others, (uint32_t)k_safe, [&](int i, bool& valid) { valid = true; return score_key(sc[i]); },
                        s_hist, s_sel, &T1, &want1);
    {
        uint32_t eq_base = 0;
        for (int base = 0; base < others; base += kSelThreads) {
            const int i = base + threadIdx.x;
            uint32_t gt = 0, eq = 0;
            if (i < others && k_safe > 0) {
                const uint32_t key = score_key(sc[i]);
                gt = key > T1;
                eq = key == T1;
            }
            unsigned long long tot;
            const unsigned long long incl = block_scan_incl((unsigned long long)eq, s_part, &tot);
            const uint32_t eq_before = eq_base + (uint32_t)incl - eq;
            const bool safe = gt || (eq && eq_before < want1);
            const unsigned long long bits = __ballot(i < others && !safe);
            if (lane == 0) s_cand[i >> 6] = bits;
            eq_base += (uint32_t)tot;
        }
    }
    __syncthreads();
    auto is_cand = [&](int i) { return (s_cand[i >> 6] >> (i & 63)) & 1ull; };

    // (2) which candidates stay: the k2 largest t = score - noise
    uint32_t T2 = 0, want2 = 0;
    if (k2 > 0)
        radix_threshold(others, (uint32_t)k2,
                        [&](int i, bool& valid) {
                            valid = is_cand(i);
                            return score_key(sc[i] - nz[i]);
                        },
                        s_hist, s_sel, &T2, &want2);

    // (3) ordered output: safe pairs, surviving candidates, protected tail
    unsigned long long run = 0;  // packed running counts: safe << 40 | gt2 << 20 | eq2
    for (int base = 0; base < others; base += kSelThreads) {
        const int i = base + threadIdx.x;
        unsigned long long safe = 0, gt = 0, eq = 0;
        if (i < others) {
            if (!is_cand(i)) {
                safe = 1;
            } else if (k2 > 0) {
                const uint32_t key = score_key(sc[i] - nz[i]);
                gt = key > T2;
                eq = key == T2;
            }
        }
        unsigned long long tot;
        const unsigned long long mine = (safe << 40) | (gt << 20) | eq;
        const unsigned long long before = run + block_scan_incl(mine, s_part, &tot) - mine;
        const uint32_t eq_before = (uint32_t)(before & 0xfffffull);
        if (safe || gt || (eq && eq_before < want2))
            out[(uint32_t)(before >> 40) + (uint32_t)((before >> 20) & 0xfffffull) + min(eq_before, want2)] = i;
        run += tot;
    }
    for (int j = threadIdx.x; j < recent; j += kSelThreads) out[budget - recent + j] = others + j;
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

extern "C" fk_status fk_select_keep_sampled(const fk_cache_desc* desc, const float* scores, const float* noise,
                                            const int32_t* pos, const int32_t* len, int32_t max_len, int32_t budget,
                                            int32_t protect_recent, int32_t n_candidates, int32_t* keep_idx,
                                            void* stream) {
    (void)pos;  // slot order stands for position order (cache precondition)
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!scores || !noise || !len || !keep_idx) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity || n_candidates < 0) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || budget > desc->capacity || protect_recent < 0 || protect_recent > budget)
        return FK_ERR_INVALID_ARG;
    if (max_len > kSampledMaxLen) return FK_ERR_UNSUPPORTED;
    const int rows = desc->batch * desc->n_kv_heads;
    hipLaunchKernelGGL(select_keep_sampled_kernel, dim3(rows), dim3(kSelThreads), 0, (hipStream_t)stream, scores,
                       noise, len, desc->capacity, budget, protect_recent, n_candidates, keep_idx);
    return launch_status();
}
