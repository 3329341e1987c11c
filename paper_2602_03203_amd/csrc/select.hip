// fk_select_keep: deterministic per-row top-k by radix select (Section 3.1: the most recent
// L pairs stay, the others are pruned to the B - L most important; Top-K form of the
// sampling ablation).
//
// One workgroup per row.  Scores are read once, mapped to order-preserving 32-bit keys (larger key =
// more important; -0 -> +0; NaN -> 0, below -inf) and kept in LDS.  Most-significant-digit-first passes over
// 8-bit digits (LDS histograms, one barrier per pass; at most four, usually one and a short ranked list: see
// msd_select) find the key T of the k-th best candidate and the number `take` of candidates equal to T that still
// fit.  One ordered pass then writes the kept slots
// ascending: every candidate above T, the first `take` candidates equal to T in slot order
// (slot order is position order, so ties go to the lower position), and the protected tail.
#include "select_common.h"
#include <type_traits>

namespace fk {

// LDS: hist [4][256] u32 (one histogram per pass, cleared once) | wavefront totals [16][2] | wavefront ORs [16] |
// keys [lds_keys] u32
static constexpr int kSelMaxLdsKeys = 36 * 1024;  // 144 KB of keys beside the histograms
static constexpr int kSelLdsHead = 4 * 256 + 32 + 16;  // words before the keys: histograms, wavefront counts, wavefront ORs
// (Four wavefronts per row instead of sixteen were measured and dropped: 11.3 against 8.1 us; a pass is a chain
// key -> atomic -> barrier -> scan of LDS round trips, which more wavefronts shorten.)
//
// Long rows of a small batch (one-shot compression of a long prompt: 32 rows of 131072 pairs) would leave most of the
// chip idle with one workgroup per row, and their keys do not fit LDS.  fk_select_keep_ws splits such rows (two launches,
// a workspace between them): kSelChunk workgroups, one per chunk of a row, each keep the k best candidates of
// their chunk (any pair among the row's k best is among its chunk's k best, under the same total order); kSelMerge
// workgroups, one per row, then select among the chunks' survivors, whose keys fit LDS.  Same result, bit for bit.
enum { kSelWhole = 0, kSelChunk = 1, kSelMerge = 2 };
struct SelSplit {
    int nchunk;      // chunks per row
    int chunk_len;   // candidates per chunk (the last chunk runs on to the row's end)
    int32_t* count;  // [rows][nchunk] survivors of every chunk
    int32_t* cand;   // [rows][nchunk][budget - recent] their slots, ascending
};

template <int THREADS, int MODE>
__global__ __launch_bounds__(THREADS) void select_keep_kernel(const float* __restrict__ scores,
                                                              const int32_t* __restrict__ len,
                                                              int cap, int budget, int recent, int lds_keys,
                                                              int32_t* __restrict__ keep, SelSplit sp) {
    const int row = MODE == kSelChunk ? blockIdx.x / sp.nchunk : blockIdx.x;
    const int chunk = MODE == kSelChunk ? blockIdx.x % sp.nchunk : 0;
    const int n = min(len[row], cap);
    const int kmax = budget - recent;
    int32_t* out = MODE == kSelChunk ? sp.cand + ((size_t)row * sp.nchunk + chunk) * kmax : keep + (size_t)row * budget;
    if (n <= budget) {  // nothing to prune: the identity over the whole row, which makes the compaction a no-op
        if (MODE != kSelChunk)
            for (int j = threadIdx.x; j < budget; j += THREADS) out[j] = j;
        return;
    }
    const float* sc = scores + (size_t)row * cap;
    const int first = MODE == kSelChunk ? chunk * sp.chunk_len : 0;  // first slot of this workgroup's candidates
    int ncand = n - recent;  // candidates: slots [first, first + ncand)
    int k = kmax;            // how many of them stay (0 <= k < ncand; a chunk: k <= ncand)

    extern __shared__ __attribute__((aligned(16))) uint32_t s_sel_mem[];
    uint32_t* s_hist = s_sel_mem;                 // [4][256]
    uint32_t* s_wtot = s_hist + 4 * 256;          // [16][2]: kept counts of every wavefront (greater, equal)
    uint32_t* s_wor = s_wtot + 32;                // [16]: every wavefront's OR of key ^ first key
    uint32_t* s_key = s_wor + 16;                 // [lds_keys]
    uint32_t* s_slot = s_key + lds_keys;          // kSelMerge: [lds_keys] the candidates' slots
    constexpr int WAVES = THREADS / kWave;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if constexpr (MODE == kSelChunk) {
        ncand = chunk == sp.nchunk - 1 ? ncand - first : min(ncand - first, sp.chunk_len);
        if (ncand < 0) ncand = 0;
        k = min(kmax, ncand);
        if (threadIdx.x == 0) sp.count[(size_t)row * sp.nchunk + chunk] = k;
        if (k == ncand) {  // the whole chunk survives (also: an empty chunk, nothing to keep)
            for (int j = threadIdx.x; j < ncand; j += THREADS) out[j] = first + j;
            return;
        }
        sc += first;
    }
    constexpr int kMaxChunks = 16;
    int base_of[kMaxChunks + 1];  // kSelMerge: where every chunk's survivors start in the merged list (registers)
    if constexpr (MODE == kSelMerge) {
        int tot = 0;
#pragma unroll
        for (int c = 0; c < kMaxChunks; ++c) {
            base_of[c] = tot;
            if (c < sp.nchunk) tot += sp.count[(size_t)row * sp.nchunk + c];
        }
        base_of[kMaxChunks] = tot;
        ncand = tot;  // >= k: every chunk keeps min(k, its size)
    }

    // The row's keys are read from global memory once and kept in LDS (rows beyond the LDS share of the launch are
    // re-read from global memory in every pass).  Eight loads in flight per thread.
    const bool in_lds = ncand <= lds_keys;  // kSelMerge: the host sized the launch so that it is
    uint32_t base = 0, diff = ~0u;          // the keys' common bits, where known (msd_select)
    for (int i = threadIdx.x; i < 4 * 256; i += THREADS) s_hist[i] = 0;
    if constexpr (MODE == kSelMerge) {
#pragma unroll
        for (int c = 0; c < kMaxChunks; ++c) {
            if (c < sp.nchunk) {
                const int32_t* list = sp.cand + ((size_t)row * sp.nchunk + c) * kmax;
                const int cnt = base_of[c + 1] - base_of[c];
                for (int o = threadIdx.x; o < cnt; o += THREADS) {
                    const int slot = list[o];
                    s_slot[base_of[c] + o] = (uint32_t)slot;
                    s_key[base_of[c] + o] = score_key(sc[slot]);
                }
            }
        }
    } else if (in_lds) {
        // on the way: which bits differ between any two keys of the row (the select starts at the highest of them)
        base = score_key(sc[0]);
        uint32_t spread = 0;
        for (int i0 = threadIdx.x; i0 < ncand; i0 += 8 * THREADS) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = sc[min(i0 + u * THREADS, ncand - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (i0 + u * THREADS < ncand) {
                    const uint32_t key = score_key(v[u]);
                    s_key[i0 + u * THREADS] = key;
                    spread |= key ^ base;
                }
            }
        }
        spread = wave_or(spread);
        if (lane == 0) s_wor[wave] = spread;
    }
    __syncthreads();
    if (MODE != kSelMerge && in_lds) {
        diff = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) diff |= s_wor[w];
    }
    auto key_at = [&](int i) { return in_lds ? s_key[i] : score_key(sc[i]); };

    // (rows read from global memory: 16 loads in flight per thread)
    uint32_t prefix = 0;
    uint32_t want = (uint32_t)k;   // how many still to take among keys equal to the threshold
    if (k > 0) {
        auto key_of = [&](int i, bool& valid) { valid = true; return key_at(i); };
        if (in_lds) msd_select<THREADS, 2>(key_of, ncand, (uint32_t)k, s_hist, base, diff, &prefix, &want);
        else msd_select<THREADS, 16>(key_of, ncand, (uint32_t)k, s_hist, base, diff, &prefix, &want);
    }
    // now: keep key > prefix, and the first `want` keys == prefix (k == 0: keep no candidate).  Ordered pass: every
    // wavefront owns one contiguous stretch of the row and walks it 64 slots at a time (coalesced, no barrier inside):
    // first to count its kept slots, then, with the counts of the stretches before it, to write them in order.
    const uint32_t T = prefix;
    const int stretch = (((ncand + WAVES - 1) / WAVES) + kWave - 1) / kWave * kWave;
    const int w0 = min(wave * stretch, ncand), w1 = min(w0 + stretch, ncand);
    auto walk = [&](auto u_, auto write_, uint32_t& gt_run, uint32_t& eq_run) {
        constexpr int U = decltype(u_)::value;
        constexpr bool WRITE = decltype(write_)::value;
        for (int i0 = w0; i0 < w1; i0 += U * kWave) {
            uint32_t kv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) kv[u] = key_at(min(i0 + u * kWave + lane, ncand - 1));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * kWave + lane;
                const bool live = i < w1;
                const unsigned long long mg = __ballot(live && kv[u] > T), me = __ballot(live && kv[u] == T);
                if constexpr (WRITE) {
                    const uint32_t g_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, 0));
                    const uint32_t e_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0));
                    const uint32_t gb = gt_run + g_below, eb = eq_run + e_below;   // kept counts before slot i
                    const int slot = MODE == kSelMerge ? (live ? (int)s_slot[i] : 0) : first + i;
                    if (live && kv[u] > T) out[gb + min(eb, want)] = slot;
                    else if (live && kv[u] == T && eb < want) out[gb + eb] = slot;
                }
                gt_run += (uint32_t)__popcll(mg);
                eq_run += (uint32_t)__popcll(me);
            }
        }
    };
    constexpr std::integral_constant<int, 2> few{};
    constexpr std::integral_constant<int, 16> many{};
    uint32_t gt = 0, eq = 0;
    if (k > 0) {
        if (in_lds) walk(few, std::false_type{}, gt, eq);
        else walk(many, std::false_type{}, gt, eq);
    }
    if (lane == 0) {
        s_wtot[2 * wave] = gt;
        s_wtot[2 * wave + 1] = eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) {
        gt_before += s_wtot[2 * w];
        eq_before += s_wtot[2 * w + 1];
    }
    if (k > 0) {
        if (in_lds) walk(few, std::true_type{}, gt_before, eq_before);
        else walk(many, std::true_type{}, gt_before, eq_before);
    }
    if (MODE != kSelChunk)
        for (int j = threadIdx.x; j < recent; j += THREADS) out[k + j] = n - recent + j;
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
    const int n = min(len[row], cap);  // cap <= kSampledMaxLen (checked on the host)
    int32_t* out = keep + (size_t)row * budget;
    if (n <= budget) {  // nothing to prune: the identity over the whole row
        for (int j = threadIdx.x; j < budget; j += kSelThreads) out[j] = j;
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


// The same selection with the row in LDS (rows of up to kSampledLdsKeys candidates): both keys of every slot are formed
// once, the radix passes and the ordered passes are those of select_keep_kernel (one barrier per pass, one ordered
// walk per wavefront stretch), and the candidate marks take the place of the first key once the safe set is known.
// LDS: hist [2][4][256] u32 | wavefront totals [16][4] | wavefront ORs [2][16] | key1 / candidate mark [lds_keys] |
// key2 [lds_keys]
static constexpr int kSampledLdsKeys = 18 * 1024;
template <int THREADS>
__global__ __launch_bounds__(THREADS) void select_keep_sampled_lds_kernel(const float* __restrict__ scores,
                                                                          const float* __restrict__ noise,
                                                                          const int32_t* __restrict__ len, int cap,
                                                                          int budget, int recent, int n_cand, int lds_keys,
                                                                          int32_t* __restrict__ keep) {
    const int row = blockIdx.x;
    const int n = min(len[row], cap);
    int32_t* out = keep + (size_t)row * budget;
    if (n <= budget) {  // nothing to prune: the identity over the whole row
        for (int j = threadIdx.x; j < budget; j += THREADS) out[j] = j;
        return;
    }
    const float* sc = scores + (size_t)row * cap;
    const float* nz = noise + (size_t)row * cap;
    const int others = n - recent;  // slots [0, others) are not protected (others <= lds_keys: checked on the host)
    const int E = n - budget;       // pairs to evict (1 <= E <= others)
    const int K = min(max(n_cand, E), others);  // candidates
    const int k_safe = others - K;  // most important pairs, never evicted
    const int k2 = K - E;           // candidates that stay

    extern __shared__ __attribute__((aligned(16))) uint32_t s_sel_mem[];
    uint32_t* s_hist = s_sel_mem;            // [2][4][256]
    uint32_t* s_wtot = s_hist + 2 * 4 * 256; // [16][4]
    uint32_t* s_wor = s_wtot + 64;           // [2][16] every wavefront's OR of key ^ first key, for either key
    uint32_t* s_k1 = s_wor + 32;             // [lds_keys] key of the score; later 1 = candidate, 0 = safe
    uint32_t* s_k2 = s_k1 + lds_keys;        // [lds_keys] key of score - noise
    constexpr int WAVES = THREADS / kWave;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

    for (int i = threadIdx.x; i < 2 * 4 * 256; i += THREADS) s_hist[i] = 0;
    // on the way: the bits in which any two keys of the row differ (either select starts at the highest of them)
    const uint32_t base1 = score_key(sc[0]), base2 = score_key(sc[0] - nz[0]);
    uint32_t spread1 = 0, spread2 = 0;
    for (int i0 = threadIdx.x; i0 < others; i0 += 8 * THREADS) {
        float v[8], z[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = min(i0 + u * THREADS, others - 1);
            v[u] = sc[i];
            z[u] = nz[i];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i0 + u * THREADS < others) {
                const uint32_t key1 = score_key(v[u]), key2 = score_key(v[u] - z[u]);
                s_k1[i0 + u * THREADS] = key1;
                s_k2[i0 + u * THREADS] = key2;
                spread1 |= key1 ^ base1;
                spread2 |= key2 ^ base2;
            }
    }
    spread1 = wave_or(spread1);
    spread2 = wave_or(spread2);
    if (lane == 0) {
        s_wor[wave] = spread1;
        s_wor[16 + wave] = spread2;
    }
    __syncthreads();
    uint32_t diff1 = 0, diff2 = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        diff1 |= s_wor[w];
        diff2 |= s_wor[16 + w];
    }

    // every wavefront owns one contiguous stretch of the row (the ordered passes walk it 64 slots at a time)
    const int stretch = (((others + WAVES - 1) / WAVES) + kWave - 1) / kWave * kWave;
    const int w0 = min(wave * stretch, others), w1 = min(w0 + stretch, others);

    // (1) safe set: the k_safe best by score; everything else becomes a candidate
    uint32_t T1 = 0, want1 = 0;
    if (k_safe > 0)
        msd_select<THREADS, 2>([&](int i, bool& valid) { valid = true; return s_k1[i]; }, others, (uint32_t)k_safe, s_hist, base1, diff1, &T1,
                               &want1);
    {
        uint32_t eq = 0;  // slots equal to T1 in this stretch
        if (k_safe > 0)
            for (int i0 = w0; i0 < w1; i0 += kWave) {
                const int i = i0 + lane;
                eq += (uint32_t)__popcll(__ballot(i < w1 && s_k1[min(i, others - 1)] == T1));
            }
        if (lane == 0) s_wtot[4 * wave] = eq;
        __syncthreads();
        uint32_t eq_run = 0;
        for (int w = 0; w < wave; ++w) eq_run += s_wtot[4 * w];
        for (int i0 = w0; i0 < w1; i0 += kWave) {
            const int i = i0 + lane;
            const bool live = i < w1;
            const uint32_t key = s_k1[min(i, others - 1)];
            const bool is_eq = k_safe > 0 && live && key == T1;
            const unsigned long long me = __ballot(is_eq);
            const uint32_t e_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0));
            const bool safe = k_safe > 0 && (key > T1 || (is_eq && eq_run + e_below < want1));
            if (live) s_k1[i] = safe ? 0u : 1u;
            eq_run += (uint32_t)__popcll(me);
        }
    }
    __syncthreads();

    // (2) which candidates stay: the k2 largest t = score - noise among them
    uint32_t T2 = 0, want2 = 0;
    if (k2 > 0)
        msd_select<THREADS, 2>([&](int i, bool& valid) { valid = s_k1[i] != 0u; return s_k2[i]; }, others, (uint32_t)k2,
                               s_hist + 4 * 256, base2, diff2, &T2, &want2);

    // (3) ordered output: safe pairs, surviving candidates (ties to the lower slot), protected tail
    auto walk = [&](auto write_, uint32_t& keep_run, uint32_t& eq_run) {
        constexpr bool WRITE = decltype(write_)::value;
        for (int i0 = w0; i0 < w1; i0 += kWave) {
            const int i = i0 + lane;
            const bool live = i < w1;
            const int ii = min(i, others - 1);
            const bool cand = s_k1[ii] != 0u;
            const uint32_t key = s_k2[ii];
            const bool sure = live && (!cand || (k2 > 0 && key > T2));   // kept whatever the ties do
            const bool tie = live && cand && k2 > 0 && key == T2;
            const unsigned long long ms = __ballot(sure), mt = __ballot(tie);
            if constexpr (WRITE) {
                const uint32_t s_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(ms >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ms, 0));
                const uint32_t t_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(mt >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mt, 0));
                const uint32_t sb = keep_run + s_below, tb = eq_run + t_below;  // kept for sure / tied, before slot i
                if (sure) out[sb + min(tb, want2)] = i;
                else if (tie && tb < want2) out[sb + tb] = i;
            }
            keep_run += (uint32_t)__popcll(ms);
            eq_run += (uint32_t)__popcll(mt);
        }
    };
    uint32_t kept = 0, tied = 0;
    walk(std::false_type{}, kept, tied);
    if (lane == 0) {
        s_wtot[4 * wave + 1] = kept;
        s_wtot[4 * wave + 2] = tied;
    }
    __syncthreads();
    uint32_t kept_before = 0, tied_before = 0;
    for (int w = 0; w < wave; ++w) {
        kept_before += s_wtot[4 * w + 1];
        tied_before += s_wtot[4 * w + 2];
    }
    walk(std::true_type{}, kept_before, tied_before);
    for (int j = threadIdx.x; j < recent; j += THREADS) out[budget - recent + j] = others + j;
}

}  // namespace fk

using namespace fk;

static fk_status select_check(const fk_cache_desc* desc, const float* scores, const int32_t* len, int32_t max_len,
                              int32_t budget, int32_t protect_recent, const int32_t* keep_idx) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!scores || !len || !keep_idx) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || budget > desc->capacity || protect_recent < 0 || protect_recent > budget)
        return FK_ERR_INVALID_ARG;
    return FK_OK;
}

static fk_status select_whole(const fk_cache_desc* desc, const float* scores, const int32_t* len, int32_t max_len,
                              int32_t budget, int32_t protect_recent, int32_t* keep_idx, hipStream_t st) {
    const int rows = desc->batch * desc->n_kv_heads;
    // LDS share for the keys: rows up to max_len keys (the hint) live in LDS; longer ones are read from global memory
    const int lds_keys = ((max_len < kSelMaxLdsKeys ? max_len : kSelMaxLdsKeys) + 3) & ~3;
    const size_t lds = sizeof(uint32_t) * (kSelLdsHead + (size_t)lds_keys);
    auto kern = select_keep_kernel<kSelThreads, kSelWhole>;
    static bool lds_ok[kMaxDevices] = {};
    if (!allow_dynamic_lds((const void*)kern, 160 * 1024, lds_ok)) return FK_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(rows), dim3(kSelThreads), lds, st, scores, len, desc->capacity, budget, protect_recent,
                       lds_keys, keep_idx, SelSplit{});
    return launch_status();
}

extern "C" fk_status fk_select_keep(const fk_cache_desc* desc, const float* scores, const int32_t* pos,
                                    const int32_t* len, int32_t max_len, int32_t budget,
                                    int32_t protect_recent, int32_t* keep_idx, void* stream) {
    (void)pos;  // slot order stands for position order (cache precondition)
    const fk_status s = select_check(desc, scores, len, max_len, budget, protect_recent, keep_idx);
    if (s != FK_OK) return s;
    return select_whole(desc, scores, len, max_len, budget, protect_recent, keep_idx, (hipStream_t)stream);
}

// Rows are split when one workgroup per row would leave most CUs idle and the rows are long enough to pay for a
// second launch; the survivors of all chunks (keys and slots) must fit the merge workgroup's LDS.
struct SelPlan {
    int nchunk, chunk_len;
    size_t count_bytes, bytes;
};
static SelPlan select_plan(const fk_cache_desc* d, int max_len, int budget, int recent) {
    SelPlan p = {1, 0, 0, 0};
    const int rows = d->batch * d->n_kv_heads, kmax = budget - recent;
    if (rows > 64 || max_len < 16384 || kmax <= 0) return p;
    int nchunk = 256 / rows;                                   // one workgroup per CU (measured: 128 and 512 are slower)
    const int fit = (kSelMaxLdsKeys / 2) / kmax;               // survivors of all chunks: keys + slots in LDS
    if (nchunk > fit) nchunk = fit;
    if (nchunk > 16) nchunk = 16;  // kMaxChunks of the kernel
    if (nchunk < 2) return p;
    p.nchunk = nchunk;
    p.chunk_len = ((max_len - recent + nchunk - 1) / nchunk + 3) & ~3;
    p.count_bytes = ((size_t)rows * nchunk * sizeof(int32_t) + 255) & ~(size_t)255;
    p.bytes = p.count_bytes + (size_t)rows * nchunk * kmax * sizeof(int32_t);
    return p;
}

extern "C" size_t fk_select_keep_workspace(const fk_cache_desc* desc, int32_t max_len, int32_t budget, int32_t protect_recent) {
    if (check_desc(desc) != FK_OK || max_len <= 0 || max_len > desc->capacity || budget <= 0 || budget > desc->capacity ||
        protect_recent < 0 || protect_recent > budget)
        return 0;
    return select_plan(desc, max_len, budget, protect_recent).bytes;
}

extern "C" fk_status fk_select_keep_ws(const fk_cache_desc* desc, const float* scores, const int32_t* pos,
                                       const int32_t* len, int32_t max_len, int32_t budget, int32_t protect_recent,
                                       int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* stream) {
    (void)pos;
    const fk_status s = select_check(desc, scores, len, max_len, budget, protect_recent, keep_idx);
    if (s != FK_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const SelPlan p = select_plan(desc, max_len, budget, protect_recent);
    if (p.nchunk < 2) return select_whole(desc, scores, len, max_len, budget, protect_recent, keep_idx, st);
    if (!workspace || workspace_bytes < p.bytes) return FK_ERR_WORKSPACE;
    const int rows = desc->batch * desc->n_kv_heads, kmax = budget - protect_recent;
    SelSplit sp = {p.nchunk, p.chunk_len, reinterpret_cast<int32_t*>(workspace),
                   reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + p.count_bytes)};
    {
        auto kern = select_keep_kernel<kSelThreads, kSelChunk>;
        const int lds_keys = ((p.chunk_len < kSelMaxLdsKeys ? p.chunk_len : kSelMaxLdsKeys) + 3) & ~3;
        const size_t lds = sizeof(uint32_t) * (kSelLdsHead + (size_t)lds_keys);
        static bool lds_ok[kMaxDevices] = {};
        if (!allow_dynamic_lds((const void*)kern, 160 * 1024, lds_ok)) return FK_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(rows * p.nchunk), dim3(kSelThreads), lds, st, scores, len, desc->capacity, budget,
                           protect_recent, lds_keys, keep_idx, sp);
        if (launch_status() != FK_OK) return FK_ERR_LAUNCH;
    }
    {
        auto kern = select_keep_kernel<kSelThreads, kSelMerge>;
        const int lds_keys = (p.nchunk * kmax + 3) & ~3;  // <= kSelMaxLdsKeys / 2 by the plan
        const size_t lds = sizeof(uint32_t) * (kSelLdsHead + 2 * (size_t)lds_keys);
        static bool lds_ok[kMaxDevices] = {};
        if (!allow_dynamic_lds((const void*)kern, 160 * 1024, lds_ok)) return FK_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(rows), dim3(kSelThreads), lds, st, scores, len, desc->capacity, budget, protect_recent,
                           lds_keys, keep_idx, sp);
    }
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
    if (desc->capacity > kSampledMaxLen) return FK_ERR_UNSUPPORTED;  // the candidate bitmap covers every slot a row can hold
    const int rows = desc->batch * desc->n_kv_heads;
    if (desc->capacity <= kSampledLdsKeys) {  // every row fits LDS with both of its keys
        const int lds_keys = (desc->capacity + 3) & ~3;
        const size_t lds = sizeof(uint32_t) * (2 * 4 * 256 + 64 + 32 + 2 * (size_t)lds_keys);
        auto kern = select_keep_sampled_lds_kernel<kSelThreads>;
        static bool lds_ok[kMaxDevices] = {};
        if (!allow_dynamic_lds((const void*)kern, 160 * 1024, lds_ok)) return FK_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(rows), dim3(kSelThreads), lds, (hipStream_t)stream, scores, noise, len, desc->capacity,
                           budget, protect_recent, n_candidates, lds_keys, keep_idx);
        return launch_status();
    }
    hipLaunchKernelGGL(select_keep_sampled_kernel, dim3(rows), dim3(kSelThreads), 0, (hipStream_t)stream, scores,
                       noise, len, desc->capacity, budget, protect_recent, n_candidates, keep_idx);
    return launch_status();
}
