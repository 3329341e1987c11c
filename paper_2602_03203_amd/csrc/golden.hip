// Golden Eviction label builder (Section 3.2 Eq. 3-5) on dense causal attention matrices.
//
//   pool   a~[h'][t][i] = 1/(g L) * sum over the g heads of group h' and the queries q of block t
//                         (B + tL <= q < min(B + (t+1)L, T)) of A[h][q][i]          (Eq. 3, 4)
//   future alpha[h'][t][i] = max_{j >= t} a~[h'][j][i]                               (Eq. 5, first half)
//   trace  step t keeps the L newest pairs and, of the other B the cache holds, the B - L with
//          the largest alpha[.][t] (ties: lower position), evicted pairs never return  (Eq. 5, second half)
//
// pool is the only kernel that touches the O(T^2) input and is HBM bound: a workgroup owns one
// (key tile, block, group) and streams g * L row segments of 256 bytes (16 lanes x 16 bytes, 16 rows per
// workgroup instruction, four instructions in flight per thread); tiles wholly above the diagonal are
// never read (A is causal), so the traffic is the lower triangle below query B + L.  future is a
// running maximum down the block axis; trace is sequential by nature: one workgroup per group walks the
// M steps with the radix select of fk_select_keep on keys in LDS (the next step's are loaded while a step selects).
#include "select_common.h"

namespace fk {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
static constexpr int kPoolThreads = 256;
static constexpr int kPoolRowGroups = kPoolThreads / 16;  // rows covered by one load instruction of the workgroup
static constexpr int kPoolU = 4;                          // loads in flight per thread

template <typename T>
__global__ __launch_bounds__(kPoolThreads) void golden_pool_kernel(const T* __restrict__ A, int g, int Tn, size_t ld,
                                                                   int budget, int L, int M,
                                                                   float* __restrict__ a_tilde) {
    constexpr int EPC = Vec16<T>::N;   // elements per 16-byte chunk
    constexpr int KT = 16 * EPC;       // keys per tile (256 bytes of a row)
    const int i0 = blockIdx.x * KT, t = blockIdx.y + 1, hp = blockIdx.z;
    const int q0 = budget + t * L, q1 = min(q0 + L, Tn);
    const int c = threadIdx.x & 15, rg = threadIdx.x >> 4;
    float acc[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
    const int qs = max(q0, i0);        // queries before the tile's first key see none of it
    const int rows = q1 - qs;          // <= 0: the tile lies above the diagonal for the whole block
    const bool col_ok = (size_t)i0 + (size_t)c * EPC < ld;
    if (rows > 0 && col_ok) {
        const int total = rows * g;    // (head, query) pairs, head-major
        const T* base = A + (size_t)hp * g * Tn * ld + (size_t)i0 + (size_t)c * EPC;
        for (int r0 = rg; r0 < total; r0 += kPoolRowGroups * kPoolU) {
            uint4 v[kPoolU];
#pragma unroll
            for (int u = 0; u < kPoolU; ++u) {
                const int r = min(r0 + u * kPoolRowGroups, total - 1);
                const int h = r / rows, q = qs + r % rows;
                // read once, never again: non-temporal, so the lines do not push anything out of the caches
                const u32x4 t4 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + ((size_t)h * Tn + q) * ld));
                v[u] = make_uint4(t4.x, t4.y, t4.z, t4.w);
            }
#pragma unroll
            for (int u = 0; u < kPoolU; ++u) {
                if (r0 + u * kPoolRowGroups < total) {
                    float x[EPC];
                    Vec16<T>::unpack(v[u], x);
#pragma unroll
                    for (int e = 0; e < EPC; ++e) acc[e] += x[e];
                }
            }
        }
    }
    __shared__ float s_acc[kPoolRowGroups][KT + 4];
#pragma unroll
    for (int e = 0; e < EPC; ++e) s_acc[rg][c * EPC + e] = acc[e];
    __syncthreads();
    if ((int)threadIdx.x < KT && i0 + (int)threadIdx.x < Tn) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < kPoolRowGroups; ++r) s += s_acc[r][threadIdx.x];
        a_tilde[((size_t)hp * M + (t - 1)) * Tn + i0 + threadIdx.x] = s / ((float)g * (float)L);
    }
}

// alpha[t] = max(a~[t], alpha[t + 1]), walking the blocks from the last to the first; one thread per key,
// eight blocks' loads in flight
__global__ void golden_future_kernel(const float* __restrict__ a_tilde, int Tn, int M, float* __restrict__ alpha) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x, hp = blockIdx.y;
    if (i >= Tn) return;
    const size_t o0 = (size_t)hp * M * Tn + i;
    float run = 0.f;
    for (int t = M; t >= 1; t -= 8) {
        float a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = t - u >= 1 ? a_tilde[o0 + (size_t)(t - u - 1) * Tn] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (t - u >= 1) {
                run = t - u == M ? a[u] : fmaxf(run, a[u]);
                alpha[o0 + (size_t)(t - u - 1) * Tn] = run;
            }
        }
    }
}

static constexpr int kTraceMaxCache = 12288;  // B + L positions and B keys in LDS (96 KB)

// One workgroup per KV group.  LDS holds the cache's positions (ascending; B + L of them: the B of this step and the
// L that are generated before the next one) and the keys of its first B entries under this step's future scores.
// A step: (1) the loads of the NEXT step's future scores at every position that can still be a candidate then are
// issued (they land while the step selects); (2) four radix passes find the key of the (B - L)-th best candidate;
// (3) every wavefront walks its own contiguous stretch of the candidates, first to count its survivors, then, with
// the counts of the stretches before it, to move them (position and next key) to the front in order.  Sources are
// in registers before the barrier that precedes the moves, so the compaction is safe in place.
// PER_LANE: candidates one lane holds (stretch of a wavefront / 64) and newest pairs one thread holds (L / 1024), at most.
template <int PER_LANE>
__global__ __launch_bounds__(kSelThreads) void golden_trace_kernel(const float* __restrict__ alpha, int Tn, int M,
                                                                   int budget, int L, int32_t* __restrict__ kept) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t* s_pos = reinterpret_cast<int32_t*>(smem);                 // [budget + L]
    uint32_t* s_key = reinterpret_cast<uint32_t*>(s_pos + budget + L);  // [budget]
    __shared__ __attribute__((aligned(16))) uint32_t s_hist[4 * 256];
    __shared__ uint32_t s_wtot[2 * kSelWaves];
    __shared__ uint32_t s_wor[kSelWaves];   // every wavefront's OR of key ^ base over the keys it wrote for the next step
    static_assert(kSelThreads == 4 * 256, "one thread clears one histogram word");
    const int hp = blockIdx.x, lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int k = budget - L;  // old pairs that stay
    const float* al = alpha + (size_t)hp * M * Tn;
    for (int j = threadIdx.x; j < budget + L; j += kSelThreads) s_pos[j] = j;
    // base, spread: one of the step's keys and the bits in which any of them differs from it (the select starts at
    // the highest such bit); the spread of the next step's keys is gathered while they are written
    uint32_t base = score_key(al[0]), spread = 0;
    for (int j = threadIdx.x; j < budget; j += kSelThreads) {
        const uint32_t key = score_key(al[j]);
        s_key[j] = key;
        spread |= key ^ base;
    }
    spread = wave_or(spread);
    if (lane == 0) s_wor[wave] = spread;
    s_hist[threadIdx.x] = 0;
    __syncthreads();
    const int stretch = ((budget + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;  // <= 64 * PER_LANE (host)
    const int w0 = min(wave * stretch, budget), w1 = min(w0 + stretch, budget);
    for (int t = 1; t <= M; ++t) {
        int32_t* out = kept + ((size_t)hp * M + (t - 1)) * budget;
        const bool more = t < M;
        const float* aln = al + (size_t)t * Tn;   // future scores of step t + 1
        const int new0 = budget + (t - 1) * L;   // first of the L newest pairs (they stay)
        uint32_t diff = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) diff |= s_wor[w];
        const uint32_t base_next = more ? score_key(aln[new0]) : 0u;
        float nxt[PER_LANE], nxt_new[PER_LANE];
#pragma unroll
        for (int u = 0; u < PER_LANE; ++u) {
            const int i = w0 + u * kWave + lane, j = (int)threadIdx.x + u * kSelThreads;
            nxt[u] = more && i < w1 ? aln[s_pos[i]] : 0.f;
            nxt_new[u] = more && j < L ? aln[new0 + j] : 0.f;
        }
        uint32_t Tk = 0, want = 0, gt = 0, eq = 0;
        uint32_t kv[PER_LANE];
        int32_t pv[PER_LANE];
        if (k > 0) {
            msd_select<kSelThreads, 2>([&](int i, bool& valid) { valid = true; return s_key[i]; }, budget, (uint32_t)k, s_hist,
                                       base, diff, &Tk, &want);
#pragma unroll
            for (int u = 0; u < PER_LANE; ++u) {
                const int i = w0 + u * kWave + lane;
                const bool live = i < w1;
                kv[u] = live ? s_key[i] : 0u;
                pv[u] = live ? s_pos[i] : 0;
                gt += (uint32_t)__popcll(__ballot(live && kv[u] > Tk));
                eq += (uint32_t)__popcll(__ballot(live && kv[u] == Tk));
            }
            if (lane == 0) {
                s_wtot[2 * wave] = gt;
                s_wtot[2 * wave + 1] = eq;
            }
        }
        __syncthreads();  // every source is in registers, the counts are visible, the histograms have been read
        s_hist[threadIdx.x] = 0;
        spread = 0;
        if (k > 0) {
            uint32_t gt_run = 0, eq_run = 0;
            for (int w = 0; w < wave; ++w) {
                gt_run += s_wtot[2 * w];
                eq_run += s_wtot[2 * w + 1];
            }
#pragma unroll
            for (int u = 0; u < PER_LANE; ++u) {
                const int i = w0 + u * kWave + lane;
                const bool live = i < w1;
                const unsigned long long mg = __ballot(live && kv[u] > Tk), me = __ballot(live && kv[u] == Tk);
                const uint32_t gb = gt_run + __builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, 0));
                const uint32_t eb = eq_run + __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0));
                const bool keep = live && (kv[u] > Tk || (kv[u] == Tk && eb < want));
                if (keep) {
                    const uint32_t dst = gb + min(eb, want);
                    const uint32_t key = score_key(nxt[u]);
                    s_pos[dst] = pv[u];
                    s_key[dst] = key;
                    spread |= key ^ base_next;
                    out[dst] = pv[u];
                }
                gt_run += (uint32_t)__popcll(mg);
                eq_run += (uint32_t)__popcll(me);
            }
        }
        // the L newest stay; then the L pairs generated before the next step join
#pragma unroll
        for (int u = 0; u < PER_LANE; ++u) {
            const int j = (int)threadIdx.x + u * kSelThreads;
            if (j < L) {
                out[k + j] = new0 + j;
                s_pos[k + j] = new0 + j;
                const uint32_t key = score_key(nxt_new[u]);
                s_key[k + j] = key;
                spread |= key ^ base_next;
                s_pos[k + L + j] = new0 + L + j;
            }
        }
        spread = wave_or(spread);
        if (lane == 0) s_wor[wave] = spread;
        base = base_next;
        __syncthreads();
    }
}

static int golden_steps(int T, int B, int L) {
    const int m = (T - B + L - 1) / L - 1;
    return m < 0 ? 0 : m;
}

}  // namespace fk

using namespace fk;

extern "C" int32_t fk_golden_steps(int32_t T, int32_t budget, int32_t interval) {
    if (T <= 0 || budget <= 0 || interval <= 0 || interval > budget) return -1;
    return golden_steps(T, budget, interval);
}

extern "C" fk_status fk_golden_scores(const void* A, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t T,
                                      int64_t ld, int32_t budget, int32_t interval, float* block_scores, float* alpha,
                                      void* stream) {
    if (!A || !block_scores || !alpha) return FK_ERR_INVALID_ARG;
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || T <= 0 || ld < T) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || interval <= 0 || interval > budget) return FK_ERR_INVALID_ARG;
    if (dtype != FK_F32 && dtype != FK_BF16) return FK_ERR_UNSUPPORTED;
    if (ld % 8 != 0 || !aligned16(A)) return FK_ERR_INVALID_ARG;
    const int M = golden_steps(T, budget, interval);
    if (M == 0) return FK_OK;
    if (M > 65535 || n_kv_heads > 65535) return FK_ERR_UNSUPPORTED;
    const int g = n_q_heads / n_kv_heads;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == FK_F32) {
        const int KT = 64;
        hipLaunchKernelGGL(golden_pool_kernel<float>, dim3((T + KT - 1) / KT, M, n_kv_heads), dim3(kPoolThreads), 0, st,
                           (const float*)A, g, T, (size_t)ld, budget, interval, M, block_scores);
    } else {
        const int KT = 128;
        hipLaunchKernelGGL(golden_pool_kernel<bf16_t>, dim3((T + KT - 1) / KT, M, n_kv_heads), dim3(kPoolThreads), 0, st,
                           (const bf16_t*)A, g, T, (size_t)ld, budget, interval, M, block_scores);
    }
    hipLaunchKernelGGL(golden_future_kernel, dim3((T + 255) / 256, n_kv_heads), dim3(256), 0, st, block_scores, T, M, alpha);
    return launch_status();
}

extern "C" fk_status fk_golden_trace(const float* alpha, int32_t n_kv_heads, int32_t T, int32_t budget, int32_t interval,
                                     int32_t* kept, void* stream) {
    if (!alpha || !kept) return FK_ERR_INVALID_ARG;
    if (n_kv_heads <= 0 || T <= 0 || budget <= 0 || interval <= 0 || interval > budget) return FK_ERR_INVALID_ARG;
    if (budget + interval > kTraceMaxCache) return FK_ERR_UNSUPPORTED;
    const int M = golden_steps(T, budget, interval);
    if (M == 0) return FK_OK;
    const size_t lds = sizeof(int32_t) * ((size_t)budget + interval) + sizeof(uint32_t) * (size_t)budget;
    // candidates per lane: a wavefront's stretch is the budget over the 16 wavefronts, rounded up to whole 64s
    const int per_lane = ((budget + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave;
    auto launch = [&](auto kern, bool (&lds_ok)[kMaxDevices]) -> fk_status {
        if (!allow_dynamic_lds((const void*)kern, sizeof(int32_t) * 2 * kTraceMaxCache, lds_ok)) return FK_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(n_kv_heads), dim3(kSelThreads), lds, (hipStream_t)stream, alpha, T, M, budget, interval,
                           kept);
        return launch_status();
    };
    static bool ok2[kMaxDevices] = {}, ok4[kMaxDevices] = {}, ok12[kMaxDevices] = {};
    if (per_lane <= 2) return launch(golden_trace_kernel<2>, ok2);
    if (per_lane <= 4) return launch(golden_trace_kernel<4>, ok4);
    return launch(golden_trace_kernel<12>, ok12);   // budget + interval <= kTraceMaxCache: at most 12
}
