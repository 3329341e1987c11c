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
// M steps with the radix select of fk_select_keep on keys gathered into LDS.
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

static constexpr int kTraceMaxCache = 12288;  // B + L positions (48 KB) + B keys in LDS

// one workgroup per KV group; the cache (positions, ascending) lives in LDS
__global__ __launch_bounds__(kSelThreads) void golden_trace_kernel(const float* __restrict__ alpha, int Tn, int M,
                                                                   int budget, int L, int32_t* __restrict__ kept) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t* s_pos = reinterpret_cast<int32_t*>(smem);                 // [budget + L]
    uint32_t* s_key = reinterpret_cast<uint32_t*>(s_pos + budget + L);  // [budget]
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_sel[2];
    __shared__ unsigned long long s_part[kSelWaves];
    const int hp = blockIdx.x;
    const int k = budget - L;  // old pairs that stay
    for (int j = threadIdx.x; j < budget + L; j += kSelThreads) s_pos[j] = j;
    __syncthreads();
    for (int t = 1; t <= M; ++t) {
        const float* al = alpha + ((size_t)hp * M + (t - 1)) * Tn;
        int32_t* out = kept + ((size_t)hp * M + (t - 1)) * budget;
        for (int j = threadIdx.x; j < budget; j += kSelThreads) s_key[j] = score_key(al[s_pos[j]]);
        __syncthreads();
        uint32_t Tk = 0, want = 0;
        if (k > 0)
            radix_threshold(budget, (uint32_t)k, [&](int i, bool& valid) { valid = true; return s_key[i]; }, s_hist, s_sel,
                            &Tk, &want);
        // ordered pass: survivors move to the front of the cache, in order (destination <= source, and every
        // source of a chunk is read before the barriers inside the scan, so the move is safe in place)
        uint32_t gt_base = 0, eq_base = 0;
        for (int base = 0; base < budget; base += kSelThreads) {
            const int i = base + threadIdx.x;
            uint32_t gt = 0, eq = 0;
            int32_t p = 0;
            if (i < budget && k > 0) {
                const uint32_t key = s_key[i];
                gt = key > Tk;
                eq = key == Tk;
                p = s_pos[i];
            }
            unsigned long long tot;
            const unsigned long long incl = block_scan_incl(((unsigned long long)gt << 32) | eq, s_part, &tot);
            const uint32_t gt_before = gt_base + (uint32_t)(incl >> 32) - gt;
            const uint32_t eq_before = eq_base + (uint32_t)(incl & 0xffffffffu) - eq;
            if (gt || (eq && eq_before < want)) {
                const uint32_t dst = gt_before + min(eq_before, want);
                s_pos[dst] = p;
                out[dst] = p;
            }
            gt_base += (uint32_t)(tot >> 32);
            eq_base += (uint32_t)(tot & 0xffffffffu);
        }
        __syncthreads();
        // the L newest stay; then the L pairs generated before the next step join
        for (int j = threadIdx.x; j < L; j += kSelThreads) {
            const int32_t p = budget + t * L - L + j;
            out[k + j] = p;
        }
        for (int j = threadIdx.x; j < 2 * L; j += kSelThreads) s_pos[k + j] = budget + t * L - L + j;
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
    static bool lds_ok[kMaxDevices] = {};
    if (!allow_dynamic_lds((const void*)golden_trace_kernel, sizeof(int32_t) * 2 * kTraceMaxCache, lds_ok)) return FK_ERR_LAUNCH;
    hipLaunchKernelGGL(golden_trace_kernel, dim3(n_kv_heads), dim3(kSelThreads), lds, (hipStream_t)stream, alpha, T, M,
                       budget, interval, kept);
    return launch_status();
}
