// fk_decode_attn: split-K flash-decode attention over the retained set
// (Appendix A, "Problem Setup": o_hat = sum_{i in S} softmax_S(s)_i v_i).
//
// A row (sequence, KV head) is cut into splits of `split_len` keys; one workgroup of four
// wavefronts handles one split for all g query heads of the group, so K and V are fetched
// from HBM once per group.  A row of K or V is D*sizeof(T) bytes = LPK lanes x 16 bytes; a
// wavefront load instruction therefore covers 64/LPK consecutive keys, fully coalesced.
// Every aligned group of LPK lanes runs its own online softmax over the keys it sees
// (running maximum m, running sum l, un-normalised accumulator acc for its 16-byte slice
// of D); the groups of a wavefront, the wavefronts of a workgroup and finally the splits
// of a row are merged with the log-sum-exp rule.
#include "fk_common.h"

namespace fk {

static constexpr int kAttnThreads = 256;
static constexpr int kAttnWaves = kAttnThreads / kWave;
static constexpr float kNegBig = -1.0e30f;  // "no key seen yet"; exp2(kNegBig - m) == 0

struct AttnPlan {
    int split_len;  // keys per split (multiple of the workgroup tile)
    int nsplit;     // splits per row
};

// Keys per workgroup iteration: 4 waves x (64/LPK) keys x U loads in flight.
template <typename T, int D> struct AttnGeom {
    static constexpr int LPK = D * (int)sizeof(T) / 16;  // lanes per key
    static constexpr int KPW = kWave / LPK;              // keys per wave load
    static constexpr int U = 4;                          // loads in flight per lane (K and V each)
    static constexpr int TILE = kAttnWaves * KPW * U;    // keys per workgroup iteration
    static constexpr int EPL = Vec16<T>::N;              // elements per lane
};

static AttnPlan attn_plan(const fk_cache_desc* d, int max_len) {
    const int rows = d->batch * d->n_kv_heads;
    const int lpk = d->head_dim * (d->dtype == FK_F32 ? 4 : 2) / 16;
    const int tile = kAttnWaves * (kWave / lpk) * 4;
    const int target_blocks = 256 * 8;  // a few workgroups per CU in flight
    int want = (target_blocks + rows - 1) / rows;
    int max_split = (max_len + tile - 1) / tile;
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    int split_len = (max_len + want - 1) / want;
    split_len = (split_len + tile - 1) / tile * tile;
    AttnPlan p;
    p.split_len = split_len;
    p.nsplit = (max_len + split_len - 1) / split_len;
    if (p.nsplit < 1) p.nsplit = 1;
    return p;
}

// partial record per (row, split, head): acc[D], m, l
template <typename T, int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ len, float scale_log2e, int n_kv, int cap, int split_len,
    int nsplit, float* __restrict__ ws) {
    using Gm = AttnGeom<T, D>;
    constexpr int LPK = Gm::LPK, KPW = Gm::KPW, U = Gm::U, EPL = Gm::EPL;
    const int row = blockIdx.y;
    const int split = blockIdx.x;
    const int b = row / n_kv;
    const int n = min(len[b], cap);
    const int start = split * split_len;
    if (start >= n) return;
    const int end = min(start + split_len, n);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int kg = lane / LPK;   // key group inside the wave
    const int dl = lane % LPK;   // which 16-byte slice of the row

    // queries of the group, this lane's slice, pre-multiplied by scale*log2(e)
    float qf[G][EPL];
    {
        const int hkv = row % n_kv;
        const T* qrow = q + ((size_t)b * n_kv * G + (size_t)hkv * G) * D;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            uint4 r = *reinterpret_cast<const uint4*>(qrow + (size_t)h * D + dl * EPL);
            Vec16<T>::unpack(r, qf[h]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qf[h][e] *= scale_log2e;
        }
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    const uint4* Krow = reinterpret_cast<const uint4*>(K + (size_t)row * cap * D);
    const uint4* Vrow = reinterpret_cast<const uint4*>(V + (size_t)row * cap * D);

    for (int base = start + wave * (KPW * U); base < end; base += kAttnWaves * KPW * U) {
        uint4 kr[U], vr[U];
        int key[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            key[u] = base + u * KPW + kg;
            const int kc = min(key[u], end - 1);  // clamp: always a live slot of this split
            kr[u] = Krow[(size_t)kc * LPK + dl];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kc = min(key[u], end - 1);
            vr[u] = Vrow[(size_t)kc * LPK + dl];
        }
        float s[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
            Vec16<T>::unpack(kr[u], kf);
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qf[h][e], kf[e], d);
                d = group_sum<LPK>(d);
                s[u][h] = key[u] < end ? d : kNegBig;
            }
        }
        float p[U][G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float mn = m[h];
#pragma unroll
            for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][h]);
            const float corr = exp2f(m[h] - mn);
            float ps = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[u][h] = key[u] < end ? exp2f(s[u][h] - mn) : 0.f;
                ps += p[u][h];
            }
            l[h] = l[h] * corr + ps;
            m[h] = mn;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] *= corr;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[EPL];
            Vec16<T>::unpack(vr[u], vf);
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(p[u][h], vf[e], acc[h][e]);
        }
    }

    // merge the key groups of the wave (lanes that hold the same slice of D)
#pragma unroll
    for (int off = LPK; off < kWave; off <<= 1) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float mo = __shfl_xor(m[h], off);
            const float lo = __shfl_xor(l[h], off);
            const float mn = fmaxf(m[h], mo);
            const float ca = exp2f(m[h] - mn), cb = exp2f(mo - mn);
            l[h] = l[h] * ca + lo * cb;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float ao = __shfl_xor(acc[h][e], off);
                acc[h][e] = acc[h][e] * ca + ao * cb;
            }
            m[h] = mn;
        }
    }

    // merge the four waves through LDS
    __shared__ float s_acc[kAttnWaves][G][D];
    __shared__ float s_m[kAttnWaves][G];
    __shared__ float s_l[kAttnWaves][G];
    if (kg == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) s_acc[wave][h][dl * EPL + e] = acc[h][e];
            if (dl == 0) {
                s_m[wave][h] = m[h];
                s_l[wave][h] = l[h];
            }
        }
    }
    __syncthreads();
    float* rec = ws + ((size_t)row * nsplit + split) * G * (D + 2);
    for (int idx = threadIdx.x; idx < G * D; idx += kAttnThreads) {
        const int h = idx / D, d = idx % D;
        float mn = s_m[0][h];
#pragma unroll
        for (int w = 1; w < kAttnWaves; ++w) mn = fmaxf(mn, s_m[w][h]);
        float a = 0.f, ls = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float c = exp2f(s_m[w][h] - mn);
            a += s_acc[w][h][d] * c;
            ls += s_l[w][h] * c;
        }
        rec[(size_t)h * (D + 2) + d] = a;
        if (d == 0) {
            rec[(size_t)h * (D + 2) + D] = mn;
            rec[(size_t)h * (D + 2) + D + 1] = ls;
        }
    }
}

// out[b][hq][d] = sum_s acc_s[d] 2^(m_s - m*) / sum_s l_s 2^(m_s - m*)
template <typename T, int D, int G>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ ws,
                                                        const int32_t* __restrict__ len, int n_kv,
                                                        int cap, int split_len, int nsplit,
                                                        T* __restrict__ out) {
    const int row = blockIdx.x / G, h = blockIdx.x % G;
    const int b = row / n_kv, hkv = row % n_kv;
    const int d = threadIdx.x;
    const int n = min(len[b], cap);
    T* o = out + (((size_t)b * n_kv + hkv) * G + h) * D;
    if (n <= 0) {
        store_out(o + d, 0.f);
        return;
    }
    const int used = (n + split_len - 1) / split_len;
    const float* rec = ws + (size_t)row * nsplit * G * (D + 2) + (size_t)h * (D + 2);
    const size_t stride = (size_t)G * (D + 2);
    float mn = kNegBig;
    for (int s = 0; s < used; ++s) mn = fmaxf(mn, rec[s * stride + D]);
    float a = 0.f, ls = 0.f;
    for (int s = 0; s < used; ++s) {
        const float c = exp2f(rec[s * stride + D] - mn);
        a += rec[s * stride + d] * c;
        ls += rec[s * stride + D + 1] * c;
    }
    store_out(o + d, a / ls);
}

template <typename T, int D, int G>
static fk_status attn_launch(const fk_cache_desc* d, const void* q, const void* K, const void* V,
                             const int32_t* len, int max_len, float scale, void* out, float* ws,
                             hipStream_t st) {
    const AttnPlan p = attn_plan(d, max_len);
    const int rows = d->batch * d->n_kv_heads;
    const float scale_log2e = scale * 1.4426950408889634f;
    dim3 grid(p.nsplit, rows);
    hipLaunchKernelGGL((attn_partial_kernel<T, D, G>), grid, dim3(kAttnThreads), 0, st,
                       (const T*)q, (const T*)K, (const T*)V, len, scale_log2e, d->n_kv_heads,
                       d->capacity, p.split_len, p.nsplit, ws);
    hipLaunchKernelGGL((attn_combine_kernel<T, D, G>), dim3(rows * G), dim3(D), 0, st, ws, len,
                       d->n_kv_heads, d->capacity, p.split_len, p.nsplit, (T*)out);
    return launch_status();
}

template <typename T, int D>
static fk_status attn_dispatch_g(int g, const fk_cache_desc* d, const void* q, const void* K,
                                 const void* V, const int32_t* len, int max_len, float scale,
                                 void* out, float* ws, hipStream_t st) {
    switch (g) {
        case 1: return attn_launch<T, D, 1>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 2: return attn_launch<T, D, 2>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 3: return attn_launch<T, D, 3>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 4: return attn_launch<T, D, 4>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 5: return attn_launch<T, D, 5>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 6: return attn_launch<T, D, 6>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 7: return attn_launch<T, D, 7>(d, q, K, V, len, max_len, scale, out, ws, st);
        case 8: return attn_launch<T, D, 8>(d, q, K, V, len, max_len, scale, out, ws, st);
    }
    return FK_ERR_UNSUPPORTED;
}

}  // namespace fk

using namespace fk;

extern "C" size_t fk_decode_attn_workspace(const fk_cache_desc* desc, int32_t max_len) {
    if (check_desc(desc) != FK_OK || max_len <= 0 || max_len > desc->capacity) return 0;
    const AttnPlan p = attn_plan(desc, max_len);
    const size_t g = desc->n_q_heads / desc->n_kv_heads;
    return (size_t)desc->batch * desc->n_kv_heads * p.nsplit * g * (desc->head_dim + 2) * sizeof(float);
}

extern "C" fk_status fk_decode_attn(const fk_cache_desc* desc, const void* q, const void* K,
                                    const void* V, const int32_t* len, int32_t max_len,
                                    float softmax_scale, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!q || !K || !V || !len || !out) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out)) return FK_ERR_INVALID_ARG;
    const size_t need = fk_decode_attn_workspace(desc, max_len);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return FK_ERR_WORKSPACE;
    const int g = desc->n_q_heads / desc->n_kv_heads;
    hipStream_t st = (hipStream_t)stream;
    float* ws = (float*)workspace;
    if (desc->dtype == FK_F32) {
        if (desc->head_dim == 64) return attn_dispatch_g<float, 64>(g, desc, q, K, V, len, max_len, softmax_scale, out, ws, st);
        return attn_dispatch_g<float, 128>(g, desc, q, K, V, len, max_len, softmax_scale, out, ws, st);
    }
    if (desc->head_dim == 64) return attn_dispatch_g<bf16_t, 64>(g, desc, q, K, V, len, max_len, softmax_scale, out, ws, st);
    return attn_dispatch_g<bf16_t, 128>(g, desc, q, K, V, len, max_len, softmax_scale, out, ws, st);
}
