// fk_score_kv: the MLP scorer of Appendix B.1 on x = concat(k, v):
//   phi = sum_j gelu(sum_f x_f W1[f][j] + b1[j]) W2[j] + b2          (gelu: exact erf form)
//
// bf16 path.  The contraction [hidden x F] . [F x pairs] runs on the matrix cores with
// v_mfma_f32_32x32x16_bf16, hidden units as the M dimension and pairs as the N dimension:
//   A operand = W1^T tile (lane: hidden j = lane%32, 8 consecutive features), read from LDS
//               where the workgroup keeps the whole transposed W1 of its KV head;
//   B operand = X^T tile (lane: pair = lane%32, 8 consecutive features) = 16 contiguous bytes
//               of the pair's K row (features < D) or V row (features >= D), loaded straight
//               from the cache into registers once and reused for every hidden tile;
//   C tile    = lane holds 16 hidden units of ONE pair, so bias, gelu, the W2 dot and the
//               reduction over the hidden dimension stay in registers (one cross-half add).
// fp32 path: plain fp32 FMA (the fp32 matrix rate equals the vector rate on this chip).
#include "fk_common.h"

namespace fk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

static constexpr int kScoreThreads = 1024;  // four wavefronts per SIMD: MFMAs of one overlap the gelu of the others
static constexpr int kScoreWaves = kScoreThreads / kWave;
static constexpr int kWPad = 8;  // bf16 elements of padding per transposed W1 row in LDS

// gelu(z) = z Phi(z) = 0.5 z + 0.5 |z| erf(|z| / sqrt 2), erf by the Abramowitz-Stegun rational
// form 7.1.26 (|error| < 1.5e-7 on erf, < 5e-7 on gelu): one reciprocal, one exp2, 9 FMA/mul.
// The scorer's epilogue is bound by this function, not by the MFMAs.
__device__ __forceinline__ float gelu_erf(float z) {
    const float az = fabsf(z);
    const float u = az * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, u, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(-(u * u) * 1.4426950408889634f);
    const float erf_abs = fmaf(-p, e, 1.0f);
    return fmaf(0.5f * az, erf_abs, 0.5f * z);
}

// reference-accuracy form for the fp32 path
__device__ __forceinline__ float gelu_erf_precise(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }

union B128 {
    uint4 u;
    bf16x8_t v;
};

// LDS: Wt [H][F + kWPad] bf16 | b1 [H] f32 | w2 [H] f32
template <int D, int NT>
__global__ __launch_bounds__(kScoreThreads) void score_mfma_kernel(
    const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const int32_t* __restrict__ len,
    const bf16_t* __restrict__ W1, const float* __restrict__ b1, const float* __restrict__ W2,
    const float* __restrict__ b2, int H, int per_head, int n_kv, int cap, int pairs_per_block,
    float* __restrict__ scores) {
    constexpr int F = 2 * D;
    constexpr int FS = F + kWPad;  // LDS row stride in bf16 elements
    constexpr int KS = F / 16;     // k-steps of 16 features
    const int row = blockIdx.y;
    const int hkv = row % n_kv;
    const int n = min(len[row], cap);
    const int p_begin = blockIdx.x * pairs_per_block;
    if (p_begin >= n) return;
    const int p_end = min(p_begin + pairs_per_block, n);
    const int hw = per_head ? hkv : 0;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* s_wt = reinterpret_cast<bf16_t*>(smem);
    float* s_b1 = reinterpret_cast<float*>(smem + (size_t)H * FS * sizeof(bf16_t));
    float* s_w2 = s_b1 + H;

    // stage W1^T: a thread takes two consecutive features f, f+1 and 8 consecutive hidden
    // units, and writes 8 dwords (W1[f][j], W1[f+1][j]) to Wt[j][f..f+1]; consecutive lanes
    // take consecutive feature pairs, so the dword writes of a wave are conflict free
    {
        const bf16_t* w = W1 + (size_t)hw * F * H;
        const int jchunks = H / 8;
        for (int t = threadIdx.x; t < (F / 2) * jchunks; t += kScoreThreads) {
            const int fp = t % (F / 2), jc = t / (F / 2);
            const uint4 r0 = *reinterpret_cast<const uint4*>(w + (size_t)(2 * fp) * H + jc * 8);
            const uint4 r1 = *reinterpret_cast<const uint4*>(w + (size_t)(2 * fp + 1) * H + jc * 8);
            const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w}, c[4] = {r1.x, r1.y, r1.z, r1.w};
            uint32_t* dst = reinterpret_cast<uint32_t*>(s_wt);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = (a[e] & 0xffffu) | (c[e] << 16);          // hidden jc*8 + 2e
                const uint32_t hi = (a[e] >> 16) | (c[e] & 0xffff0000u);      // hidden jc*8 + 2e + 1
                dst[((size_t)(jc * 8 + 2 * e) * FS + 2 * fp) / 2] = lo;
                dst[((size_t)(jc * 8 + 2 * e + 1) * FS + 2 * fp) / 2] = hi;
            }
        }
        for (int j = threadIdx.x; j < H; j += kScoreThreads) {
            s_b1[j] = b1[(size_t)hw * H + j];
            s_w2[j] = W2[(size_t)hw * H + j];
        }
    }
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int l32 = lane & 31, half = lane >> 5;
    const float bias2 = b2[hw];
    const bf16_t* Krow = K + (size_t)row * cap * D;
    const bf16_t* Vrow = V + (size_t)row * cap * D;
    float* srow = scores + (size_t)row * cap;

    for (int base = p_begin + wave * (32 * NT); base < p_end; base += kScoreWaves * 32 * NT) {
        // B operands: the pair's features, 16 bytes per k-step
        B128 xk[NT][KS];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int p = min(base + t * 32 + l32, p_end - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int f = ks * 16 + half * 8;
                const bf16_t* src = f < D ? Krow + (size_t)p * D + f : Vrow + (size_t)p * D + (f - D);
                xk[t][ks].u = *reinterpret_cast<const uint4*>(src);
            }
        }
        float phi[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) phi[t] = 0.f;

        for (int ht = 0; ht < H / 32; ++ht) {
            f32x16_t acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
            const bf16_t* wrow = s_wt + (size_t)(ht * 32 + l32) * FS + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                B128 a;
                a.u = *reinterpret_cast<const uint4*>(wrow + ks * 16);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, xk[t][ks].v, acc[t], 0, 0, 0);
            }
            // C layout: element i of a lane is hidden unit ht*32 + (i/4)*8 + half*4 + i%4
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int j = ht * 32 + i4 * 8 + half * 4;
                const float4 bb = *reinterpret_cast<const float4*>(s_b1 + j);
                const float4 ww = *reinterpret_cast<const float4*>(s_w2 + j);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 0] + bb.x), ww.x, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 1] + bb.y), ww.y, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 2] + bb.z), ww.z, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 3] + bb.w), ww.w, phi[t]);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float tot = phi[t] + __shfl_xor(phi[t], 32);
            const int p = base + t * 32 + l32;
            if (half == 0 && p < p_end) srow[p] = tot + bias2;
        }
    }
}

// fp32 (and fallback) path: one thread per pair, hidden units in chunks of 8, features
// accumulated in order.  T = float or bf16 storage.
template <typename T, int D>
__global__ __launch_bounds__(128) void score_simple_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                           const int32_t* __restrict__ len,
                                                           const T* __restrict__ W1, const float* __restrict__ b1,
                                                           const float* __restrict__ W2, const float* __restrict__ b2,
                                                           int H, int per_head, int n_kv, int cap,
                                                           float* __restrict__ scores) {
    constexpr int EPL = Vec16<T>::N;
    const int row = blockIdx.y;
    const int hkv = row % n_kv;
    const int n = min(len[row], cap);
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const int hw = per_head ? hkv : 0;
    const T* w = W1 + (size_t)hw * 2 * D * H;
    const T* krow = K + ((size_t)row * cap + p) * D;
    const T* vrow = V + ((size_t)row * cap + p) * D;
    float phi = 0.f;
    for (int j0 = 0; j0 < H; j0 += 8) {
        float z[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = 0.f;
        for (int half = 0; half < 2; ++half) {
            const T* xr = half == 0 ? krow : vrow;
            for (int c = 0; c < D / EPL; ++c) {
                float xf[EPL];
                Vec16<T>::unpack(*reinterpret_cast<const uint4*>(xr + c * EPL), xf);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    const int f = half * D + c * EPL + e;
                    const T* wr = w + (size_t)f * H + j0;
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj) {
                        if (j0 + jj < H) {
                            float wv;
                            if constexpr (sizeof(T) == 4) wv = wr[jj];
                            else wv = __uint_as_float(((uint32_t)wr[jj]) << 16);
                            z[jj] = fmaf(xf[e], wv, z[jj]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
            if (j0 + jj < H)
                phi = fmaf(gelu_erf_precise(z[jj] + b1[(size_t)hw * H + j0 + jj]), W2[(size_t)hw * H + j0 + jj], phi);
    }
    scores[(size_t)row * cap + p] = phi + b2[hw];
}

static size_t score_lds_bytes(int D, int H) { return (size_t)H * (2 * D + kWPad) * 2 + (size_t)H * 8; }

template <int D>
static fk_status score_mfma_launch(const fk_cache_desc* d, const void* K, const void* V, const int32_t* len,
                                   int max_len, const fk_scorer* sc, float* scores, hipStream_t st) {
    constexpr int NT = 1;
    const int rows = d->batch * d->n_kv_heads;
    const size_t lds = score_lds_bytes(D, sc->hidden);
    // pairs per workgroup: fill the chip about once, in whole wave tiles
    const int tile = 32 * NT;  // the waves of a workgroup take tiles round robin
    int chunks = (256 + rows - 1) / rows;
    if (chunks < 1) chunks = 1;
    int ppb = (max_len + chunks - 1) / chunks;
    ppb = (ppb + tile - 1) / tile * tile;
    chunks = (max_len + ppb - 1) / ppb;
    auto kern = score_mfma_kernel<D, NT>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return FK_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(chunks, rows), dim3(kScoreThreads), lds, st, (const bf16_t*)K,
                       (const bf16_t*)V, len, (const bf16_t*)sc->w1, sc->b1, sc->w2, sc->b2, sc->hidden,
                       sc->per_head, d->n_kv_heads, d->capacity, ppb, scores);
    return launch_status();
}

template <typename T, int D>
static fk_status score_simple_launch(const fk_cache_desc* d, const void* K, const void* V, const int32_t* len,
                                     int max_len, const fk_scorer* sc, float* scores, hipStream_t st) {
    const int rows = d->batch * d->n_kv_heads;
    hipLaunchKernelGGL((score_simple_kernel<T, D>), dim3((max_len + 127) / 128, rows), dim3(128), 0, st,
                       (const T*)K, (const T*)V, len, (const T*)sc->w1, sc->b1, sc->w2, sc->b2, sc->hidden,
                       sc->per_head, d->n_kv_heads, d->capacity, scores);
    return launch_status();
}

}  // namespace fk

using namespace fk;

extern "C" fk_status fk_score_kv(const fk_cache_desc* desc, const void* K, const void* V, const int32_t* len,
                                 int32_t max_len, const fk_scorer* scorer, float* scores, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !len || !scorer || !scores) return FK_ERR_INVALID_ARG;
    if (!scorer->w1 || !scorer->b1 || !scorer->w2 || !scorer->b2 || scorer->hidden <= 0) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(scorer->w1)) return FK_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int D = desc->head_dim, H = scorer->hidden;
    if (desc->dtype == FK_F32) {
        if (D == 64) return score_simple_launch<float, 64>(desc, K, V, len, max_len, scorer, scores, st);
        return score_simple_launch<float, 128>(desc, K, V, len, max_len, scorer, scores, st);
    }
    const bool mfma_ok = (H % 32 == 0) && score_lds_bytes(D, H) <= 160 * 1024;
    if (!mfma_ok) return FK_ERR_UNSUPPORTED;
    if (D == 64) return score_mfma_launch<64>(desc, K, V, len, max_len, scorer, scores, st);
    return score_mfma_launch<128>(desc, K, V, len, max_len, scorer, scores, st);
}
