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
//
// fk_score_kv_feat: x = concat(k, v, a) with the 6 g attention features of the pair (Appendix B.1).
// The features are fp32 state; each is split into a bf16 head and a bf16 remainder (x = hi + lo, 16
// significant bits) and both parts are multiplied with the same W1^T tile, so the contraction stays
// on the matrix cores without rounding the features to 8 bits.
#include "fk_common.h"

namespace fk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// NT pair tiles of a wavefront share every LDS read of a W1^T operand (1: with two, only 8 wavefronts fit the
// registers and the kernel is slower); 16 wavefronts per workgroup, the most the pair operands leave registers for
static constexpr int kScoreNT = 1;
static constexpr int kScoreThreads = 1024;
static constexpr int kScoreWaves = kScoreThreads / kWave;
static constexpr int kWPad = 8;  // bf16 elements of padding per transposed W1 row in LDS

// gelu(z) = z Phi(z) = max(z, 0) - |z| Phi(-|z|) with the lower normal tail as Phi(-a) = 2^P(a), P a quintic
// fitted to log2 Phi(-a) on a >= 0 (weighted minimax on the error of gelu; the leading coefficient is negative,
// so the tail keeps falling beyond the fitted range).  |error| <= 6.4e-7 on gelu over all finite z (checked against
// the erf form in double precision on a 1e-5 grid over [-40, 40]); five FMAs, one exp2, one integer max, one FMA.
// The scorer's epilogue is bound by this function, not by the MFMAs.
__device__ __forceinline__ float gelu_erf(float z) {
    const float a = fabsf(z);
    float p = fmaf(-4.733092552e-04f, a, 7.084556704e-03f);
    p = fmaf(p, a, -5.182738105e-02f);
    p = fmaf(p, a, -4.599924418e-01f);
    p = fmaf(p, a, -1.150787850e+00f);
    p = fmaf(p, a, -1.000037623e+00f);
    // max(z, 0) on the bit pattern: a float with its sign bit set is a negative integer.  One instruction; a float
    // max would get a canonicalising copy of z in front of it.
    const float zp = __int_as_float(max(__float_as_int(z), 0));
    return fmaf(-a, __builtin_amdgcn_exp2f(p), zp);
}

// reference-accuracy form for the fp32 path
__device__ __forceinline__ float gelu_erf_precise(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }

union B128 {
    uint4 u;
    bf16x8_t v;
};


// geometry of the feature part for group size GF (0: no features)
template <int D, int GF> struct ScoreCfg {
    static constexpr int A = kFeatPlanes * GF;       // attention features per pair
    static constexpr int KA = (A + 15) / 16;         // their k-steps of 16 (zero padded)
    static constexpr int F = 2 * D + A;              // rows of W1
    static constexpr int FP = 2 * D + 16 * KA;       // features after padding
    static constexpr int FS = FP + kWPad;            // LDS row stride in bf16 elements
    static constexpr int GP = GF <= 4 ? 4 : 8;       // heads per slot in the feature state
};

__device__ __forceinline__ uint32_t bf16_rn(float x) { return (__float_as_uint(x) + 0x7fffu + ((__float_as_uint(x) >> 16) & 1u)) >> 16; }

// LDS of the MFMA kernels: Wt [HP][FS] bf16 | b1 [HP] f32 | w2 [HP] f32
template <int D, int GF>
__device__ __forceinline__ void stage_w1t(const bf16_t* __restrict__ W1, const float* __restrict__ b1, const float* __restrict__ W2,
                                          int hw, int H, int HP, bf16_t* s_wt, float* s_b1, float* s_w2) {
    using SC = ScoreCfg<D, GF>;
    constexpr int F = SC::F;
    constexpr int FS = SC::FS;
    // stage W1^T: a thread takes two consecutive features f, f+1 and 8 consecutive hidden
    // units, and writes 8 dwords (W1[f][j], W1[f+1][j]) to Wt[j][f..f+1].  Four consecutive lanes take four
    // consecutive 16-byte chunks of the same two W1 rows (64 contiguous bytes per row: one request to the memory
    // pipeline instead of four, which is what bounds this phase), the next four lanes the next feature pair; the
    // dword writes of a wave then meet four ways on a bank, which costs less than the separate requests did
    // (staging alone: 4.2 -> 1.7 us).  Eight lanes per row with the columns of rows 8 apart XOR-swizzled onto
    // different banks stage in 0.9 us, but the swizzled operand reads cost more than that in the main loop.
    {
        const bf16_t* w = W1 + (size_t)hw * F * H;
        const int jchunks = H / 8;
        const int items = (F / 2) * ((jchunks + 3) / 4) * 4;
        for (int t = threadIdx.x; t < items; t += kScoreThreads) {
            const int jc = (t & 3) + 4 * (t / (4 * (F / 2))), fp = (t >> 2) % (F / 2);
            if (jc >= jchunks) continue;
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
        if constexpr (SC::FP > F) {  // zero the padding features (dwords: F is even)
            constexpr int padw = (SC::FP - F) / 2;
            for (int t = threadIdx.x; t < H * padw; t += kScoreThreads)
                reinterpret_cast<uint32_t*>(s_wt)[((size_t)(t / padw) * FS + F) / 2 + t % padw] = 0u;
        }
        for (int t = threadIdx.x; t < (HP - H) * (FS / 2); t += kScoreThreads)  // the padding hidden units
            reinterpret_cast<uint32_t*>(s_wt)[(size_t)H * (FS / 2) + t] = 0u;
        for (int j = threadIdx.x; j < HP; j += kScoreThreads) {
            s_b1[j] = j < H ? b1[(size_t)hw * H + j] : 0.f;
            s_w2[j] = j < H ? W2[(size_t)hw * H + j] : 0.f;
        }
    }
}

// LDS: Wt [H][FS] bf16 | b1 [H] f32 | w2 [H] f32
template <int D, int NT, int GF>
__global__ __launch_bounds__(kScoreThreads) void score_mfma_kernel(
    const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const float* __restrict__ feat,
    const int32_t* __restrict__ len,
    const bf16_t* __restrict__ W1, const float* __restrict__ b1, const float* __restrict__ W2,
    const float* __restrict__ b2, int H, int per_head, int skip_len, int n_kv, int cap, int pairs_per_block,
    float* __restrict__ scores) {
    using SC = ScoreCfg<D, GF>;
    constexpr int FS = SC::FS;     // LDS row stride in bf16 elements
    constexpr int KS = 2 * D / 16; // k-steps of 16 features over k and v
    constexpr int KA = SC::KA;
    const int row = blockIdx.y;
    const int hkv = row % n_kv;
    const int n = min(len[row], cap);
    const int p_begin = blockIdx.x * pairs_per_block;
    if (p_begin >= n || n <= skip_len) return;
    // the last workgroup of a row runs on to the row's end (a max_len hint below len[row] costs time, not scores)
    const int p_end = blockIdx.x == gridDim.x - 1 ? n : min(p_begin + pairs_per_block, n);
    const int hw = per_head ? hkv : 0;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* s_wt = reinterpret_cast<bf16_t*>(smem);
    const int HP = (H + 31) / 32 * 32;  // hidden units padded to whole MFMA tiles: zero weights, zero W2
    float* s_b1 = reinterpret_cast<float*>(smem + (size_t)HP * FS * sizeof(bf16_t));
    float* s_w2 = s_b1 + HP;

    stage_w1t<D, GF>(W1, b1, W2, hw, H, HP, s_wt, s_b1, s_w2);
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
        // attention features of the pair as two bf16 operands (head and remainder); feature
        // a = head * 6 + plane; the carried planes already include this chunk (cum + wL, 0.9 dec + wL)
        B128 xh[NT][KA > 0 ? KA : 1], xl[NT][KA > 0 ? KA : 1];
        if constexpr (GF > 0) {
            constexpr int GP = SC::GP;
            const float* frow = feat + (size_t)row * kFeatPlanes * cap * GP;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int p = min(base + t * 32 + l32, p_end - 1);
                float fv[GP][kFeatPlanes];
#pragma unroll
                for (int pl = 0; pl < kFeatPlanes; ++pl)
#pragma unroll
                    for (int q4 = 0; q4 < GP / 4; ++q4) {
                        const float4 v = *reinterpret_cast<const float4*>(frow + ((size_t)pl * cap + p) * GP + q4 * 4);
                        fv[q4 * 4 + 0][pl] = v.x;
                        fv[q4 * 4 + 1][pl] = v.y;
                        fv[q4 * 4 + 2][pl] = v.z;
                        fv[q4 * 4 + 3][pl] = v.w;
                    }
#pragma unroll
                for (int h = 0; h < GP; ++h) {
                    fv[h][4] = fv[h][4] + fv[h][3];
                    fv[h][5] = fmaf(kFeatDecay, fv[h][5], fv[h][3]);
                }
#pragma unroll
                for (int ka = 0; ka < KA; ++ka) {
                    uint32_t hi[8], lo[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int a0 = ka * 16 + e, a1 = ka * 16 + 8 + e;  // this lane's feature: a0 (half 0) or a1 (half 1)
                        const float v0 = a0 < SC::A ? fv[a0 / kFeatPlanes][a0 % kFeatPlanes] : 0.f;
                        const float v1 = a1 < SC::A ? fv[a1 / kFeatPlanes][a1 % kFeatPlanes] : 0.f;
                        const float x = half ? v1 : v0;
                        hi[e] = bf16_rn(x);
                        lo[e] = bf16_rn(x - __uint_as_float(hi[e] << 16));
                    }
                    xh[t][ka].u = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
                    xl[t][ka].u = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
                }
            }
        }
        float phi[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) phi[t] = 0.f;

        for (int ht = 0; ht < HP / 32; ++ht) {
            // C layout: element i of a lane is hidden unit ht*32 + (i/4)*8 + half*4 + i%4; the accumulators
            // start from the bias of their hidden unit
            f32x16_t acc[NT];
            float4 ww[4];
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int j = ht * 32 + i4 * 8 + half * 4;
                const float4 bb = *reinterpret_cast<const float4*>(s_b1 + j);
                ww[i4] = *reinterpret_cast<const float4*>(s_w2 + j);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    acc[t][i4 * 4 + 0] = bb.x;
                    acc[t][i4 * 4 + 1] = bb.y;
                    acc[t][i4 * 4 + 2] = bb.z;
                    acc[t][i4 * 4 + 3] = bb.w;
                }
            }
            const bf16_t* wrow = s_wt + (size_t)(ht * 32 + l32) * FS + half * 8;
            // the MFMA chain issues ahead of the other wavefronts' gelu instructions (measured: 51.8 -> 50.0 us per event)
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                B128 a;
                a.u = *reinterpret_cast<const uint4*>(wrow + ks * 16);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, xk[t][ks].v, acc[t], 0, 0, 0);
            }
            if constexpr (GF > 0) {
#pragma unroll
                for (int ka = 0; ka < KA; ++ka) {
                    B128 a;
                    a.u = *reinterpret_cast<const uint4*>(wrow + (KS + ka) * 16);
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, xh[t][ka].v, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, xl[t][ka].v, acc[t], 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 0]), ww[i4].x, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 1]), ww[i4].y, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 2]), ww[i4].z, phi[t]);
                    phi[t] = fmaf(gelu_erf(acc[t][i4 * 4 + 3]), ww[i4].w, phi[t]);
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

// fp32 path.  A wavefront scores four pairs: their inputs x (k, v and, with features, a) are staged in LDS as
// fp32; lane j owns the hidden units j, j + 64, ...; for every input feature the lane's W1 element (coalesced
// over the lanes, shared by the four pairs) meets the four x values (LDS broadcasts).  Features are
// accumulated in order, the hidden units are reduced over the wavefront in a fixed order.
static constexpr int kSimpleWaves = 4;  // wavefronts per workgroup
static constexpr int kSimplePairs = 4;  // pairs per wavefront

template <typename T, int D>
__global__ __launch_bounds__(kSimpleWaves * kWave) void score_simple_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const float* __restrict__ feat, int g,
    const int32_t* __restrict__ len, const T* __restrict__ W1, const float* __restrict__ b1,
    const float* __restrict__ W2, const float* __restrict__ b2, int H, int per_head, int skip_len, int n_kv, int cap,
    float* __restrict__ scores) {
    constexpr int PP = kSimplePairs;
    extern __shared__ __attribute__((aligned(16))) float s_x[];  // [waves][PP][F]
    const int row = blockIdx.y;
    const int hkv = row % n_kv;
    const int n = min(len[row], cap);
    if (n <= skip_len) return;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int hw = per_head ? hkv : 0;
    const int A = feat ? kFeatPlanes * g : 0;  // attention features behind k and v
    const int F = 2 * D + A;
    const int GP = g <= 4 ? 4 : 8;
    const T* w = W1 + (size_t)hw * F * H;
    auto widen = [](const T* ptr) -> float {
        if constexpr (sizeof(T) == 4) return *ptr;
        else return __uint_as_float(((uint32_t)*ptr) << 16);
    };
    float* x = s_x + (size_t)wave * PP * F;
    const float bias2 = b2[hw];
    // the grid covers max_len pairs; rows longer than that are finished by further rounds of the same workgroups
    for (int pb = blockIdx.x * kSimpleWaves * PP; pb < n; pb += gridDim.x * kSimpleWaves * PP) {
        const int p0 = pb + wave * PP;
        if (p0 < n) {
            for (int p = 0; p < PP; ++p) {
                const int pair = min(p0 + p, n - 1);
                const T* krow = K + ((size_t)row * cap + pair) * D;
                const T* vrow = V + ((size_t)row * cap + pair) * D;
                for (int f = lane; f < 2 * D; f += kWave) x[p * F + f] = f < D ? widen(krow + f) : widen(vrow + f - D);
                for (int a = lane; a < A; a += kWave) {  // feature a = head * 6 + plane; carried planes include this chunk
                    const int head = a / kFeatPlanes, pl = a % kFeatPlanes;
                    const float* fp = feat + (size_t)row * kFeatPlanes * cap * GP + (size_t)pair * GP + head;
                    const size_t plane = (size_t)cap * GP;
                    float v = fp[pl * plane];
                    if (pl == 4) v += fp[3 * plane];
                    if (pl == 5) v = fmaf(kFeatDecay, v, fp[3 * plane]);
                    x[p * F + 2 * D + a] = v;
                }
            }
        }
        __syncthreads();
        if (p0 < n) {
            float phi[PP];
#pragma unroll
            for (int p = 0; p < PP; ++p) phi[p] = 0.f;
            for (int j = lane; j < (H + kWave - 1) / kWave * kWave; j += kWave) {
                const bool live = j < H;
                const T* wj = w + (live ? j : 0);
                float z[PP];
#pragma unroll
                for (int p = 0; p < PP; ++p) z[p] = 0.f;
                for (int f = 0; f < F; ++f) {
                    const float wv = widen(wj + (size_t)f * H);
#pragma unroll
                    for (int p = 0; p < PP; ++p) z[p] = fmaf(x[p * F + f], wv, z[p]);
                }
                if (live) {
                    const float bb = b1[(size_t)hw * H + j], ww = W2[(size_t)hw * H + j];
#pragma unroll
                    for (int p = 0; p < PP; ++p) phi[p] = fmaf(gelu_erf_precise(z[p] + bb), ww, phi[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < PP; ++p) {
                const float tot = group_sum<64>(phi[p]);
                if (lane == 0 && p0 + p < n) scores[(size_t)row * cap + p0 + p] = tot + bias2;
            }
        }
        __syncthreads();  // the staged inputs are free for the next round
    }
}

// LDS of the MFMA kernel for group size gf of the feature part (0: no features)
static size_t score_lds_bytes(int D, int H, int gf = 0) {
    const int fp = 2 * D + (kFeatPlanes * gf + 15) / 16 * 16;
    const int hp = (H + 31) / 32 * 32;
    return (size_t)hp * (fp + kWPad) * 2 + (size_t)hp * 8;
}

template <int D, int GF>
static fk_status score_mfma_launch(const fk_cache_desc* d, const void* K, const void* V, const float* feat,
                                   const int32_t* len, int max_len, const fk_scorer* sc, float* scores, hipStream_t st) {
    constexpr int NT = kScoreNT;
    const int rows = d->batch * d->n_kv_heads;
    const size_t lds = score_lds_bytes(D, sc->hidden, GF);
    // pairs per workgroup: fill the chip about once, in whole wave tiles
    const int tile = 32 * NT;  // the waves of a workgroup take tiles round robin
    int chunks = (256 + rows - 1) / rows;
    if (chunks < 1) chunks = 1;
    int ppb = (max_len + chunks - 1) / chunks;
    ppb = (ppb + tile - 1) / tile * tile;
    chunks = (max_len + ppb - 1) / ppb;
    auto kern = score_mfma_kernel<D, NT, GF>;
    static bool lds_ok[kMaxDevices] = {};  // per template instantiation; the limit covers every hidden width it admits
    if (!allow_dynamic_lds((const void*)kern, 160 * 1024, lds_ok)) return FK_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(chunks, rows), dim3(kScoreThreads), lds, st, (const bf16_t*)K,
                       (const bf16_t*)V, feat, len, (const bf16_t*)sc->w1, sc->b1, sc->w2, sc->b2, sc->hidden,
                       sc->per_head, sc->skip_len, d->n_kv_heads, d->capacity, ppb, scores);
    return launch_status();
}

template <typename T, int D>
static fk_status score_simple_launch(const fk_cache_desc* d, const void* K, const void* V, const float* feat,
                                     const int32_t* len, int max_len, const fk_scorer* sc, float* scores, hipStream_t st) {
    const int rows = d->batch * d->n_kv_heads;
    const int g = d->n_q_heads / d->n_kv_heads;
    const int per_block = kSimpleWaves * kSimplePairs;
    const size_t lds = sizeof(float) * per_block * (2 * D + (feat ? kFeatPlanes * g : 0));
    hipLaunchKernelGGL((score_simple_kernel<T, D>), dim3((max_len + per_block - 1) / per_block, rows), dim3(kSimpleWaves * kWave), lds, st,
                       (const T*)K, (const T*)V, feat, d->n_q_heads / d->n_kv_heads, len, (const T*)sc->w1, sc->b1, sc->w2, sc->b2, sc->hidden,
                       sc->per_head, sc->skip_len, d->n_kv_heads, d->capacity, scores);
    return launch_status();
}

}  // namespace fk

using namespace fk;

extern "C" fk_status fk_score_kv(const fk_cache_desc* desc, const void* K, const void* V, const int32_t* len,
                                 int32_t max_len, const fk_scorer* scorer, float* scores, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !len || !scorer || !scores) return FK_ERR_INVALID_ARG;
    if (!scorer->w1 || !scorer->b1 || !scorer->w2 || !scorer->b2 || scorer->hidden <= 0 || scorer->skip_len < 0) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(scorer->w1)) return FK_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int D = desc->head_dim, H = scorer->hidden;
    if (desc->dtype == FK_F32) {
        if (D == 64) return score_simple_launch<float, 64>(desc, K, V, nullptr, len, max_len, scorer, scores, st);
        return score_simple_launch<float, 128>(desc, K, V, nullptr, len, max_len, scorer, scores, st);
    }
    const bool mfma_ok = (H % 8 == 0) && score_lds_bytes(D, H) <= 160 * 1024;
    if (!mfma_ok) return FK_ERR_UNSUPPORTED;
    if (D == 64) return score_mfma_launch<64, 0>(desc, K, V, nullptr, len, max_len, scorer, scores, st);
    return score_mfma_launch<128, 0>(desc, K, V, nullptr, len, max_len, scorer, scores, st);
}

extern "C" fk_status fk_score_kv_feat(const fk_cache_desc* desc, const void* K, const void* V, const float* feat,
                                      const int32_t* len, int32_t max_len, const fk_scorer* scorer, float* scores,
                                      void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !feat || !len || !scorer || !scores) return FK_ERR_INVALID_ARG;
    if (!scorer->w1 || !scorer->b1 || !scorer->w2 || !scorer->b2 || scorer->hidden <= 0 || scorer->skip_len < 0) return FK_ERR_INVALID_ARG;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(scorer->w1) || !aligned16(feat)) return FK_ERR_INVALID_ARG;
    const int g = desc->n_q_heads / desc->n_kv_heads, H = scorer->hidden, D = desc->head_dim;
    hipStream_t st = (hipStream_t)stream;
    if (desc->dtype == FK_F32) {
        if (D == 64) return score_simple_launch<float, 64>(desc, K, V, feat, len, max_len, scorer, scores, st);
        return score_simple_launch<float, 128>(desc, K, V, feat, len, max_len, scorer, scores, st);
    }
    if (H % 8 != 0 || score_lds_bytes(D, H, g) > 160 * 1024) return FK_ERR_UNSUPPORTED;
#define FK_SCORE_FEAT_CASE(GG)                                                                              \
    case GG:                                                                                                \
        return D == 64 ? score_mfma_launch<64, GG>(desc, K, V, feat, len, max_len, scorer, scores, st)      \
                       : score_mfma_launch<128, GG>(desc, K, V, feat, len, max_len, scorer, scores, st);
    switch (g) {
        FK_SCORE_FEAT_CASE(1)
        FK_SCORE_FEAT_CASE(2)
        FK_SCORE_FEAT_CASE(3)
        FK_SCORE_FEAT_CASE(4)
        FK_SCORE_FEAT_CASE(5)
        FK_SCORE_FEAT_CASE(6)
        FK_SCORE_FEAT_CASE(7)
        FK_SCORE_FEAT_CASE(8)
    }
#undef FK_SCORE_FEAT_CASE
    return FK_ERR_UNSUPPORTED;
}
