// fk_decode_attn / fk_decode_step: split-K flash-decode attention over the retained set
// (Appendix A, "Problem Setup": o_hat = sum_{i in S} softmax_S(s)_i v_i), optionally fused with
// the append of the step's new pair (Section 3.1) so that one decode step is ONE launch.
//
// Work decomposition.  A row (sequence, KV head) is cut into `nsplit` splits of `split_len`
// keys; one workgroup handles one split for all g query heads of the group, so K and V are
// fetched from HBM once per group.  Inside a workgroup every wavefront walks its own tiles of
// the split and keeps an online softmax (running maximum m, running sum l, un-normalised
// accumulator acc); the wavefronts are merged through LDS and the splits of a row through a
// small record in the workspace, the last workgroup of the row to arrive doing the final
// log-sum-exp merge and the store of `out` (no second launch).  With at least 128 rows a row is
// not split at all and the launch has no cross-workgroup traffic.
//
// bf16, D = 128.  K and V tiles of 32 keys are fetched with fully coalesced 128-bit loads (a row is
// 16 lanes x 16 bytes, four rows per wavefront instruction).  The K tile is staged in LDS (padded
// rows) and read back in the MFMA operand layout (one key per lane, 8 consecutive channels), so
// q.K^T is a 16x16x32 MFMA chain with A = the group's query rows zero padded to 16.  The softmax
// runs on the MFMA result layout (one key per lane, 4 heads per lane).  The probabilities, rounded
// to bf16 (the same rounded values feed the normaliser), go through LDS into the A operand of the
// second contraction; its B operand is the V tile, transposed 8x8 inside each lane's registers
// (byte permutes, no cross-lane traffic), so P.V is MFMA too and the accumulator lives in the
// MFMA result layout.  The vector ALUs only do the softmax.
// bf16, D = 64.  q.K^T on MFMA with the K operand loaded directly, P.V as fp32 FMA.
// fp32.  q.K^T as fp32 FMA plus a DPP row reduction, P.V as fp32 FMA.
//
// fk_decode_step_feat (FEAT variant, Appendix B.1).  One workgroup per row.  The scaled base-2 logits
// are stored to a per-row scratch as they are formed; after the wavefront merge, with the final maximum
// and normaliser known, a second pass turns them into attention weights and adds them to the open
// planes of the row's feature state.
#include "fk_common.h"
#include <mutex>

namespace fk {

static constexpr float kNegBig = -1.0e30f;  // "no key seen yet"; exp2(kNegBig - m) == 0

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
union B128 {
    uint4 u;
    bf16x8_t v;
};

// Cross-workgroup traffic (split records, arrival counters) uses agent-scope relaxed atomics:
// they compile to loads / stores that bypass the per-XCD caches (sc1), which costs nothing next
// to a device-wide fence (that one writes back and invalidates a whole L2).
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this wave's earlier global stores have been acknowledged (vmcnt(0); expcnt, lgkmcnt untouched)
__device__ __forceinline__ void wait_stores_done() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

// 16-byte load of streamed cache data.  NT marks it non-temporal: a cache that is larger than the Infinity Cache
// (256 MB) is re-read from HBM every step anyway, and lines that are not kept in the caches make room faster
// (+8 .. 11 % bandwidth measured at 0.5 .. 4 GB); below that size the plain load is the faster one.
template <bool NT>
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
    if constexpr (NT) {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    } else {
        return *p;
    }
}
static constexpr size_t kStreamNtBytes = (size_t)352 << 20;  // K + V bytes of a launch from which NT loads are used

// i-th dword of a 16-byte register quad; i is a compile-time constant after unrolling
__device__ __forceinline__ uint32_t dword_of(const uint4& v, int i) { return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w)); }

template <int CTRL>
__device__ __forceinline__ float dpp_max_step(float v) { return fmaxf(v, dpp_f<CTRL>(v)); }
__device__ __forceinline__ float row16_max(float v) {
    v = dpp_max_step<DPP_QUAD_XOR1>(v);
    v = dpp_max_step<DPP_QUAD_XOR2>(v);
    v = dpp_max_step<DPP_ROW_HALF_MIRROR>(v);
    v = dpp_max_step<DPP_ROW_MIRROR>(v);
    return v;
}

// ---- geometry ------------------------------------------------------------------------------
template <typename T, int D, int G> struct AttnCfg {
    static constexpr bool MFMA = sizeof(T) == 2;
    static constexpr bool PVM = MFMA && D == 128;           // P.V on MFMA as well
    static constexpr int CH = D * (int)sizeof(T) / 16;      // 16-byte chunks per row = lanes per key (P.V layout)
    static constexpr int KG = kWave / CH;                   // key groups per wave in the P.V layout
    static constexpr int WAVES = PVM ? 8 : (MFMA ? (G <= 4 ? 8 : 4) : 4);
    static constexpr int THREADS = WAVES * kWave;
    static constexpr int KT = MFMA ? 32 : KG * 4;           // keys per wave iteration
    static constexpr int VU = KT / KG;                      // V (and fp32 K) loads per lane per iteration
    static constexpr int EPL = Vec16<T>::N;                 // channels per lane
    static constexpr int GP = G <= 4 ? 4 : 8;               // heads padded to the MFMA result rows in use
    static constexpr int NG = PVM ? WAVES : WAVES * KG;     // partial accumulators per workgroup
    static constexpr int PS = KT + 8;                       // PVM: bf16 row stride of the P tile in LDS
    static constexpr int KRS = 272;                         // PVM: padded byte stride of a K row in LDS
    // dynamic LDS (floats unless noted):
    //   PVM:   m [NG][G] | l [NG][G] | w [NG][G] | M [8] | P tiles [WAVES][GP][PS] bf16 | K tiles [WAVES][KT][KRS] bytes
    //          (a wavefront's partial accumulator [G][D] reuses its own K tile once its loop is over), 73 KB at G = 4:
    //          two workgroups fit the 160 KB of a CU
    //   other: acc [NG][G][D] | m [NG][G] | l [NG][G] | w [NG][G] | M [8] | p [WAVES][KT][GP] | corr [WAVES][GP]
    static constexpr int ACC_STRIDE = PVM ? KT * KRS / 4 : G * D;  // floats between the partial accumulators
    static constexpr size_t HEAD_FLOATS = 3 * (size_t)NG * G + 8;   // m, l, w, M
    static constexpr size_t PB_BYTES = (size_t)WAVES * GP * PS * 2;  // PVM: the bf16 P tiles
    static constexpr size_t LDS_BYTES =
        PVM ? sizeof(float) * HEAD_FLOATS + PB_BYTES + (size_t)WAVES * KT * KRS
            : sizeof(float) * ((size_t)NG * G * D + HEAD_FLOATS + (size_t)WAVES * KT * GP + (size_t)WAVES * GP + 4);
    // attention-feature variant: lx [NG][G] exact normaliser partials | invL [8], behind everything else
    static constexpr size_t LDS_BYTES_FEAT = LDS_BYTES + sizeof(float) * ((size_t)NG * G + 8);
    static constexpr size_t LX_OFFSET = LDS_BYTES / sizeof(float);  // float index of lx in the dynamic LDS
};

struct AttnPlan {
    int split_len;  // keys per split (multiple of the wave tile)
    int nsplit;     // splits per row
    bool rotate;    // workgroups start at different tiles of their splits
};

// Splits per row the plan aims at.  The bf16 D = 128 kernel saturates the memory system from 128 workgroups of
// eight wavefronts when the cache sits in the Infinity Cache, so rows are split only when there are fewer rows
// than that (no split = no cross-workgroup merge at the end of the launch); a cold cache comes from HBM, whose
// latency takes every CU to cover: up to 256 workgroups; the other kernels want about two per CU.
static int attn_want_splits(const fk_cache_desc* d) {
    const int rows = d->batch * d->n_kv_heads;
    if (d->dtype == FK_BF16 && d->head_dim == 128 && (d->flags & FK_CACHE_COLD)) {
        const int want = 256 / rows;
        return want < 1 ? 1 : want;
    }
    const int target = (d->dtype == FK_BF16 && d->head_dim == 128) ? 128 : 512;
    const int want = (target + rows - 1) / rows;
    return want < 1 ? 1 : want;
}

// Upper bound on the splits any max_len can get (sizes the workspace).
static int attn_max_splits(const fk_cache_desc* d) { return attn_want_splits(d); }

static AttnPlan attn_plan(const fk_cache_desc* d, int max_len) {
    const int tile = 32;
    int want = attn_want_splits(d);
    const int max_split = (max_len + tile - 1) / tile;
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    int split_len = (max_len + want - 1) / want;
    split_len = (split_len + tile - 1) / tile * tile;
    // (Rounding the splits down to whole rounds of the workgroup, with the rest of the row as a short split of its
    // own, was measured and dropped: more workgroups than CUs end up two to a CU while other CUs idle, 85 -> 112 us
    // at 64 rows of 16448 keys.)
    AttnPlan p;
    p.split_len = split_len;
    p.nsplit = (max_len + split_len - 1) / split_len;
    if (p.nsplit < 1) p.nsplit = 1;
    // Start every workgroup at another tile of its split when the splits are long and the cache comes from HBM:
    // workgroups that walk rows a near power of two apart in step crowd the same memory channels (measured on
    // 512 MB per launch, 4128 keys per split: 5.2 TB/s in step, 6.3 TB/s rotated); short splits lose 2 % to it.
    p.rotate = p.nsplit > 1 && split_len >= 2048;
    return p;
}

// workspace: [row arrival counters: rows u32] padded to 256 B | records
static size_t attn_counter_bytes(const fk_cache_desc* d) {
    const size_t n = (size_t)d->batch * d->n_kv_heads;
    return (n * sizeof(uint32_t) + 255) / 256 * 256;
}

struct AttnParams {
    const void* q;
    void* K;
    void* V;
    int32_t* pos;
    int32_t* len;
    const void* k_new;  // null: no append
    const void* v_new;
    const int32_t* pos_new;
    float scale_log2e;
    int n_kv, cap, split_len, nsplit;
    int rotate;          // bf16 D = 128: workgroups start at different tiles of their splits
    float* rec;          // [rows][nsplit][G][D + 2]
    uint32_t* row_cnt;   // [rows], zero between launches
    void* out;
    // attention features (Appendix B.1), only read by the feature variant of the kernel
    float* feat;      // [rows][6][cap][GP]
    float* logit;     // [rows][cap][GP] scratch: base-2 logits of this step
    int chunk_pos, chunk_len;
};

// planes of the feature state: sums of this chunk's attention weights over the last 8 / 16 / 32
// queries and over the whole chunk, then the sums carried over the earlier chunks (plain, 0.9-decayed)
enum { FEAT_W8 = 0, FEAT_W16, FEAT_W32, FEAT_WL, FEAT_CUM, FEAT_DEC, FEAT_PLANES };

__device__ __forceinline__ void feat_add(float4* dst, const float4 p) {
    const float4 v = *dst;
    *dst = make_float4(v.x + p.x, v.y + p.y, v.z + p.z, v.w + p.w);
}

__device__ __forceinline__ float4 keep_if(bool c, const float4 p) {
    return make_float4(c ? p.x : 0.f, c ? p.y : 0.f, c ? p.z : 0.f, c ? p.w : 0.f);
}

template <typename T, int D, int G, bool FEAT, bool NT>
__global__ __launch_bounds__((AttnCfg<T, D, G>::THREADS)) void attn_kernel(const AttnParams P) {
    using C = AttnCfg<T, D, G>;
    constexpr int CH = C::CH, KG = C::KG, WAVES = C::WAVES, KT = C::KT, VU = C::VU, EPL = C::EPL, GP = C::GP, NG = C::NG;
    const int row = blockIdx.y, split = blockIdx.x;
    const int b = row / P.n_kv, hkv = row % P.n_kv;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

    extern __shared__ __attribute__((aligned(16))) float smem[];
    // PVM: head | P tiles | K tiles, the partial accumulators live in the K tiles; other paths: acc | head | p | corr
    float* s_m = C::PVM ? smem : smem + (size_t)NG * G * D;  // [NG][G]
    float* s_l = s_m + NG * G;                 // [NG][G]
    float* s_w = s_l + NG * G;                 // [NG][G] merge weights 2^(m_g - M)
    float* s_M = s_w + NG * G;                 // [8] merged maximum per head
    float* s_p = s_M + 8;                      // other paths: [WAVES][KT][GP]; PVM: the bf16 P tiles
    float* s_corr = s_p + WAVES * KT * GP;     // other paths: [WAVES][GP]
    unsigned char* s_kt = reinterpret_cast<unsigned char*>(s_p) + C::PB_BYTES;  // PVM: K tiles [WAVES][KT][KRS]
    float* s_acc = C::PVM ? reinterpret_cast<float*>(s_kt) : smem;  // partial g2 at s_acc + g2 * ACC_STRIDE, [G][D]
    __shared__ int s_last;

    const bool appending = P.k_new != nullptr;
    const int n_old = min(max(P.len[row], 0), P.cap);
    const bool do_append = appending && n_old < P.cap;
    const int n = n_old + (do_append ? 1 : 0);
    // splits in use; if the caller's max_len was too small the last split runs on to the row's end (slower, still right)
    const int used = min((n + P.split_len - 1) / P.split_len, P.nsplit);
    T* out = reinterpret_cast<T*>(P.out) + ((size_t)b * P.n_kv + hkv) * G * D;

    // Every workgroup of the row calls finish() once, as its last action.  With one workgroup per
    // row it just publishes the new length.  With several, all of them (also those whose split lies
    // beyond the row's end) report to the row's arrival counter; the last one to arrive merges the
    // splits, out = sum_s acc_s 2^(m_s - m*) / sum_s l_s 2^(m_s - m*), and only then bumps len[row],
    // which every workgroup of the row has read by that time.
    auto finish = [&](bool wrote_record) {
        if (gridDim.x == 1) {
            if (do_append && tid == 0) P.len[row] = n;
            return;
        }
        if (!appending && used <= 1) return;  // same decision in every workgroup of the row
        if (wrote_record) wait_stores_done();
        __syncthreads();
        if (tid == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(&P.row_cnt[row], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = prev == gridDim.x - 1;
            if (s_last) __hip_atomic_store(&P.row_cnt[row], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!s_last) return;
        if (used > 1) {
            // log-sum-exp merge of the splits' records, eight records' loads in flight per thread
            const float* r0 = P.rec + (size_t)row * P.nsplit * G * (D + 2);
            const size_t stride = (size_t)G * (D + 2);
            for (int idx = tid; idx < G * D; idx += C::THREADS) {
                const int h = idx / D, d = idx % D;
                const float* r = r0 + (size_t)h * (D + 2);
                float M = kNegBig, a = 0.f, ls = 0.f;
                for (int s0 = 0; s0 < used; s0 += 8) {
                    float mv[8], lv[8], av[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float* rs = r + (size_t)min(s0 + u, used - 1) * stride;
                        mv[u] = ld_agent(rs + D);
                        lv[u] = ld_agent(rs + D + 1);
                        av[u] = ld_agent(rs + d);
                    }
                    float cm = M;
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (s0 + u < used) cm = fmaxf(cm, mv[u]);
                    const float c0 = exp2f(M - cm);
                    a *= c0;
                    ls *= c0;
                    M = cm;
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (s0 + u < used) {
                            const float cw = exp2f(mv[u] - M);
                            a = fmaf(av[u], cw, a);
                            ls = fmaf(lv[u], cw, ls);
                        }
                    }
                }
                store_out(out + idx, a / ls);
            }
        }
        if (do_append && tid == 0) P.len[row] = n;
    };

    if (n == 0) {
        if (split == 0)
            for (int i = tid; i < G * D; i += C::THREADS) store_out(out + i, 0.f);
        finish(false);
        return;
    }
    if (split >= used) {
        finish(false);
        return;
    }
    const int start = split * P.split_len;
    const int end = split == used - 1 ? n : start + P.split_len;

    T* Kr = reinterpret_cast<T*>(P.K) + (size_t)row * P.cap * D;
    T* Vr = reinterpret_cast<T*>(P.V) + (size_t)row * P.cap * D;
    // The workgroup whose split holds the slot of the new pair stores it into the cache.  The bf16
    // D = 128 path never waits for that store: lanes that need the new row read it from k_new / v_new.
    const bool owns_new = do_append && n_old >= start && n_old < end;
    const uint4* knew_row = reinterpret_cast<const uint4*>(reinterpret_cast<const T*>(P.k_new) + (size_t)row * D);
    const uint4* vnew_row = reinterpret_cast<const uint4*>(reinterpret_cast<const T*>(P.v_new) + (size_t)row * D);
    if (owns_new) {
        if (tid < CH) {
            reinterpret_cast<uint4*>(Kr + (size_t)n_old * D)[tid] = knew_row[tid];
        } else if (tid < 2 * CH) {
            reinterpret_cast<uint4*>(Vr + (size_t)n_old * D)[tid - CH] = vnew_row[tid - CH];
        } else if (tid == 2 * CH) {
            P.pos[(size_t)row * P.cap + n_old] = P.pos_new[b];
        }
        if constexpr (!C::PVM) __syncthreads();  // the other paths read the row back from the cache
    }
    const int new_slot = owns_new ? n_old : -1;
    const uint4* Krow = reinterpret_cast<const uint4*>(Kr);
    const uint4* Vrow = reinterpret_cast<const uint4*>(Vr);
    const T* qrow = reinterpret_cast<const T*>(P.q) + ((size_t)b * P.n_kv + hkv) * G * D;

    const int dl = lane % CH;   // 16-byte chunk of the row (P.V layout)
    const int kgv = lane / CH;  // key group (P.V layout)
    float acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;

    if constexpr (C::PVM) {
        constexpr int PS = C::PS, KRS = C::KRS;
        const int n16 = lane & 15, quad = lane >> 4;
        uint16_t* my_pb = reinterpret_cast<uint16_t*>(s_p) + (size_t)wave * GP * PS;           // [GP][PS] bf16
        unsigned char* my_k = s_kt + (size_t)wave * KT * KRS;
        B128 qa[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (n16 < G) qa[ks].u = *reinterpret_cast<const uint4*>(qrow + (size_t)n16 * D + ks * 32 + quad * 8);
            else qa[ks].u = make_uint4(0, 0, 0, 0);
        }
        float m_run[4], l_run[4], lx_run[4];  // lx: sum of the unrounded weights (feature variant)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m_run[i] = kNegBig;
            l_run[i] = 0.f;
            lx_run[i] = 0.f;
        }
        float* lg_row = FEAT ? P.logit + (size_t)row * P.cap * GP : nullptr;
        f32x4_t o[8];  // o[e][i] = out[head quad*4 + i][channel n16*8 + e], un-normalised
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

        // Tiles are dealt round robin to the wavefronts; with P.rotate the deal starts from a tile that differs
        // from workgroup to workgroup (the online softmax does not care about the order).
        const int ntiles = (end - start + KT - 1) / KT;
        const int rot = P.rotate ? (int)(((unsigned)row * 37u + (unsigned)split * 11u) % (unsigned)ntiles) : 0;
        for (int t = wave; t < ntiles; t += WAVES) {
            const int tt = t + rot < ntiles ? t + rot : t + rot - ntiles;
            const int base = start + tt * KT;
            uint4 vr[8];
            {
                uint4 kr[8];  // lane (quad, n16): key base + quad*8 + u, 16-byte chunk n16
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int kc = min(base + quad * 8 + u, end - 1);
                    kr[u] = ld_stream<NT>((kc == new_slot ? knew_row : Krow + (size_t)kc * CH) + n16);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int kc = min(base + quad * 8 + u, end - 1);
                    vr[u] = ld_stream<NT>((kc == new_slot ? vnew_row : Vrow + (size_t)kc * CH) + n16);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) *reinterpret_cast<uint4*>(my_k + (quad * 8 + u) * KRS + n16 * 16) = kr[u];
            }
            __builtin_amdgcn_wave_barrier();
            // B operand of q.K^T: lane = key n16 of tile nt, channels ks*32 + quad*8 .. +8
            f32x4_t c[2];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                c[nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    B128 kb;
                    kb.u = *reinterpret_cast<const uint4*>(my_k + (nt * 16 + n16) * KRS + (ks * 4 + quad) * 16);
                    c[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks].v, kb.v, c[nt], 0, 0, 0);
                }
            }
            bool changed = false;
            float corr[4];
            uint32_t pb[2][4];
            if constexpr (FEAT) {  // keep the step's logits: the second pass turns them into attention weights
                if (quad * 4 < GP) {
                    if (base + n16 < end)
                        *reinterpret_cast<float4*>(lg_row + (size_t)(base + n16) * GP + quad * 4) =
                            make_float4(c[0][0] * P.scale_log2e, c[0][1] * P.scale_log2e, c[0][2] * P.scale_log2e, c[0][3] * P.scale_log2e);
                    if (base + 16 + n16 < end)
                        *reinterpret_cast<float4*>(lg_row + (size_t)(base + 16 + n16) * GP + quad * 4) =
                            make_float4(c[1][0] * P.scale_log2e, c[1][1] * P.scale_log2e, c[1][2] * P.scale_log2e, c[1][3] * P.scale_log2e);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s0 = (base + n16 < end) ? c[0][i] * P.scale_log2e : kNegBig;
                const float s1 = (base + 16 + n16 < end) ? c[1][i] * P.scale_log2e : kNegBig;
                const float mn = fmaxf(m_run[i], row16_max(fmaxf(s0, s1)));
                changed |= mn > m_run[i];
                corr[i] = exp2f(m_run[i] - mn);
                // probabilities rounded to bf16; the SAME rounded values go into l, so the weights stay normalised
                const float e0 = exp2f(s0 - mn), e1 = exp2f(s1 - mn);
                const uint32_t u0 = __float_as_uint(e0) + 0x8000u, u1 = __float_as_uint(e1) + 0x8000u;
                pb[0][i] = u0 >> 16;
                pb[1][i] = u1 >> 16;
                l_run[i] = l_run[i] * corr[i] + __uint_as_float(u0 & 0xffff0000u) + __uint_as_float(u1 & 0xffff0000u);
                if constexpr (FEAT) lx_run[i] = lx_run[i] * corr[i] + e0 + e1;
                m_run[i] = mn;
            }
            if (quad * 4 < GP) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    my_pb[(quad * 4 + i) * PS + n16] = (uint16_t)pb[0][i];
                    my_pb[(quad * 4 + i) * PS + 16 + n16] = (uint16_t)pb[1][i];
                }
            }
            if (__any(changed)) {  // the running maximum moved: rescale what has been accumulated
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[e][i] *= corr[i];
            }
            __builtin_amdgcn_wave_barrier();
            // A operand of P.V: P[head n16][k-slots quad*8 .. +8]; k-slot u of group quad is key base + quad*8 + u
            B128 pa;
            if (n16 < GP) pa.u = *reinterpret_cast<const uint4*>(my_pb + n16 * PS + quad * 8);
            else pa.u = make_uint4(0, 0, 0, 0);
            // B operand: tile e = channel n16*8 + e over this lane's 8 k-slots (8x8 transpose in registers)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                B128 vb;
                vb.u.x = __builtin_amdgcn_perm(dword_of(vr[1], e >> 1), dword_of(vr[0], e >> 1), sel);
                vb.u.y = __builtin_amdgcn_perm(dword_of(vr[3], e >> 1), dword_of(vr[2], e >> 1), sel);
                vb.u.z = __builtin_amdgcn_perm(dword_of(vr[5], e >> 1), dword_of(vr[4], e >> 1), sel);
                vb.u.w = __builtin_amdgcn_perm(dword_of(vr[7], e >> 1), dword_of(vr[6], e >> 1), sel);
                o[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.v, vb.v, o[e], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
        // publish one partial per wave
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = quad * 4 + i;
            const float ls = group_sum<16>(l_run[i]);
            if (h < G) {
                float* dst = s_acc + (size_t)wave * C::ACC_STRIDE + (size_t)h * D + n16 * 8;  // own K tile: its loop is over
                *reinterpret_cast<float4*>(dst) = make_float4(o[0][i], o[1][i], o[2][i], o[3][i]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(o[4][i], o[5][i], o[6][i], o[7][i]);
                if (n16 == 0) {
                    s_m[wave * G + h] = m_run[i];
                    s_l[wave * G + h] = ls;
                }
            }
            if constexpr (FEAT) {
                const float lxs = group_sum<16>(lx_run[i]);
                if (h < G && n16 == 0) smem[C::LX_OFFSET + wave * G + h] = lxs;
            }
        }
    } else if constexpr (C::MFMA) {
        constexpr int KS = D / 32;  // MFMA k-steps
        const int n16 = lane & 15, quad = lane >> 4;
        B128 qa[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (n16 < G) qa[ks].u = *reinterpret_cast<const uint4*>(qrow + (size_t)n16 * D + ks * 32 + quad * 8);
            else qa[ks].u = make_uint4(0, 0, 0, 0);
        }
        float m_run[4], l_run[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m_run[i] = kNegBig;
            l_run[i] = 0.f;
        }
        float* my_p = s_p + (size_t)wave * KT * GP;
        float* my_corr = s_corr + wave * GP;

        for (int base = start + wave * KT; base < end; base += WAVES * KT) {
            B128 kb[2][KS];
            uint4 vr[VU];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int kc = min(base + nt * 16 + n16, end - 1);  // clamp: always a live slot
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kb[nt][ks].u = Krow[(size_t)kc * CH + ks * 4 + quad];
            }
#pragma unroll
            for (int u = 0; u < VU; ++u) {
                const int kc = min(base + u * KG + kgv, end - 1);
                vr[u] = Vrow[(size_t)kc * CH + dl];
            }
            f32x4_t c[2];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                c[nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    c[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks].v, kb[nt][ks].v, c[nt], 0, 0, 0);
            }
            // result layout: lane = key n16 of tile nt, element i = head quad*4 + i
            if constexpr (FEAT) {
                float* lg_row = P.logit + (size_t)row * P.cap * GP;
                if (quad * 4 < GP) {
                    if (base + n16 < end)
                        *reinterpret_cast<float4*>(lg_row + (size_t)(base + n16) * GP + quad * 4) =
                            make_float4(c[0][0] * P.scale_log2e, c[0][1] * P.scale_log2e, c[0][2] * P.scale_log2e, c[0][3] * P.scale_log2e);
                    if (base + 16 + n16 < end)
                        *reinterpret_cast<float4*>(lg_row + (size_t)(base + 16 + n16) * GP + quad * 4) =
                            make_float4(c[1][0] * P.scale_log2e, c[1][1] * P.scale_log2e, c[1][2] * P.scale_log2e, c[1][3] * P.scale_log2e);
                }
            }
            float p[2][4], corr[4];
            bool changed = false;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s0 = (base + n16 < end) ? c[0][i] * P.scale_log2e : kNegBig;
                const float s1 = (base + 16 + n16 < end) ? c[1][i] * P.scale_log2e : kNegBig;
                const float mn = fmaxf(m_run[i], row16_max(fmaxf(s0, s1)));
                changed |= mn > m_run[i];
                corr[i] = exp2f(m_run[i] - mn);
                p[0][i] = exp2f(s0 - mn);
                p[1][i] = exp2f(s1 - mn);
                l_run[i] = l_run[i] * corr[i] + p[0][i] + p[1][i];
                m_run[i] = mn;
            }
            const bool any_changed = __any(changed);
            if (quad * 4 < GP) {
                *reinterpret_cast<float4*>(my_p + (size_t)n16 * GP + quad * 4) = make_float4(p[0][0], p[0][1], p[0][2], p[0][3]);
                *reinterpret_cast<float4*>(my_p + (size_t)(16 + n16) * GP + quad * 4) = make_float4(p[1][0], p[1][1], p[1][2], p[1][3]);
                if (n16 == 0) *reinterpret_cast<float4*>(my_corr + quad * 4) = make_float4(corr[0], corr[1], corr[2], corr[3]);
            }
            __builtin_amdgcn_wave_barrier();
            if (any_changed) {  // the running maximum moved: rescale what has been accumulated
                float cr[GP];
#pragma unroll
                for (int h4 = 0; h4 < GP; h4 += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(my_corr + h4);
                    cr[h4] = t.x; cr[h4 + 1] = t.y; cr[h4 + 2] = t.z; cr[h4 + 3] = t.w;
                }
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[h][e] *= cr[h];
            }
#pragma unroll
            for (int u = 0; u < VU; ++u) {
                float pp[GP];
#pragma unroll
                for (int h4 = 0; h4 < GP; h4 += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(my_p + (size_t)(u * KG + kgv) * GP + h4);
                    pp[h4] = t.x; pp[h4 + 1] = t.y; pp[h4 + 2] = t.z; pp[h4 + 3] = t.w;
                }
                float vf[EPL];
                Vec16<T>::unpack(vr[u], vf);
#pragma unroll
                for (int e = 0; e < EPL; ++e)
#pragma unroll
                    for (int h = 0; h < G; ++h) acc[h][e] = fmaf(pp[h], vf[e], acc[h][e]);
            }
            __builtin_amdgcn_wave_barrier();
        }
        // publish: every (wave, key group) its accumulator; m is uniform in the wave, l is the
        // sum over the 16 key lanes and is credited to key group 0
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float ls = group_sum<16>(l_run[i]);
            const int h = quad * 4 + i;
            if (n16 == 0 && h < G) {
#pragma unroll
                for (int g2 = 0; g2 < KG; ++g2) {
                    s_m[(wave * KG + g2) * G + h] = m_run[i];
                    s_l[(wave * KG + g2) * G + h] = g2 == 0 ? ls : 0.f;
                }
            }
        }
    } else {
        // fp32: every key group (CH lanes) keeps its own online softmax over the keys it sees
        float qf[G][EPL];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            Vec16<T>::unpack(*reinterpret_cast<const uint4*>(qrow + (size_t)h * D + dl * EPL), qf[h]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qf[h][e] *= P.scale_log2e;
        }
        float m[G], l[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            m[h] = kNegBig;
            l[h] = 0.f;
        }
        for (int base = start + wave * KT; base < end; base += WAVES * KT) {
            uint4 kr[VU], vr[VU];
            int key[VU];
#pragma unroll
            for (int u = 0; u < VU; ++u) {
                key[u] = base + u * KG + kgv;
                kr[u] = Krow[(size_t)min(key[u], end - 1) * CH + dl];
            }
#pragma unroll
            for (int u = 0; u < VU; ++u) vr[u] = Vrow[(size_t)min(key[u], end - 1) * CH + dl];
            float s[VU][G];
#pragma unroll
            for (int u = 0; u < VU; ++u) {
                float kf[EPL];
                Vec16<T>::unpack(kr[u], kf);
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) d = fmaf(qf[h][e], kf[e], d);
                    d = group_sum<CH>(d);
                    s[u][h] = key[u] < end ? d : kNegBig;
                }
                if constexpr (FEAT) {
                    if (dl == 0 && key[u] < end) {  // heads beyond the group hold zeros
                        float* lg = P.logit + ((size_t)row * P.cap + key[u]) * GP;
#pragma unroll
                        for (int h4 = 0; h4 < GP; h4 += 4)
                            *reinterpret_cast<float4*>(lg + h4) =
                                make_float4(h4 + 0 < G ? s[u][h4 + 0 < G ? h4 + 0 : 0] : 0.f, h4 + 1 < G ? s[u][h4 + 1 < G ? h4 + 1 : 0] : 0.f,
                                            h4 + 2 < G ? s[u][h4 + 2 < G ? h4 + 2 : 0] : 0.f, h4 + 3 < G ? s[u][h4 + 3 < G ? h4 + 3 : 0] : 0.f);
                    }
                }
            }
            float p[VU][G];
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float mn = m[h];
#pragma unroll
                for (int u = 0; u < VU; ++u) mn = fmaxf(mn, s[u][h]);
                const float corr = exp2f(m[h] - mn);
                float ps = 0.f;
#pragma unroll
                for (int u = 0; u < VU; ++u) {
                    p[u][h] = key[u] < end ? exp2f(s[u][h] - mn) : 0.f;
                    ps += p[u][h];
                }
                l[h] = l[h] * corr + ps;
                m[h] = mn;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] *= corr;
            }
#pragma unroll
            for (int u = 0; u < VU; ++u) {
                float vf[EPL];
                Vec16<T>::unpack(vr[u], vf);
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(p[u][h], vf[e], acc[h][e]);
            }
        }
        if (dl == 0) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                s_m[(wave * KG + kgv) * G + h] = m[h];
                s_l[(wave * KG + kgv) * G + h] = l[h];
            }
        }
    }

    // ---- merge the partials of the workgroup -----------------------------------------------------
    if constexpr (!C::PVM) {
        float* dst = s_acc + (size_t)(wave * KG + kgv) * C::ACC_STRIDE + dl * EPL;
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e4 = 0; e4 < EPL; e4 += 4)
                *reinterpret_cast<float4*>(dst + (size_t)h * D + e4) =
                    make_float4(acc[h][e4], acc[h][e4 + 1], acc[h][e4 + 2], acc[h][e4 + 3]);
    }
    __syncthreads();
    for (int t = tid; t < NG * G; t += C::THREADS) {  // weight of every partial: 2^(m_g - M)
        const int h = t % G;
        float mn = kNegBig;
#pragma unroll 8
        for (int g2 = 0; g2 < NG; ++g2) mn = fmaxf(mn, s_m[g2 * G + h]);
        s_w[t] = exp2f(s_m[t] - mn);
        if (t < G) s_M[t] = mn;
    }
    __syncthreads();
    float* rec = P.rec + ((size_t)row * P.nsplit + split) * G * (D + 2);
    for (int idx = tid; idx < G * D; idx += C::THREADS) {
        const int h = idx / D, d = idx % D;
        const float mn = s_M[h];
        float a = 0.f, ls = 0.f;
#pragma unroll 8
        for (int g2 = 0; g2 < NG; ++g2) a = fmaf(s_acc[(size_t)g2 * C::ACC_STRIDE + (size_t)h * D + d], s_w[g2 * G + h], a);
        if (d == 0 || used == 1) {
#pragma unroll 8
            for (int g2 = 0; g2 < NG; ++g2) ls = fmaf(s_l[g2 * G + h], s_w[g2 * G + h], ls);
        }
        if (used == 1) {
            store_out(out + idx, a / ls);
        } else {
            st_agent(rec + (size_t)h * (D + 2) + d, a);
            if (d == 0) {
                st_agent(rec + (size_t)h * (D + 2) + D, mn);
                st_agent(rec + (size_t)h * (D + 2) + D + 1, ls);
            }
        }
    }
    if constexpr (FEAT) {
        // Second pass (one workgroup per row): weight of key i for head h = 2^(s_i - M_h) / L_h with the
        // merged maximum M_h and the exact (unrounded) normaliser L_h.  Every live slot gains its weight
        // in the chunk plane and in the windows that reach back to this step; the slot appended at this
        // step starts all six planes afresh.
        // exact normaliser partials: the bf16 D = 128 path keeps them apart from the rounded ones it uses for P.V
        const float* s_lx = C::PVM ? smem + C::LX_OFFSET : s_l;
        float* s_invL = smem + C::LX_OFFSET + NG * G;
        if (tid < G) {
            float ls = 0.f;
#pragma unroll 8
            for (int g2 = 0; g2 < NG; ++g2) ls = fmaf(s_lx[g2 * G + tid], s_w[g2 * G + tid], ls);
            s_invL[tid] = 1.0f / ls;
        }
        __syncthreads();  // also: the logits stored above by other waves of this workgroup are visible
        const float* lg_row = P.logit + (size_t)row * P.cap * GP;
        float* frow = P.feat + (size_t)row * FEAT_PLANES * P.cap * GP;
        constexpr int Q4 = GP / 4;
        const size_t pl4 = (size_t)P.cap * Q4;  // float4 units per plane
        const bool on8 = P.chunk_pos >= P.chunk_len - 8, on16 = P.chunk_pos >= P.chunk_len - 16,
                   on32 = P.chunk_pos >= P.chunk_len - 32;
        const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
        // four units (slot, 4 heads) per thread and pass, all loads issued before the first use
        constexpr int U = 4;
        const int units = n * Q4;
        const int h0 = (tid % Q4) * 4;  // THREADS is a multiple of Q4: a thread keeps its head quad
        float4 mq, iq;                  // maxima and 1 / normalisers of this thread's heads
        mq.x = h0 + 0 < G ? s_M[h0 + 0] : 0.f;  iq.x = h0 + 0 < G ? s_invL[h0 + 0] : 0.f;
        mq.y = h0 + 1 < G ? s_M[h0 + 1] : 0.f;  iq.y = h0 + 1 < G ? s_invL[h0 + 1] : 0.f;
        mq.z = h0 + 2 < G ? s_M[h0 + 2] : 0.f;  iq.z = h0 + 2 < G ? s_invL[h0 + 2] : 0.f;
        mq.w = h0 + 3 < G ? s_M[h0 + 3] : 0.f;  iq.w = h0 + 3 < G ? s_invL[h0 + 3] : 0.f;
        const float4* lg4 = reinterpret_cast<const float4*>(lg_row);
        float4* f4 = reinterpret_cast<float4*>(frow);
        for (int t0 = tid; t0 < units; t0 += C::THREADS * U) {
            float4 s[U], w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = min(t0 + u * C::THREADS, units - 1);
                s[u] = lg4[t];
                w[u] = f4[FEAT_WL * pl4 + t];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0 + u * C::THREADS;
                if (t >= units) break;
                // padded heads: their logits are 0 and iq is 0, so p = 0
                const float4 p = make_float4(exp2f(s[u].x - mq.x) * iq.x, exp2f(s[u].y - mq.y) * iq.y,
                                             exp2f(s[u].z - mq.z) * iq.z, exp2f(s[u].w - mq.w) * iq.w);
                float4* f = f4 + t;
                if (t / Q4 == new_slot) {
                    f[FEAT_W8 * pl4] = keep_if(on8, p);
                    f[FEAT_W16 * pl4] = keep_if(on16, p);
                    f[FEAT_W32 * pl4] = keep_if(on32, p);
                    f[FEAT_WL * pl4] = p;
                    f[FEAT_CUM * pl4] = zero;
                    f[FEAT_DEC * pl4] = zero;
                } else {
                    f[FEAT_WL * pl4] = make_float4(w[u].x + p.x, w[u].y + p.y, w[u].z + p.z, w[u].w + p.w);
                    if (on32) feat_add(f + FEAT_W32 * pl4, p);
                    if (on16) feat_add(f + FEAT_W16 * pl4, p);
                    if (on8) feat_add(f + FEAT_W8 * pl4, p);
                }
            }
        }
    }
    finish(used > 1);
}

template <typename T, int D, int G>
static fk_status attn_launch(const fk_cache_desc* d, const AttnParams& base, int max_len, void* ws, hipStream_t st) {
    using C = AttnCfg<T, D, G>;
    {
        if (base.feat) {  // feature variant: one workgroup per row, the logit scratch sits behind the counters
            AttnParams P = base;
            P.split_len = (d->capacity + 31) / 32 * 32;  // the whole row, whatever max_len says
            P.nsplit = 1;
            P.row_cnt = reinterpret_cast<uint32_t*>(ws);
            P.rec = nullptr;
            P.logit = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + attn_counter_bytes(d));
            const int frows = d->batch * d->n_kv_heads;
            if constexpr (C::PVM) {
                if ((d->flags & FK_CACHE_COLD) || (size_t)frows * max_len * D * sizeof(T) * 2 >= kStreamNtBytes) {
                    auto kern = attn_kernel<T, D, G, true, true>;
                    static bool lds_ok[kMaxDevices] = {};
                    if (!allow_dynamic_lds((const void*)kern, C::LDS_BYTES_FEAT, lds_ok)) return FK_ERR_LAUNCH;
                    hipLaunchKernelGGL(kern, dim3(1, frows), dim3(C::THREADS), C::LDS_BYTES_FEAT, st, P);
                    return launch_status();
                }
            }
            auto kern = attn_kernel<T, D, G, true, false>;
            static bool lds_ok[kMaxDevices] = {};  // per template instantiation
            if (!allow_dynamic_lds((const void*)kern, C::LDS_BYTES_FEAT, lds_ok)) return FK_ERR_LAUNCH;
            hipLaunchKernelGGL(kern, dim3(1, frows), dim3(C::THREADS), C::LDS_BYTES_FEAT, st, P);
            return launch_status();
        }
    }
    const AttnPlan p = attn_plan(d, max_len);
    const int rows = d->batch * d->n_kv_heads;
    AttnParams P = base;
    P.split_len = p.split_len;
    P.nsplit = p.nsplit;
    P.rotate = p.rotate ? 1 : 0;
    P.row_cnt = reinterpret_cast<uint32_t*>(ws);
    P.rec = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + attn_counter_bytes(d));
    if constexpr (C::PVM) {
        if ((d->flags & FK_CACHE_COLD) || (size_t)rows * max_len * D * sizeof(T) * 2 >= kStreamNtBytes) {  // not cache resident
            auto kern = attn_kernel<T, D, G, false, true>;
            static bool lds_ok[kMaxDevices] = {};
            if (!allow_dynamic_lds((const void*)kern, C::LDS_BYTES, lds_ok)) return FK_ERR_LAUNCH;
            hipLaunchKernelGGL(kern, dim3(p.nsplit, rows), dim3(C::THREADS), C::LDS_BYTES, st, P);
            return launch_status();
        }
    }
    auto kern = attn_kernel<T, D, G, false, false>;
    static bool lds_ok[kMaxDevices] = {};  // per template instantiation
    if (!allow_dynamic_lds((const void*)kern, C::LDS_BYTES, lds_ok)) return FK_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(p.nsplit, rows), dim3(C::THREADS), C::LDS_BYTES, st, P);
    return launch_status();
}

template <typename T, int D>
static fk_status attn_dispatch_g(int g, const fk_cache_desc* d, const AttnParams& P, int max_len, void* ws, hipStream_t st) {
    switch (g) {
        case 1: return attn_launch<T, D, 1>(d, P, max_len, ws, st);
        case 2: return attn_launch<T, D, 2>(d, P, max_len, ws, st);
        case 3: return attn_launch<T, D, 3>(d, P, max_len, ws, st);
        case 4: return attn_launch<T, D, 4>(d, P, max_len, ws, st);
        case 5: return attn_launch<T, D, 5>(d, P, max_len, ws, st);
        case 6: return attn_launch<T, D, 6>(d, P, max_len, ws, st);
        case 7: return attn_launch<T, D, 7>(d, P, max_len, ws, st);
        case 8: return attn_launch<T, D, 8>(d, P, max_len, ws, st);
    }
    return FK_ERR_UNSUPPORTED;
}

static size_t feat_workspace_bytes(const fk_cache_desc* d) {
    const size_t g = d->n_q_heads / d->n_kv_heads;
    return attn_counter_bytes(d) + (size_t)d->batch * d->n_kv_heads * d->capacity * (g <= 4 ? 4 : 8) * sizeof(float);
}

static fk_status attn_entry(const fk_cache_desc* desc, AttnParams P, int max_len, float softmax_scale, void* workspace,
                            size_t workspace_bytes, void* stream) {
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    const size_t need = P.feat ? feat_workspace_bytes(desc) : fk_decode_attn_workspace(desc, max_len);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return FK_ERR_WORKSPACE;
    const int g = desc->n_q_heads / desc->n_kv_heads;
    P.scale_log2e = softmax_scale * 1.4426950408889634f;
    P.n_kv = desc->n_kv_heads;
    P.cap = desc->capacity;
    hipStream_t st = (hipStream_t)stream;
    if (desc->dtype == FK_F32) {
        if (desc->head_dim == 64) return attn_dispatch_g<float, 64>(g, desc, P, max_len, workspace, st);
        return attn_dispatch_g<float, 128>(g, desc, P, max_len, workspace, st);
    }
    if (desc->head_dim == 64) return attn_dispatch_g<bf16_t, 64>(g, desc, P, max_len, workspace, st);
    return attn_dispatch_g<bf16_t, 128>(g, desc, P, max_len, workspace, st);
}

}  // namespace fk

using namespace fk;

extern "C" size_t fk_decode_attn_workspace(const fk_cache_desc* desc, int32_t max_len) {
    if (check_desc(desc) != FK_OK || max_len <= 0 || max_len > desc->capacity) return 0;
    // sized for the largest split count any max_len can get, so one workspace serves every call
    const size_t g = desc->n_q_heads / desc->n_kv_heads;
    return attn_counter_bytes(desc) +
           (size_t)desc->batch * desc->n_kv_heads * attn_max_splits(desc) * g * (desc->head_dim + 2) * sizeof(float);
}

extern "C" fk_status fk_decode_attn(const fk_cache_desc* desc, const void* q, const void* K, const void* V,
                                    const int32_t* len, int32_t max_len, float softmax_scale, void* out,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!q || !K || !V || !len || !out) return FK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out)) return FK_ERR_INVALID_ARG;
    AttnParams P = {};
    P.q = q;
    P.K = const_cast<void*>(K);
    P.V = const_cast<void*>(V);
    P.len = const_cast<int32_t*>(len);
    P.out = out;
    return attn_entry(desc, P, max_len, softmax_scale, workspace, workspace_bytes, stream);
}

extern "C" fk_status fk_decode_step(const fk_cache_desc* desc, const void* q, void* K, void* V, int32_t* pos,
                                    int32_t* len, const void* k_new, const void* v_new, const int32_t* pos_new,
                                    int32_t max_len, float softmax_scale, void* out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!q || !K || !V || !pos || !len || !k_new || !v_new || !pos_new || !out) return FK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new))
        return FK_ERR_INVALID_ARG;
    AttnParams P = {};
    P.q = q;
    P.K = K;
    P.V = V;
    P.pos = pos;
    P.len = len;
    P.k_new = k_new;
    P.v_new = v_new;
    P.pos_new = pos_new;
    P.out = out;
    return attn_entry(desc, P, max_len, softmax_scale, workspace, workspace_bytes, stream);
}

extern "C" fk_status fk_decode_window(const fk_cache_desc* desc, const void* q_seq, void* K, void* V, int32_t* pos,
                                      int32_t* len, const void* k_seq, const void* v_seq, const int32_t* pos_seq,
                                      int32_t n_steps, int32_t max_len_first, float softmax_scale, void* out_seq,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (n_steps < 0 || max_len_first <= 0 || max_len_first > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!q_seq || !k_seq || !v_seq || !pos_seq || !out_seq) return FK_ERR_INVALID_ARG;
    const size_t e = desc->dtype == FK_F32 ? 4 : 2;
    const size_t q_step = (size_t)desc->batch * desc->n_q_heads * desc->head_dim * e;   // bytes per step, multiples of 16
    const size_t kv_step = (size_t)desc->batch * desc->n_kv_heads * desc->head_dim * e;
    for (int32_t t = 0; t < n_steps; ++t) {
        const int64_t ml = (int64_t)max_len_first + t;
        s = fk_decode_step(desc, static_cast<const char*>(q_seq) + t * q_step, K, V, pos, len,
                           static_cast<const char*>(k_seq) + t * kv_step, static_cast<const char*>(v_seq) + t * kv_step,
                           pos_seq + (size_t)t * desc->batch, ml > desc->capacity ? desc->capacity : (int32_t)ml, softmax_scale,
                           static_cast<char*>(out_seq) + t * q_step, workspace, workspace_bytes, stream);
        if (s != FK_OK) return s;
    }
    return FK_OK;
}

// ---------------------------------------------------------------------------------------------------------
// fk_decode_step_static: fk_decode_step for callers that cannot allocate.  The workspace (row arrival counters
// and split records) is a fixed array in the library's device image; every GPU the library runs on holds
// its own copy at its own address, looked up once per device.
// ---------------------------------------------------------------------------------------------------------
namespace fk {
static constexpr size_t kStaticScratchBytes = FK_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, null until looked up
static std::mutex g_scratch_mutex;

__global__ void scratch_clear_kernel(uint4* p, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// Device address of the static scratch on the current device; on the first call on a device the address is looked
// up and the array is cleared on `st` (a fill kernel, no memset node: the caller may be capturing a graph), which
// orders the clear before the first launch that uses it.  Null on failure.
static void* static_scratch(hipStream_t st) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        hipLaunchKernelGGL(scratch_clear_kernel, dim3(256), dim3(256), 0, st, reinterpret_cast<uint4*>(ptr), kStaticScratchBytes / 16);
        if (hipGetLastError() != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace fk

extern "C" fk_status fk_decode_step_static(const fk_cache_desc* desc, const void* q, void* K, void* V, int32_t* pos,
                                           int32_t* len, const void* k_new, const void* v_new, const int32_t* pos_new,
                                           int32_t max_len, float softmax_scale, void* out, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (max_len <= 0 || max_len > desc->capacity) return FK_ERR_INVALID_ARG;
    if (fk_decode_attn_workspace(desc, max_len) > kStaticScratchBytes) return FK_ERR_WORKSPACE;  // beyond the fixed scratch
    if (!q || !K || !V || !pos || !len || !k_new || !v_new || !pos_new || !out) return FK_ERR_INVALID_ARG;
    void* ws = static_scratch((hipStream_t)stream);
    if (!ws) return FK_ERR_LAUNCH;
    return fk_decode_step(desc, q, K, V, pos, len, k_new, v_new, pos_new, max_len, softmax_scale, out, ws, kStaticScratchBytes, stream);
}

extern "C" size_t fk_decode_step_feat_workspace(const fk_cache_desc* desc) {
    if (check_desc(desc) != FK_OK) return 0;
    return feat_workspace_bytes(desc);
}

extern "C" fk_status fk_decode_step_feat(const fk_cache_desc* desc, const void* q, void* K, void* V, int32_t* pos,
                                         int32_t* len, const void* k_new, const void* v_new, const int32_t* pos_new,
                                         int32_t max_len, float softmax_scale, float* feat, int32_t chunk_pos,
                                         int32_t chunk_len, void* out, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!q || !K || !V || !pos || !len || !k_new || !v_new || !pos_new || !out || !feat) return FK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new) ||
        !aligned16(feat))
        return FK_ERR_INVALID_ARG;
    if (chunk_len <= 0 || chunk_pos < 0 || chunk_pos >= chunk_len) return FK_ERR_INVALID_ARG;
    AttnParams P = {};
    P.q = q;
    P.K = K;
    P.V = V;
    P.pos = pos;
    P.len = len;
    P.k_new = k_new;
    P.v_new = v_new;
    P.pos_new = pos_new;
    P.out = out;
    P.feat = feat;
    P.chunk_pos = chunk_pos;
    P.chunk_len = chunk_len;
    return attn_entry(desc, P, max_len, softmax_scale, workspace, workspace_bytes, stream);
}

// fk_decode_step_feat for the steps from chunk_pos_first to the end of a window inside one chunk, enqueued by one call
extern "C" fk_status fk_decode_window_feat(const fk_cache_desc* desc, const void* q_seq, void* K, void* V, int32_t* pos,
                                           int32_t* len, const void* k_seq, const void* v_seq, const int32_t* pos_seq,
                                           int32_t n_steps, int32_t max_len_first, float softmax_scale, float* feat,
                                           int32_t chunk_pos_first, int32_t chunk_len, void* out_seq, void* workspace,
                                           size_t workspace_bytes, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (n_steps < 0 || max_len_first <= 0 || max_len_first > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!q_seq || !k_seq || !v_seq || !pos_seq || !out_seq) return FK_ERR_INVALID_ARG;
    if (chunk_len <= 0 || chunk_pos_first < 0 || (int64_t)chunk_pos_first + n_steps > chunk_len) return FK_ERR_INVALID_ARG;
    const size_t e = desc->dtype == FK_F32 ? 4 : 2;
    const size_t q_step = (size_t)desc->batch * desc->n_q_heads * desc->head_dim * e;   // bytes per step, multiples of 16
    const size_t kv_step = (size_t)desc->batch * desc->n_kv_heads * desc->head_dim * e;
    for (int32_t t = 0; t < n_steps; ++t) {
        const int64_t ml = (int64_t)max_len_first + t;
        s = fk_decode_step_feat(desc, static_cast<const char*>(q_seq) + t * q_step, K, V, pos, len,
                                static_cast<const char*>(k_seq) + t * kv_step, static_cast<const char*>(v_seq) + t * kv_step,
                                pos_seq + (size_t)t * desc->batch, ml > desc->capacity ? desc->capacity : (int32_t)ml,
                                softmax_scale, feat, chunk_pos_first + t, chunk_len,
                                static_cast<char*>(out_seq) + t * q_step, workspace, workspace_bytes, stream);
        if (s != FK_OK) return s;
    }
    return FK_OK;
}
