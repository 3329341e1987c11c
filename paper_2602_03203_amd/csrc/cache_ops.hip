// fk_append, fk_compact and fk_compact_feat: the calls that rewrite the cache (and the attention-feature state).
#include "fk_common.h"

namespace fk {

// ---------------------------------------------------------------------------------------
// append (Section 3.1: each generated token adds one pair to every KV-head row)
// one workgroup per row; 16-byte chunks of the new K and V rows
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void append_kernel(uint4* __restrict__ K, uint4* __restrict__ V,
                                                    int32_t* __restrict__ pos, int32_t* __restrict__ len,
                                                    const uint4* __restrict__ k_new,
                                                    const uint4* __restrict__ v_new,
                                                    const int32_t* __restrict__ pos_new, int n_kv,
                                                    int cap, int chunks /* 16-byte chunks per row */) {
    const int row = blockIdx.x;
    const int n = len[row];
    if (n < 0 || n >= cap) return;
    const size_t dst = ((size_t)row * cap + n) * chunks;
    for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
        K[dst + c] = k_new[(size_t)row * chunks + c];
        V[dst + c] = v_new[(size_t)row * chunks + c];
    }
    if (threadIdx.x == 0) {
        pos[(size_t)row * cap + n] = pos_new[row / n_kv];
        len[row] = n + 1;  // only this workgroup reads or writes len[row]
    }
}

// ---------------------------------------------------------------------------------------
// compact (stable in-place gather)
//
// keep[] is ascending with keep[j] >= j.  A workgroup owns one 128-byte column slice of one
// tensor of one row (bytes of different slices never alias, so slices are independent; 128
// bytes = two whole 64-byte memory requests per slot, narrower slices fetch and write partial
// lines and cost 1.5x the time) and walks the destination slots in ascending tiles of 512
// slots: all sources of a tile are loaded into registers, a barrier, then the tile is stored.  A store of tile t lands in slots
// [tT, (t+1)T); a source of any later tile is >= (t+1)T, and every source of tile t or of an
// earlier tile has already been read, so no live source is overwritten.  Entries with
// keep[j] == j (the untouched prefix) cost no traffic.
// grid.x = row, grid.y = tensor * slices + slice (K slices, then V slices), last y = pos
// ---------------------------------------------------------------------------------------
static constexpr int kCompactThreads = 1024;
static constexpr int kCompactU = 4;     // 16-byte loads in flight per thread
static constexpr int kSliceChunks = 8;  // 16-byte chunks per column slice

// The workgroup that moves the positions also sets len[row] = min(len[row], budget) (no second launch).  No other
// workgroup may then read len[row]: what moves is decided by keep alone (rows at or under budget carry the
// identity, entries with keep[j] == j or outside [0, cap) move nothing).
__global__ __launch_bounds__(kCompactThreads) void compact_kernel(uint4* __restrict__ K, uint4* __restrict__ V,
                                                                  int32_t* __restrict__ pos,
                                                                  int32_t* __restrict__ len,
                                                                  const int32_t* __restrict__ keep,
                                                                  int cap, int budget, int chunks) {
    const int row = blockIdx.x;
    const int n = cap;
    const int32_t* kp = keep + (size_t)row * budget;
    const int slices = chunks / kSliceChunks;
    if ((int)blockIdx.y == 2 * slices) {
        if (threadIdx.x == 0 && len[row] > budget) len[row] = budget;
        int32_t* p = pos + (size_t)row * cap;
        for (int base = 0; base < budget; base += kCompactThreads * kCompactU) {
            int32_t val[kCompactU];
            int src[kCompactU];
#pragma unroll
            for (int u = 0; u < kCompactU; ++u) {
                const int j = base + u * kCompactThreads + threadIdx.x;
                src[u] = j < budget ? kp[j] : -1;
                if (src[u] >= 0 && src[u] < n) val[u] = p[src[u]];
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kCompactU; ++u) {
                const int j = base + u * kCompactThreads + threadIdx.x;
                if (src[u] >= 0 && src[u] < n && src[u] != j) p[j] = val[u];
            }
        }
        return;
    }
    const int tensor = blockIdx.y / slices, slice = blockIdx.y % slices;
    uint4* X = (tensor == 0 ? K : V) + (size_t)row * cap * chunks + slice * kSliceChunks;
    constexpr int spi = kCompactThreads / kSliceChunks;  // slots per load instruction of the workgroup
    const int sl = threadIdx.x / kSliceChunks;           // slot within that group
    const int c = threadIdx.x % kSliceChunks;            // 16-byte chunk inside the slice
    for (int base = 0; base < budget; base += spi * kCompactU) {
        uint4 val[kCompactU];
        int src[kCompactU];
#pragma unroll
        for (int u = 0; u < kCompactU; ++u) {
            const int j = base + u * spi + sl;
            src[u] = j < budget ? kp[j] : -1;
            if (src[u] >= 0 && src[u] < n && src[u] != j) val[u] = X[(size_t)src[u] * chunks + c];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kCompactU; ++u) {
            const int j = base + u * spi + sl;
            if (src[u] >= 0 && src[u] < n && src[u] != j) X[(size_t)j * chunks + c] = val[u];
        }
    }
}

// ---------------------------------------------------------------------------------------
// close a chunk of the attention features (Appendix B.1) and compact them with the cache
//
// feat [rows][6][cap][GP]: planes w8, w16, w32, wL (sums of this chunk's attention weights over
// the last 8 / 16 / 32 queries and over the whole chunk), cum, dec (sums carried over earlier
// chunks, plain and decayed by 0.9 per chunk).  At the end of a chunk cum += wL, dec = 0.9 dec
// + wL and the four chunk planes restart from zero; rows over budget move slot keep[j] to slot
// j in the same pass (ascending tiles, all sources of a tile read before it is written: the
// argument of compact_kernel).  One workgroup per row; a thread owns 4 heads of a slot.
// ---------------------------------------------------------------------------------------

template <int Q4 /* float4 units per slot */>
__global__ __launch_bounds__(kCompactThreads) void feat_roll_kernel(float4* __restrict__ feat,
                                                                    const int32_t* __restrict__ len,
                                                                    const int32_t* __restrict__ keep, int cap,
                                                                    int budget) {
    const int row = blockIdx.x;
    const int n = min(len[row], cap);
    if (n <= 0) return;
    const size_t pl4 = (size_t)cap * Q4;
    float4* f = feat + (size_t)row * 6 * pl4;
    float4 *wl = f + 3 * pl4, *cum = f + 4 * pl4, *dec = f + 5 * pl4;
    const bool gather = n > budget;
    const int32_t* kp = keep + (size_t)row * budget;
    const int n_out = gather ? budget : n;
    constexpr int tile = kCompactThreads / Q4;  // slots per pass
    const int sl = threadIdx.x / Q4, q = threadIdx.x % Q4;
    for (int base = 0; base < n_out; base += tile) {
        const int j = base + sl;
        int src = -1;
        if (j < n_out) src = gather ? kp[j] : j;
        const bool ok = src >= 0 && src < n;
        float4 c = make_float4(0.f, 0.f, 0.f, 0.f), d = c, w = c;
        if (ok) {
            c = cum[(size_t)src * Q4 + q];
            d = dec[(size_t)src * Q4 + q];
            w = wl[(size_t)src * Q4 + q];
        }
        __syncthreads();
        if (ok) {
            cum[(size_t)j * Q4 + q] = make_float4(c.x + w.x, c.y + w.y, c.z + w.z, c.w + w.w);
            dec[(size_t)j * Q4 + q] = make_float4(fmaf(kFeatDecay, d.x, w.x), fmaf(kFeatDecay, d.y, w.y),
                                                  fmaf(kFeatDecay, d.z, w.z), fmaf(kFeatDecay, d.w, w.w));
        }
    }
    __syncthreads();  // every wL source has been read
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = threadIdx.x; t < n * Q4; t += kCompactThreads) {
        f[t] = zero;
        f[pl4 + t] = zero;
        f[2 * pl4 + t] = zero;
        f[3 * pl4 + t] = zero;
    }
}

}  // namespace fk

using namespace fk;

extern "C" fk_status fk_append(const fk_cache_desc* desc, void* K, void* V, int32_t* pos, int32_t* len,
                               const void* k_new, const void* v_new, const int32_t* pos_new, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !pos || !len || !k_new || !v_new || !pos_new) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(k_new) || !aligned16(v_new)) return FK_ERR_INVALID_ARG;
    const int chunks = desc->head_dim * (desc->dtype == FK_F32 ? 4 : 2) / 16;
    hipLaunchKernelGGL(append_kernel, dim3(desc->batch * desc->n_kv_heads), dim3(64), 0, (hipStream_t)stream, (uint4*)K,
                       (uint4*)V, pos, len, (const uint4*)k_new, (const uint4*)v_new, pos_new,
                       desc->n_kv_heads, desc->capacity, chunks);
    return launch_status();
}

extern "C" fk_status fk_compact(const fk_cache_desc* desc, void* K, void* V, int32_t* pos, int32_t* len,
                                const int32_t* keep_idx, int32_t budget, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !pos || !len || !keep_idx) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || budget > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V)) return FK_ERR_INVALID_ARG;
    const int chunks = desc->head_dim * (desc->dtype == FK_F32 ? 4 : 2) / 16;
    const int rows = desc->batch * desc->n_kv_heads;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(compact_kernel, dim3(rows, 2 * (chunks / kSliceChunks) + 1), dim3(kCompactThreads), 0, st, (uint4*)K, (uint4*)V,
                       pos, len, keep_idx, desc->capacity, budget, chunks);
    return launch_status();
}

extern "C" fk_status fk_compact_feat(const fk_cache_desc* desc, void* K, void* V, int32_t* pos, float* feat,
                                     int32_t* len, const int32_t* keep_idx, int32_t budget, void* stream) {
    fk_status s = check_desc(desc);
    if (s != FK_OK) return s;
    if (!K || !V || !pos || !feat || !len || !keep_idx) return FK_ERR_INVALID_ARG;
    if (budget <= 0 || budget > desc->capacity) return FK_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(feat)) return FK_ERR_INVALID_ARG;
    const int chunks = desc->head_dim * (desc->dtype == FK_F32 ? 4 : 2) / 16;
    const int rows = desc->batch * desc->n_kv_heads;
    const int g = desc->n_q_heads / desc->n_kv_heads;
    hipStream_t st = (hipStream_t)stream;
    // the features first: their kernel needs the lengths as they were; the cache's compaction then clamps them
    if (g <= 4)
        hipLaunchKernelGGL(feat_roll_kernel<1>, dim3(rows), dim3(kCompactThreads), 0, st, (float4*)feat, len, keep_idx,
                           desc->capacity, budget);
    else
        hipLaunchKernelGGL(feat_roll_kernel<2>, dim3(rows), dim3(kCompactThreads), 0, st, (float4*)feat, len, keep_idx,
                           desc->capacity, budget);
    hipLaunchKernelGGL(compact_kernel, dim3(rows, 2 * (chunks / kSliceChunks) + 1), dim3(kCompactThreads), 0, st, (uint4*)K, (uint4*)V,
                       pos, len, keep_idx, desc->capacity, budget, chunks);
    return launch_status();
}
