// Internal helpers shared by the fk kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fk.h"

namespace fk {

typedef uint16_t bf16_t;  // raw bfloat16 bits

static constexpr int kWave = 64;

// ---- storage <-> fp32 ------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// 16 bytes of a row as fp32 lanes: 4 floats (fp32) or 8 floats (bf16)
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    __device__ __forceinline__ static void unpack(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    __device__ __forceinline__ static void unpack(const uint4& r, float* f) {
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
};

__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(bf16_t* p, float v) { *p = (bf16_t)f32_to_bf16(v); }

// ---- cross-lane ------------------------------------------------------------------------
// DPP controls (GCN/CDNA encoding)
static constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
static constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
static constexpr int DPP_ROW_HALF_MIRROR = 0x141; // lane i <-> 7-i inside each 8
static constexpr int DPP_ROW_MIRROR = 0x140;      // lane i <-> 15-i inside each 16

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// sum over aligned groups of W lanes (W = 8, 16, 32 or 64); every lane gets the total
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_f<DPP_QUAD_XOR1>(v);
    v += dpp_f<DPP_QUAD_XOR2>(v);
    v += dpp_f<DPP_ROW_HALF_MIRROR>(v);
    if (W >= 16) v += dpp_f<DPP_ROW_MIRROR>(v);
    if (W >= 32) v += __shfl_xor(v, 16);
    if (W >= 64) v += __shfl_xor(v, 32);
    return v;
}

// attention-feature state (Appendix B.1): six planes per (slot, query head); the carried sum decays by 0.9 per chunk
static constexpr int kFeatPlanes = 6;
static constexpr float kFeatDecay = 0.9f;

// ---- host side --------------------------------------------------------------------------
inline fk_status check_desc(const fk_cache_desc* d) {
    if (!d) return FK_ERR_INVALID_ARG;
    if (d->batch <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->capacity <= 0)
        return FK_ERR_INVALID_ARG;
    if (d->n_q_heads % d->n_kv_heads != 0) return FK_ERR_INVALID_ARG;
    if (d->dtype != FK_F32 && d->dtype != FK_BF16) return FK_ERR_UNSUPPORTED;
    if (d->head_dim != 64 && d->head_dim != 128) return FK_ERR_UNSUPPORTED;
    if (d->n_q_heads / d->n_kv_heads > 8) return FK_ERR_UNSUPPORTED;
    if (d->capacity >= (1 << 24)) return FK_ERR_UNSUPPORTED;
    return FK_OK;
}

inline fk_status launch_status() { return hipGetLastError() == hipSuccess ? FK_OK : FK_ERR_LAUNCH; }

// Raise a kernel's dynamic-LDS limit once per device (the attribute belongs to the function on the current
// device).  `done` is the caller's static flag array, one per kernel.  Concurrent first calls both set it: harmless.
static constexpr int kMaxDevices = 64;
inline bool allow_dynamic_lds(const void* kernel, size_t bytes, bool (&done)[kMaxDevices]) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (!done[dev]) {
        if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
        done[dev] = true;
    }
    return true;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace fk
