// Device-side pieces of the per-token absmax int8 quantizer, shared by the stand-alone
// bl_quant_act kernel and by the fused decode kernel.  Every fp32 operation here is a single
// IEEE round-to-nearest operation (translation units are compiled with -ffp-contract=off).
#pragma once
#include "bl_internal.hpp"

namespace bl {

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Wave-wide reductions on the vector ALU's data-parallel-primitive lane moves (no LDS round trips):
// four steps reduce each row of 16 lanes, four v_readlane pick up the rows.  The result is uniform.
#define BL_DPP(x, ctrl) __builtin_amdgcn_update_dpp(0, (x), (ctrl), 0xf, 0xf, false)
__device__ __forceinline__ float wave_max(float v) {   // v >= 0: compare the bit patterns as integers
    int x = __float_as_int(v);
    x = max(x, BL_DPP(x, 0xB1));    // quad_perm [1,0,3,2]
    x = max(x, BL_DPP(x, 0x4E));    // quad_perm [2,3,0,1]
    x = max(x, BL_DPP(x, 0x141));   // row_half_mirror
    x = max(x, BL_DPP(x, 0x140));   // row_mirror
    const int a = __builtin_amdgcn_readlane(x, 0), b = __builtin_amdgcn_readlane(x, 16);
    const int c = __builtin_amdgcn_readlane(x, 32), d = __builtin_amdgcn_readlane(x, 48);
    return __int_as_float(max(max(a, b), max(c, d)));
}

__device__ __forceinline__ int wave_sum(int x) {
    x += BL_DPP(x, 0xB1);
    x += BL_DPP(x, 0x4E);
    x += BL_DPP(x, 0x141);
    x += BL_DPP(x, 0x140);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) + __builtin_amdgcn_readlane(x, 32) +
           __builtin_amdgcn_readlane(x, 48);
}

__device__ __forceinline__ float wave_sum_f(float v) {   // a fixed tree: the same bits on every run
#define BL_DPP_F(x, ctrl) __int_as_float(BL_DPP(__float_as_int(x), (ctrl)))
    v += BL_DPP_F(v, 0xB1);
    v += BL_DPP_F(v, 0x4E);
    v += BL_DPP_F(v, 0x141);
    v += BL_DPP_F(v, 0x140);
#undef BL_DPP_F
    const int x = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(x, 0)) + __int_as_float(__builtin_amdgcn_readlane(x, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(x, 32)) + __int_as_float(__builtin_amdgcn_readlane(x, 48)));
}
#undef BL_DPP

__device__ __forceinline__ float silu(float t) { return t / (1.0f + expf(-t)); }

// q = clip(round_half_even(v * inv), -128, 127)
__device__ __forceinline__ int quant_one(float v, float inv) {
    float r = rintf(v * inv);
    r = fminf(fmaxf(r, -128.0f), 127.0f);
    return (int)r;
}

// inv = 127/amax and scale = amax/127 (one IEEE division each); a row whose inv is not finite
// (amax zero or tiny) is an all-zero token: inv = 0 makes every product +-0, scale = 0.
__device__ __forceinline__ void quant_scales(float amax, float& inv, float& scale) {
    inv = 127.0f / amax;
    const bool zero_row = !(fabsf(inv) <= 3.402823466e+38f);
    if (zero_row) inv = 0.0f;
    scale = zero_row ? 0.0f : amax / 127.0f;
}

// 8 consecutive elements starting at element k (k % 8 == 0, row base 16-byte aligned).
template <bool BF16>
__device__ __forceinline__ void load8(const void* row, int k, float (&v)[8]) {
    if constexpr (BF16) {
        uint4 u = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(row) + k);
        uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = bf16_to_f32(w[i] & 0xffffu);
            v[2 * i + 1] = bf16_to_f32(w[i] >> 16);
        }
    } else {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(row) + k);
        float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

// The same 8 elements as raw bits (kept in registers between the absmax and the quantize pass).
template <bool BF16>
struct Raw8 {
    uint4 a, b;   // bf16: a only; fp32: a, b
};

template <bool BF16>
__device__ __forceinline__ Raw8<BF16> load_raw8(const void* row, int k) {
    Raw8<BF16> r;
    if constexpr (BF16) {
        r.a = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(row) + k);
        r.b = r.a;
    } else {
        const uint4* p = reinterpret_cast<const uint4*>(static_cast<const float*>(row) + k);
        r.a = p[0];
        r.b = p[1];
    }
    return r;
}

template <bool BF16>
__device__ __forceinline__ void unpack_raw8(const Raw8<BF16>& r, float (&v)[8]) {
    if constexpr (BF16) {
        const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = bf16_to_f32(w[i] & 0xffffu);
            v[2 * i + 1] = bf16_to_f32(w[i] >> 16);
        }
    } else {
        const uint32_t w[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __uint_as_float(w[i]);
    }
}

__device__ __forceinline__ float absmax8(const float (&v)[8]) {
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(v[i]));
    return m;
}

// Quantize 8 values and store them as 8 bytes at q8; returns their sum.
__device__ __forceinline__ int quantize8(const float (&v)[8], float inv, int8_t* q8) {
    uint32_t lo = 0, hi = 0;
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int a = quant_one(v[i], inv), b = quant_one(v[4 + i], inv);
        sum += a + b;
        lo |= (uint32_t)(a & 0xff) << (8 * i);
        hi |= (uint32_t)(b & 0xff) << (8 * i);
    }
    *reinterpret_cast<uint2*>(q8) = make_uint2(lo, hi);
    return sum;
}

// The same, the 8 bytes returned instead of stored.
__device__ __forceinline__ int quantize8_packed(const float (&v)[8], float inv, uint32_t& lo, uint32_t& hi) {
    lo = hi = 0;
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int a = quant_one(v[i], inv), b = quant_one(v[4 + i], inv);
        sum += a + b;
        lo |= (uint32_t)(a & 0xff) << (8 * i);
        hi |= (uint32_t)(b & 0xff) << (8 * i);
    }
    return sum;
}

template <bool BF16>
__device__ __forceinline__ float load1(const void* row, int k) {
    if constexpr (BF16) return bf16_to_f32(static_cast<const uint16_t*>(row)[k]);
    else return static_cast<const float*>(row)[k];
}

// max |x| over this thread's share of a row (threads stride the row).  K <= BL_MAX_K: 32-bit indices.
template <bool BF16, bool VEC>
__device__ __forceinline__ float thread_absmax(const void* row, int K, int tid, int nthreads) {
    float amax = 0.0f;
    if constexpr (VEC) {
        for (int k = tid * 8; k < K; k += nthreads * 8) {
            float v[8];
            load8<BF16>(row, k, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
        }
    } else {
        for (int k = tid; k < K; k += nthreads) amax = fmaxf(amax, fabsf(load1<BF16>(row, k)));
    }
    return amax;
}

// Quantize this thread's share of a row into qrow (global or LDS); returns the thread's sum(q).
template <bool BF16, bool VEC>
__device__ __forceinline__ int thread_quantize(const void* row, int K, int Kp, float inv, int8_t* qrow,
                                               int tid, int nthreads) {
    int sum = 0;
    if constexpr (VEC) {
        for (int k = tid * 8; k < K; k += nthreads * 8) {
            float v[8];
            load8<BF16>(row, k, v);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int a = quant_one(v[i], inv), b = quant_one(v[4 + i], inv);
                sum += a + b;
                lo |= (uint32_t)(a & 0xff) << (8 * i);
                hi |= (uint32_t)(b & 0xff) << (8 * i);
            }
            *reinterpret_cast<uint2*>(qrow + k) = make_uint2(lo, hi);
        }
    } else {
        for (int k = tid; k < K; k += nthreads) {
            int a = quant_one(load1<BF16>(row, k), inv);
            sum += a;
            qrow[k] = (int8_t)a;
        }
    }
    for (int k = K + tid; k < Kp; k += nthreads) qrow[k] = 0;  // layout padding
    return sum;
}

}  // namespace bl
