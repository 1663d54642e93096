// Device-side pieces of the per-token absmax int8 quantizer, shared by the stand-alone
// bl_quant_act kernel and by the fused decode kernel.  Every fp32 operation here is a single
// IEEE round-to-nearest operation (translation units are compiled with -ffp-contract=off).
#pragma once
#include "bl_internal.hpp"

namespace bl {

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

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
