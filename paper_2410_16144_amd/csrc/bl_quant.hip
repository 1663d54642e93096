// bl_quant_act: per-token absmax quantization of activations to int8 (the BitNet b1.58
// activation quantizer that the ternary kernels of arXiv 2410.16144 consume).
//
// One workgroup per token row.  Pass 1 reduces max|x| over the row (wave shuffle, then LDS
// across waves); pass 2 re-reads the row (an L2 hit), multiplies by inv = 127/amax, rounds to
// nearest-even, clips, stores int8 and reduces sum(q).  Every fp32 operation is a single IEEE
// round-to-nearest operation (this file is compiled with -ffp-contract=off): the int8 result
// must be bit-identical to the plain definition.
#include "bl_internal.hpp"

namespace bl {

namespace {

constexpr int kQuantThreads = 256;

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

__device__ __forceinline__ int quant_one(float v, float inv) {
    float r = rintf(v * inv);
    r = fminf(fmaxf(r, -128.0f), 127.0f);
    return (int)r;
}

// Loads 8 consecutive elements starting at element index k (k % 8 == 0, row base 16-byte aligned).
template <bool BF16>
__device__ __forceinline__ void load8(const void* row, int64_t k, float (&v)[8]) {
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
__device__ __forceinline__ float load1(const void* row, int64_t k) {
    if constexpr (BF16) return bf16_to_f32(static_cast<const uint16_t*>(row)[k]);
    else return static_cast<const float*>(row)[k];
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kQuantThreads) void quant_kernel(const void* __restrict__ x, int64_t K, int64_t ldx,
                                                              int64_t Kp, int8_t* __restrict__ q,
                                                              float* __restrict__ a_scale,
                                                              int32_t* __restrict__ q_sum) {
    __shared__ float s_max[kQuantThreads / kWave];
    __shared__ int s_sum[kQuantThreads / kWave];
    const int tid = threadIdx.x;
    const int64_t m = blockIdx.x;
    const void* row = static_cast<const char*>(x) + m * ldx * (BF16 ? 2 : 4);
    int8_t* qrow = q + m * Kp;

    // ---- pass 1: amax = max_k |x|
    float amax = 0.0f;
    if constexpr (VEC) {
        for (int64_t k = (int64_t)tid * 8; k < K; k += kQuantThreads * 8) {
            float v[8];
            load8<BF16>(row, k, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
        }
    } else {
        for (int64_t k = tid; k < K; k += kQuantThreads) amax = fmaxf(amax, fabsf(load1<BF16>(row, k)));
    }
    amax = wave_max(amax);
    if ((tid & (kWave - 1)) == 0) s_max[tid / kWave] = amax;
    __syncthreads();
    amax = s_max[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / kWave; ++w) amax = fmaxf(amax, s_max[w]);

    // ---- scales: one IEEE division each
    float inv = 127.0f / amax;
    const bool zero_row = !(fabsf(inv) <= 3.402823466e+38f);  // inf (amax tiny or 0)
    if (zero_row) inv = 0.0f;                                  // every product becomes +-0 -> q = 0
    const float scale = zero_row ? 0.0f : amax / 127.0f;

    // ---- pass 2: q = clip(rne(x * inv)); sum(q)
    int sum = 0;
    if constexpr (VEC) {
        for (int64_t k = (int64_t)tid * 8; k < K; k += kQuantThreads * 8) {
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
        for (int64_t k = tid; k < K; k += kQuantThreads) {
            int a = quant_one(load1<BF16>(row, k), inv);
            sum += a;
            qrow[k] = (int8_t)a;
        }
    }
    for (int64_t k = K + tid; k < Kp; k += kQuantThreads) qrow[k] = 0;  // layout padding

    sum = wave_sum(sum);
    if ((tid & (kWave - 1)) == 0) s_sum[tid / kWave] = sum;
    __syncthreads();
    if (tid == 0) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kQuantThreads / kWave; ++w) total += s_sum[w];
        a_scale[m] = scale;
        if (q_sum) q_sum[m] = total;
    }
}

}  // namespace

hipError_t launch_quant(const void* x, int is_bf16, int64_t M, int64_t K, int64_t ldx, int64_t Kp, int8_t* q,
                        float* a_scale, int32_t* q_sum, hipStream_t s) {
    const bool vec = (K % 8 == 0) && (ldx % 8 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
    dim3 grid((unsigned)M), block(kQuantThreads);
    if (is_bf16) {
        if (vec) quant_kernel<true, true><<<grid, block, 0, s>>>(x, K, ldx, Kp, q, a_scale, q_sum);
        else quant_kernel<true, false><<<grid, block, 0, s>>>(x, K, ldx, Kp, q, a_scale, q_sum);
    } else {
        if (vec) quant_kernel<false, true><<<grid, block, 0, s>>>(x, K, ldx, Kp, q, a_scale, q_sum);
        else quant_kernel<false, false><<<grid, block, 0, s>>>(x, K, ldx, Kp, q, a_scale, q_sum);
    }
    return hipGetLastError();
}

}  // namespace bl
