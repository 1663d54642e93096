// bl_quant_act: per-token absmax quantization of activations to int8 (the BitNet b1.58
// activation quantizer that the ternary kernels of arXiv 2410.16144 consume).
//
// One workgroup per token row.  Pass 1 reduces max|x| over the row (wave shuffle, then LDS
// across waves); pass 2 re-reads the row (an L2 hit), multiplies by inv = 127/amax, rounds to
// nearest-even, clips, stores int8 and reduces sum(q).  The int8 result must be bit-identical
// to the plain definition, so every fp32 operation is a single IEEE operation.
#include "bl_quant_device.hpp"

namespace bl {

namespace {

constexpr int kQuantThreads = 256;

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

    float amax = wave_max(thread_absmax<BF16, VEC>(row, (int)K, tid, kQuantThreads));
    if ((tid & (kWave - 1)) == 0) s_max[tid / kWave] = amax;
    __syncthreads();
    amax = s_max[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / kWave; ++w) amax = fmaxf(amax, s_max[w]);

    float inv, scale;
    quant_scales(amax, inv, scale);

    int sum = wave_sum(thread_quantize<BF16, VEC>(row, (int)K, (int)Kp, inv, qrow, tid, kQuantThreads));
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
