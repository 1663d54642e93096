// bl_quant_act: per-token absmax quantization of activations to int8 (the BitNet b1.58
// activation quantizer that the ternary kernels of arXiv 2410.16144 consume).
//
// One workgroup per token row; one launch takes up to 8 activation matrices (bl_quant_act_batch).
// Pass 1 reduces max|x| over the row (lane moves, then LDS across waves); pass 2 multiplies by
// inv = 127/amax, rounds to nearest-even, clips, stores int8 and reduces sum(q).  The int8 result
// must be bit-identical to the plain definition, so every fp32 operation is a single IEEE
// operation.
#include "bl_quant_device.hpp"

namespace bl {

namespace {

constexpr int kQuantThreads = 256;

constexpr int kRegVectors = 6;   // 8-element vectors a thread keeps in registers: rows up to 256 * 8 * 6 = 12288 elements

// One token row by one workgroup.  Rows of up to 12288 vector-loadable elements are read ONCE: all of a thread's
// loads are issued together and the raw values stay in registers between the absmax pass and the rounding pass.
// Longer or unaligned rows are read twice (the second read hits L2).
template <bool BF16, bool VEC>
__device__ __forceinline__ void quant_row(const void* row, int K, int Kp, int8_t* qrow, float* a_scale, int32_t* q_sum,
                                          float* s_max, int* s_sum) {
    const int tid = threadIdx.x;
    const bool in_regs = VEC && K <= kQuantThreads * 8 * kRegVectors;   // uniform
    Raw8<BF16> raw[kRegVectors];
    float amax = 0.0f;
    if (VEC && in_regs) {
#pragma unroll
        for (int i = 0; i < kRegVectors; ++i) {
            const int k = (tid + i * kQuantThreads) * 8;
            raw[i] = load_raw8<BF16>(row, k < K ? k : 0);
        }
#pragma unroll
        for (int i = 0; i < kRegVectors; ++i) {
            float v[8];
            unpack_raw8<BF16>(raw[i], v);
            if ((tid + i * kQuantThreads) * 8 < K) amax = fmaxf(amax, absmax8(v));
        }
    } else {
        amax = thread_absmax<BF16, VEC>(row, K, tid, kQuantThreads);
    }
    amax = wave_max(amax);
    if ((tid & (kWave - 1)) == 0) s_max[tid / kWave] = amax;
    __syncthreads();
    amax = s_max[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / kWave; ++w) amax = fmaxf(amax, s_max[w]);

    float inv, scale;
    quant_scales(amax, inv, scale);

    int sum = 0;
    if (VEC && in_regs) {
#pragma unroll
        for (int i = 0; i < kRegVectors; ++i) {
            const int k = (tid + i * kQuantThreads) * 8;
            float v[8];
            unpack_raw8<BF16>(raw[i], v);
            if (k < K) sum += quantize8(v, inv, qrow + k);
        }
        for (int k = K + tid; k < Kp; k += kQuantThreads) qrow[k] = 0;   // layout padding
    } else {
        sum = thread_quantize<BF16, VEC>(row, K, Kp, inv, qrow, tid, kQuantThreads);
    }
    sum = wave_sum(sum);
    if ((tid & (kWave - 1)) == 0) s_sum[tid / kWave] = sum;
    __syncthreads();
    if (tid == 0) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kQuantThreads / kWave; ++w) total += s_sum[w];
        *a_scale = scale;
        if (q_sum) *q_sum = total;
    }
}

// Up to BL_MAX_BATCH activation matrices in one launch: workgroup = one token row of one of them.
__global__ __launch_bounds__(kQuantThreads) void quant_kernel(BL_FIRST_WG_PARAMS, const QuantBatch b) {
    __shared__ float s_max[kQuantThreads / kWave];
    __shared__ int s_sum[kQuantThreads / kWave];
    const int blk = blockIdx.x;
    const QuantProblem& p = b.p[BL_PROBLEM_OF(blk)];
    const int64_t m = blk - p.first_row;
    const bool bf16 = p.flags & 1, vec = p.flags & 2;   // uniform
    const void* row = static_cast<const char*>(p.x) + m * p.ldx * (bf16 ? 2 : 4);
    int8_t* qrow = p.q + m * p.Kp;
    float* a_scale = p.a_scale + m;
    int32_t* q_sum = p.q_sum ? p.q_sum + m : nullptr;
    if (bf16) {
        if (vec) quant_row<true, true>(row, p.K, p.Kp, qrow, a_scale, q_sum, s_max, s_sum);
        else quant_row<true, false>(row, p.K, p.Kp, qrow, a_scale, q_sum, s_max, s_sum);
    } else {
        if (vec) quant_row<false, true>(row, p.K, p.Kp, qrow, a_scale, q_sum, s_max, s_sum);
        else quant_row<false, false>(row, p.K, p.Kp, qrow, a_scale, q_sum, s_max, s_sum);
    }
}

}  // namespace

hipError_t launch_quant(const QuantBatch& batch, hipStream_t s) {
    QuantBatch b = batch;
    int64_t rows = 0;
    for (int i = 0; i < b.count; ++i) {
        b.p[i].first_row = (int32_t)rows;
        rows += b.p[i].M;
    }
    if (rows > INT32_MAX) return hipErrorInvalidValue;
    struct { int v[BL_MAX_BATCH]; } first;
    for (int i = 0; i < BL_MAX_BATCH; ++i) first.v[i] = i < b.count ? b.p[i].first_row : INT32_MAX;
    quant_kernel<<<dim3((unsigned)rows), dim3(kQuantThreads), 0, s>>>(BL_FIRST_WG_ARGS(first), b);
    return hipGetLastError();
}

}  // namespace bl
