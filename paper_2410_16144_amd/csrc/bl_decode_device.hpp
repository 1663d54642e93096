// Device-side pieces shared by the decode kernels: the per-tile multiply-accumulate over packed
// codes and the in-kernel activation quantizers (Section 2 of arXiv 2410.16144, I2_S form).
#pragma once
#include "bl_quant_device.hpp"

namespace bl {

constexpr int kWaves = 16;            // waves per workgroup
constexpr int kThreads = kWaves * kWave;
constexpr int kInFlight = 8;          // weight tiles a wave keeps in flight

template <int M>
struct Acc {
    int lo[M];  // sums of q * code
    int hi[M];  // sums of q * (4 * code)
};

// One 64x64 tile: w = this lane's 16 bytes, qk = the tile's activations of token 0 (16 words),
// q_stride_words = distance between token rows.  Works for global (scalar loads) and LDS pointers.
template <int M, typename QPtr>
__device__ __forceinline__ void tile_mac(const uint4& w, QPtr qk, int q_stride_words, Acc<M>& a) {
    const uint32_t word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t d = word[s];
        const uint32_t e = d >> 4;
        const int c0 = (int)(d & 0x03030303u);  // k-offsets 0..3   (x1)
        const int c1 = (int)(d & 0x0c0c0c0cu);  // k-offsets 4..7   (x4)
        const int c2 = (int)(e & 0x03030303u);  // k-offsets 8..11  (x1)
        const int c3 = (int)(e & 0x0c0c0c0cu);  // k-offsets 12..15 (x4)
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int4 qv = *reinterpret_cast<const int4*>(qk + m * q_stride_words + 4 * s);
            a.lo[m] = __builtin_amdgcn_sdot4(c0, qv.x, a.lo[m], false);
            a.hi[m] = __builtin_amdgcn_sdot4(c1, qv.y, a.hi[m], false);
            a.lo[m] = __builtin_amdgcn_sdot4(c2, qv.z, a.lo[m], false);
            a.hi[m] = __builtin_amdgcn_sdot4(c3, qv.w, a.hi[m], false);
        }
    }
}

// Quantize M token rows into LDS; per-token scale and partial sums of q are left in s_f / s_i (LDS).
// General form: the row is read twice (the second read hits L1/L2).
template <int M, bool BF16, bool VEC>
__device__ __forceinline__ void quantize_rows_to_lds(const DecodeProblem& p, int8_t* lds_q, float* s_f, int* s_i,
                                                     int tid, int lane, int wave) {
    const int K = p.K, Kp = p.KC * kTileK;
    const char* x = static_cast<const char*>(p.x);
    const int64_t row_bytes = p.ldx * (BF16 ? 2 : 4);
    float amax[M];
#pragma unroll
    for (int m = 0; m < M; ++m) amax[m] = wave_max(thread_absmax<BF16, VEC>(x + m * row_bytes, K, tid, kThreads));
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) s_f[m * kWaves + wave] = amax[m];
    }
    __syncthreads();
    int sum[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        float am = s_f[m * kWaves];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) am = fmaxf(am, s_f[m * kWaves + w]);
        float inv, scale;
        quant_scales(am, inv, scale);
        sum[m] = wave_sum(thread_quantize<BF16, VEC>(x + m * row_bytes, K, Kp, inv, lds_q + m * Kp, tid, kThreads));
        if (tid == 0) s_f[M * kWaves + m] = scale;
    }
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) s_i[m * kWaves + wave] = sum[m];
    }
    __syncthreads();
}

// One token whose row fits two 8-element vectors per thread (K <= 16384, vector-loadable): the raw
// inputs are loaded by the caller BEFORE the weight tiles (loads retire in order, so waiting for x
// then leaves the 8 weight loads in flight) and stay in registers between the two passes.
template <bool BF16>
__device__ __forceinline__ void quantize_row_from_regs(const Raw8<BF16>& r0, const Raw8<BF16>& r1, bool h0, bool h1,
                                                       int K, int Kp, int8_t* lds_q, float* s_f, int* s_i, int tid,
                                                       int lane, int wave) {
    float am;
    {
        float v[8];
        unpack_raw8<BF16>(r0, v);
        am = h0 ? absmax8(v) : 0.0f;
        unpack_raw8<BF16>(r1, v);
        am = fmaxf(am, h1 ? absmax8(v) : 0.0f);
    }
    am = wave_max(am);
    if (lane == 0) s_f[wave] = am;
    __syncthreads();
    am = s_f[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) am = fmaxf(am, s_f[w]);
    float inv, scale;
    quant_scales(am, inv, scale);
    int sum = 0;
    {
        float v[8];
        unpack_raw8<BF16>(r0, v);
        if (h0) sum += quantize8(v, inv, lds_q + tid * 8);
        unpack_raw8<BF16>(r1, v);
        if (h1) sum += quantize8(v, inv, lds_q + (tid + kThreads) * 8);
    }
    for (int k = K + tid; k < Kp; k += kThreads) lds_q[k] = 0;
    sum = wave_sum(sum);
    if (tid == 0) s_f[kWaves] = scale;
    if (lane == 0) s_i[wave] = sum;
    __syncthreads();
}

}  // namespace bl
