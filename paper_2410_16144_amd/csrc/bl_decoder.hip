// The decoder block around the BitLinear products, one token at a time: what stands between the seven
// ternary projections of a layer so that a token passes through it without leaving the GPU.
//
// arXiv 2410.16144 reports tokens per second of whole models (Section 3) whose shapes Appendix A lists;
// it does not describe these operations.  They are the LLaMA-like block of BitNet b1.58: RMSNorm, rotary
// position embedding, multi-head attention over a key/value cache, SiLU-gated feed-forward, residuals.
//
// Kernels here:
//   norm_quant_kernel   residual add / SiLU gate  ->  RMSNorm  ->  per-token absmax int8 quantizer, one
//                       workgroup per token row, the row held in registers from its only read to the int8
//                       store (the quantizer is the one of bl_quant_act, bit for bit);
//   rope_table_kernel   cos / sin of every (position, frequency), fp64 arithmetic, rounded to fp32;
//   attn_chunk_kernel   one (head, chunk of 256 cache rows) per workgroup: rotate query and key, append key and
//                       value to the bf16 cache, scores, softmax within the chunk, weighted values;
//   attn_merge_kernel   one workgroup per head merges its chunks (the usual running-maximum rescaling);
//   pos_advance_kernel  the token position lives in device memory, so a captured graph replays unchanged.
// All of it is bandwidth- and latency-bound glue next to the weight streams; nothing here is a dense contraction.
#include "bl_quant_device.hpp"
#include "bitlinear_decoder.h"

namespace bl {

namespace {

// ---------------------------------------------------------------------------------------------------------------
// RMSNorm + quantizer

constexpr int kNormThreads = 1024;
constexpr int kNormWaves = kNormThreads / kWave;

struct NormArgs {
    const float* a;
    const float* b;
    float*       h;
    const float* gamma;
    int8_t*      q;
    float*       a_scale;
    int32_t*     q_sum;
    float*       y;
    int32_t      K, Kp;
    float        eps;
};

// 4 consecutive elements from element k; VEC: one 128-bit access (row base 16-byte aligned, K % 4 == 0);
// elements from K on read as zero.
template <bool VEC>
__device__ __forceinline__ void load4(const float* row, int k, int K, float (&v)[4]) {
    if constexpr (VEC) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < K) t = *reinterpret_cast<const float4*>(row + k);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = k + j < K ? row[k + j] : 0.0f;
    }
}

template <bool VEC>
__device__ __forceinline__ void store4(float* row, int k, int K, const float (&v)[4]) {
    if constexpr (VEC) {
        if (k < K) *reinterpret_cast<float4*>(row + k) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (k + j < K) row[k + j] = v[j];
    }
}

__device__ __forceinline__ float silu(float t) { return t / (1.0f + expf(-t)); }

// Thread t holds elements 4 (t + 1024 i) .. + 3, i = 0 .. NV-1.
template <int MODE, int NV, bool VEC>
__global__ __launch_bounds__(kNormThreads) void norm_quant_kernel(const NormArgs p) {
    __shared__ float s_ss[kNormWaves];
    __shared__ float s_max[kNormWaves];
    __shared__ int s_sum[kNormWaves];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int K = p.K;
    const int64_t row = (int64_t)blockIdx.x * K;
    float x[NV][4];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (tid + i * kNormThreads) * 4;
        if constexpr (MODE == BL_NORM_PLAIN) {
            load4<VEC>(p.a + row, k, K, x[i]);
        } else if constexpr (MODE == BL_NORM_RESIDUAL) {
            load4<VEC>(p.h + row, k, K, x[i]);
            if (p.a) {
                float d[4];
                load4<VEC>(p.a + row, k, K, d);
#pragma unroll
                for (int j = 0; j < 4; ++j) x[i][j] += d[j];
                store4<VEC>(p.h + row, k, K, x[i]);
            }
        } else {
            float g[4], u[4];
            load4<VEC>(p.a + row, k, K, g);
            load4<VEC>(p.b + row, k, K, u);
#pragma unroll
            for (int j = 0; j < 4; ++j) x[i][j] = silu(g[j]) * u[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) ss += x[i][j] * x[i][j];
    }
    ss = wave_sum_f(ss);
    if (lane == 0) s_ss[wave] = ss;
    __syncthreads();
    float total = 0.0f;
#pragma unroll
    for (int w = 0; w < kNormWaves; ++w) total += s_ss[w];
    const float r = 1.0f / sqrtf(total / (float)K + p.eps);

    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (tid + i * kNormThreads) * 4;
        float g[4];
        load4<VEC>(p.gamma, k, K, g);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[i][j] = (x[i][j] * r) * g[j];
            amax = fmaxf(amax, fabsf(x[i][j]));
        }
        if (p.y) store4<VEC>(p.y + row, k, K, x[i]);
    }
    if (!p.q) return;   // uniform: the final norm of a model quantizes nothing
    amax = wave_max(amax);
    if (lane == 0) s_max[wave] = amax;
    __syncthreads();
    amax = s_max[0];
#pragma unroll
    for (int w = 1; w < kNormWaves; ++w) amax = fmaxf(amax, s_max[w]);
    float inv, scale;
    quant_scales(amax, inv, scale);

    int8_t* qrow = p.q + (int64_t)blockIdx.x * p.Kp;
    int sum = 0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (tid + i * kNormThreads) * 4;
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int v = quant_one(x[i][j], inv);   // elements from K on are zero and quantize to zero
            sum += v;
            word |= (uint32_t)(v & 0xff) << (8 * j);
        }
        if (k < K) *reinterpret_cast<uint32_t*>(qrow + k) = word;
    }
    for (int k = (K + 3) / 4 * 4 + tid * 4; k < p.Kp; k += kNormThreads * 4) *reinterpret_cast<uint32_t*>(qrow + k) = 0;
    sum = wave_sum(sum);
    if (lane == 0) s_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kNormWaves; ++w) t += s_sum[w];
        p.a_scale[blockIdx.x] = scale;
        if (p.q_sum) p.q_sum[blockIdx.x] = t;
    }
}

template <int MODE, int NV>
hipError_t launch_norm_nv(const NormArgs& p, int M, bool vec, hipStream_t s) {
    if (vec) norm_quant_kernel<MODE, NV, true><<<dim3((unsigned)M), dim3(kNormThreads), 0, s>>>(p);
    else norm_quant_kernel<MODE, NV, false><<<dim3((unsigned)M), dim3(kNormThreads), 0, s>>>(p);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_norm_mode(const NormArgs& p, int M, bool vec, hipStream_t s) {
    const int per_thread = (p.K + kNormThreads * 4 - 1) / (kNormThreads * 4);
    if (per_thread <= 1) return launch_norm_nv<MODE, 1>(p, M, vec, s);
    if (per_thread <= 2) return launch_norm_nv<MODE, 2>(p, M, vec, s);
    if (per_thread <= 4) return launch_norm_nv<MODE, 4>(p, M, vec, s);
    if (per_thread <= 8) return launch_norm_nv<MODE, 8>(p, M, vec, s);
    if (per_thread <= 12) return launch_norm_nv<MODE, 12>(p, M, vec, s);
    return hipErrorInvalidValue;
}
static_assert(BL_NORM_MAX_K == 12 * kNormThreads * 4, "the longest row fills 12 vectors per thread");

// ---------------------------------------------------------------------------------------------------------------
// Rotary table

__global__ __launch_bounds__(256) void rope_table_kernel(float2* table, int half, int64_t entries, double theta) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= entries) return;
    const int64_t pos = idx / half;
    const int i = (int)(idx - pos * half);
    const double angle = (double)pos * pow(theta, -(double)i / (double)half);   // theta^(-2 i / head_dim)
    table[idx] = make_float2((float)cos(angle), (float)sin(angle));
}

// ---------------------------------------------------------------------------------------------------------------
// Attention over the cache

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kChunk = BL_ATTN_CHUNK;
static_assert(kChunk == kAttnThreads, "one cache row per thread in the score pass");

struct AttnArgs {
    const float*   q_lin;
    const float*   k_lin;
    const float*   v_lin;
    const int32_t* pos;
    const float2*  rope;
    uint16_t*      k_cache;
    uint16_t*      v_cache;
    float*         out;
    float*         scratch;     // [n_heads][chunks][head_dim + 2]: weighted values, running maximum, weight sum
    int32_t        n_heads, head_dim, max_pos, chunks;
};

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {   // nearest, ties to even; finite inputs
    const uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ float block_max(float v, float* s_red, int wave, int lane) {   // any sign
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();   // the previous use of s_red has been read
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float m = s_red[0];
#pragma unroll
    for (int w = 1; w < kAttnWaves; ++w) m = fmaxf(m, s_red[w]);
    return m;
}

__device__ __forceinline__ float block_sum(float v, float* s_red, int wave, int lane) {
    v = wave_sum_f(v);
    __syncthreads();
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) t += s_red[w];
    return t;
}

__global__ __launch_bounds__(kAttnThreads) void attn_chunk_kernel(const AttnArgs p) {
    __shared__ float s_q[BL_ATTN_MAX_HEAD_DIM];       // rotated query, pre-scaled by 1 / sqrt(head_dim)
    __shared__ float s_newk[BL_ATTN_MAX_HEAD_DIM];    // the token's own key and value as the cache holds them
    __shared__ float s_newv[BL_ATTN_MAX_HEAD_DIM];
    __shared__ float s_w[kChunk];                     // softmax numerators of the chunk's rows
    __shared__ float s_o[kAttnThreads];               // partial weighted values, [part][element]
    __shared__ float s_red[kAttnWaves];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int head = blockIdx.x, chunk = blockIdx.y;
    const int d = p.head_dim, half = d / 2;
    const int hidden = p.n_heads * d;
    const int pos = *p.pos;
    if (pos < 0 || pos >= p.max_pos) return;            // uniform
    const int j0 = chunk * kChunk;
    if (j0 > pos) return;                               // uniform: nothing cached this far yet
    const int rows = min(kChunk, pos + 1 - j0);
    const bool owner = pos < j0 + kChunk;               // uniform: this chunk holds the token's own row
    const float scale = 1.0f / sqrtf((float)d);

    if (tid < half) {
        const float2 cs = p.rope[(int64_t)pos * half + tid];
        const float a = p.q_lin[head * d + tid], b = p.q_lin[head * d + tid + half];
        s_q[tid] = (a * cs.x - b * cs.y) * scale;
        s_q[tid + half] = (a * cs.y + b * cs.x) * scale;
        if (owner) {
            const float ka = p.k_lin[head * d + tid], kb = p.k_lin[head * d + tid + half];
            const uint16_t k0 = f32_to_bf16(ka * cs.x - kb * cs.y), k1 = f32_to_bf16(ka * cs.y + kb * cs.x);
            const uint16_t v0 = f32_to_bf16(p.v_lin[head * d + tid]), v1 = f32_to_bf16(p.v_lin[head * d + tid + half]);
            uint16_t* krow = p.k_cache + (int64_t)pos * hidden + head * d;
            uint16_t* vrow = p.v_cache + (int64_t)pos * hidden + head * d;
            krow[tid] = k0; krow[tid + half] = k1;
            vrow[tid] = v0; vrow[tid + half] = v1;
            s_newk[tid] = bf16_to_f32(k0); s_newk[tid + half] = bf16_to_f32(k1);
            s_newv[tid] = bf16_to_f32(v0); s_newv[tid + half] = bf16_to_f32(v1);
        }
    }
    __syncthreads();

    // scores: thread t takes cache row j0 + t (its d values are contiguous)
    float score = -INFINITY;
    if (tid < rows) {
        const int j = j0 + tid;
        float acc = 0.0f;
        if (j == pos) {
            for (int e = 0; e < d; ++e) acc += s_q[e] * s_newk[e];
        } else {
            const uint16_t* krow = p.k_cache + (int64_t)j * hidden + head * d;
            auto mac2 = [&](uint32_t pair, int e) {
                acc += s_q[e] * bf16_to_f32(pair & 0xffffu);
                acc += s_q[e + 1] * bf16_to_f32(pair >> 16);
            };
            if (d % 8 == 0) {                                   // uniform: 128-bit loads
                for (int c = 0; c < d / 8; ++c) {
                    const uint4 u = reinterpret_cast<const uint4*>(krow)[c];
                    mac2(u.x, 8 * c); mac2(u.y, 8 * c + 2); mac2(u.z, 8 * c + 4); mac2(u.w, 8 * c + 6);
                }
            } else {                                            // head_dim % 4 == 0: 64-bit loads
                for (int c = 0; c < d / 4; ++c) {
                    const uint2 u = reinterpret_cast<const uint2*>(krow)[c];
                    mac2(u.x, 4 * c); mac2(u.y, 4 * c + 2);
                }
            }
        }
        score = acc;
    }
    const float m = block_max(score, s_red, wave, lane);
    const float w = tid < rows ? expf(score - m) : 0.0f;
    s_w[tid] = w;
    const float l = block_sum(w, s_red, wave, lane);    // its barriers also publish s_w

    // weighted values: thread (part, e) sums rows part, part + parts, ... for element e; a row's d values are
    // consecutive 16-bit loads across the threads of a part
    const int parts = kAttnThreads / d;                 // >= 1: head_dim <= 256
    const int part = tid / d, e = tid - part * d;
    float o = 0.0f;
    if (part < parts) {
        for (int t = part; t < rows; t += parts) {
            const int j = j0 + t;
            const float v = j == pos ? s_newv[e] : bf16_to_f32(p.v_cache[(int64_t)j * hidden + head * d + e]);
            o += s_w[t] * v;
        }
    }
    s_o[tid] = o;
    __syncthreads();
    float* dst = p.scratch + ((int64_t)head * p.chunks + chunk) * (d + 2);
    if (tid < d) {
        float t = 0.0f;
        for (int q = 0; q < parts; ++q) t += s_o[q * d + tid];
        dst[tid] = t;
    }
    if (tid == 0) {
        dst[d] = m;
        dst[d + 1] = l;
    }
}

__global__ __launch_bounds__(kAttnThreads) void attn_merge_kernel(const AttnArgs p) {
    const int tid = threadIdx.x, head = blockIdx.x;
    const int d = p.head_dim;
    const int pos = *p.pos;
    if (pos < 0 || pos >= p.max_pos) return;            // uniform
    const int used = pos / kChunk + 1;                   // chunks that hold rows 0 .. pos
    const float* src = p.scratch + (int64_t)head * p.chunks * (d + 2);
    if (tid >= d) return;
    float m = -INFINITY;
    for (int c = 0; c < used; ++c) m = fmaxf(m, src[c * (d + 2) + d]);
    float l = 0.0f, o = 0.0f;
    for (int c = 0; c < used; ++c) {
        const float f = expf(src[c * (d + 2) + d] - m);
        l += f * src[c * (d + 2) + d + 1];
        o += f * src[c * (d + 2) + tid];
    }
    p.out[head * d + tid] = o / l;
}

__global__ void pos_advance_kernel(int32_t* pos) {
    if (threadIdx.x == 0) *pos = *pos + 1;
}

}  // namespace

hipError_t launch_norm_quant(const bl_norm_quant_args& a, hipStream_t s) {
    NormArgs p;
    p.a = a.a_dev; p.b = a.b_dev; p.h = a.h_dev; p.gamma = a.gamma_dev;
    p.q = a.q_dev; p.a_scale = a.a_scale_dev; p.q_sum = a.q_sum_dev; p.y = a.y_dev;
    p.K = (int32_t)a.K; p.Kp = (int32_t)a.Kp; p.eps = a.eps;
    auto ok16 = [](const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; };
    const bool vec = a.K % 4 == 0 && ok16(a.a_dev) && ok16(a.b_dev) && ok16(a.h_dev) && ok16(a.gamma_dev) && ok16(a.y_dev);
    switch (a.mode) {
        case BL_NORM_PLAIN: return launch_norm_mode<BL_NORM_PLAIN>(p, a.M, vec, s);
        case BL_NORM_RESIDUAL: return launch_norm_mode<BL_NORM_RESIDUAL>(p, a.M, vec, s);
        case BL_NORM_GATED: return launch_norm_mode<BL_NORM_GATED>(p, a.M, vec, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_rope_table(float* table, int head_dim, int max_pos, double theta, hipStream_t s) {
    const int half = head_dim / 2;
    const int64_t entries = (int64_t)max_pos * half;
    const int64_t blocks = (entries + 255) / 256;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    rope_table_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(reinterpret_cast<float2*>(table), half, entries, theta);
    return hipGetLastError();
}

int attn_chunks(int max_pos) { return (max_pos + kChunk - 1) / kChunk; }

hipError_t launch_attn_decode(const bl_attn_args& a, hipStream_t s) {
    AttnArgs p;
    p.q_lin = a.q_lin_dev; p.k_lin = a.k_lin_dev; p.v_lin = a.v_lin_dev; p.pos = a.pos_dev;
    p.rope = reinterpret_cast<const float2*>(a.rope_table_dev);
    p.k_cache = a.k_cache_dev; p.v_cache = a.v_cache_dev; p.out = a.out_dev;
    p.scratch = static_cast<float*>(a.scratch_dev);
    p.n_heads = a.n_heads; p.head_dim = a.head_dim; p.max_pos = a.max_pos; p.chunks = attn_chunks(a.max_pos);
    attn_chunk_kernel<<<dim3((unsigned)a.n_heads, (unsigned)p.chunks), dim3(kAttnThreads), 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    attn_merge_kernel<<<dim3((unsigned)a.n_heads), dim3(kAttnThreads), 0, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_pos_advance(int32_t* pos, hipStream_t s) {
    pos_advance_kernel<<<dim3(1), dim3(64), 0, s>>>(pos);
    return hipGetLastError();
}

}  // namespace bl
