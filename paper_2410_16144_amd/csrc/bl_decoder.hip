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
//   attn_chunk_kernel   one (head, chunk of 64 cache rows) per workgroup: rotate query and key, append key and
//                       value to the bf16 cache, scores, softmax within the chunk, weighted values;
//                       the head's workgroup that finishes last merges its chunks (running-maximum rescaling);
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
    float2*      scratch;   // wide form: per row kWideMaxSlices x (sum of squares, absmax of x * gamma)
    int32_t      pieces;    // pre-multiplied form: pairs in scratch (read only)
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
    // short rows: the norm weights are requested with the row, before the first barrier (one memory round trip
    // instead of two); long rows have no registers to spare for that
    constexpr bool kGammaEarly = NV <= 4;
    float gam[kGammaEarly ? NV : 1][4];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = (tid + i * kNormThreads) * 4;
        if constexpr (kGammaEarly) load4<VEC>(p.gamma, k, K, gam[i]);
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
        if constexpr (kGammaEarly) {
#pragma unroll
            for (int j = 0; j < 4; ++j) g[j] = gam[i][j];
        } else {
            load4<VEC>(p.gamma, k, K, g);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[i][j] = (x[i][j] * g[j]) * r;
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

// Long rows (K >= kWideMinK, with scratch memory from the caller): one workgroup is bound by its compute unit's ALU on
// such a row (45568 gated elements: 20 us), so the row is cut into slices of 2048 elements, one workgroup each, and the
// work into two launches with the grid-wide reductions between them:
//   1. x (residual add stored, or the gate), z = x * gamma; per slice sum(x^2) and max|z| to scratch; sum(q) zeroed;
//   2. every workgroup adds up the slices' figures in the same order (so all get the same bits): r, and max|y| =
//      max|z| * r -- rounding is monotone and r > 0, so the largest |z| gives the largest |z * r|, which is why y is
//      defined as (x * gamma) * r in that order; then y and the codes of its slice; sum(q) by integer atomics.
constexpr int kWideThreads = 256;
constexpr int kWideSlice = kWideThreads * 8;
constexpr int kWideMinK = 16384;
constexpr int kWideMaxSlices = BL_NORM_MAX_K / kWideSlice;
static_assert(kWideMaxSlices * sizeof(float2) <= BL_NORM_SCRATCH_BYTES, "a row's partial figures fit its scratch");

template <int MODE, bool VEC>
__device__ __forceinline__ void wide_inputs(const NormArgs& p, int64_t row, int k, int K, bool second_pass, float (&x)[4]) {
    if constexpr (MODE == BL_NORM_PLAIN || MODE == BL_NORM_PREMULTIPLIED) {
        load4<VEC>(p.a + row, k, K, x);
    } else if constexpr (MODE == BL_NORM_RESIDUAL) {
        load4<VEC>(p.h + row, k, K, x);
        if (p.a && !second_pass) {     // the first launch adds and stores; the second finds the sum in h
            float d[4];
            load4<VEC>(p.a + row, k, K, d);
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] += d[j];
            store4<VEC>(p.h + row, k, K, x);
        }
    } else {
        float g[4], u[4];
        load4<VEC>(p.a + row, k, K, g);
        load4<VEC>(p.b + row, k, K, u);
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = silu(g[j]) * u[j];
    }
}

template <int MODE, bool VEC>
__global__ __launch_bounds__(kWideThreads) void norm_wide_stats_kernel(const NormArgs p) {
    __shared__ float s_ss[kWideThreads / kWave], s_max[kWideThreads / kWave];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int K = p.K, slice = blockIdx.x;
    const int64_t row = (int64_t)blockIdx.y * K;
    float ss = 0.0f, amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int k = slice * kWideSlice + (tid + i * kWideThreads) * 4;
        float x[4], g[4];
        load4<VEC>(p.gamma, k, K, g);
        wide_inputs<MODE, VEC>(p, row, k, K, false, x);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ss += x[j] * x[j];
            amax = fmaxf(amax, fabsf(x[j] * g[j]));
        }
    }
    ss = wave_sum_f(ss);
    amax = wave_max(amax);
    if (lane == 0) { s_ss[wave] = ss; s_max[wave] = amax; }
    __syncthreads();
    if (tid == 0) {
        static_assert(kWideThreads / kWave == 4, "four partial figures");
        p.scratch[(int64_t)blockIdx.y * kWideMaxSlices + slice] =
            make_float2((s_ss[0] + s_ss[1]) + (s_ss[2] + s_ss[3]), fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3])));
        if (slice == 0 && p.q_sum) p.q_sum[blockIdx.y] = 0;
    }
}

template <int MODE, bool VEC>
__global__ __launch_bounds__(kWideThreads) void norm_wide_quant_kernel(const NormArgs p) {
    __shared__ int s_sum[kWideThreads / kWave];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int K = p.K, slice = blockIdx.x, slices = gridDim.x;
    const int64_t row = (int64_t)blockIdx.y * K;
    float total = 0.0f, amax_z = 0.0f;
    if constexpr (MODE == BL_NORM_PREMULTIPLIED) {
        // the pieces of a gated launch, hundreds of them: every workgroup adds them up the same way (thread t takes
        // pieces t, t + 256, ...; lanes, then waves) and so arrives at the same bits
        __shared__ float s_tot[kWideThreads / kWave], s_amax[kWideThreads / kWave];
        for (int i = tid; i < p.pieces; i += kWideThreads) {
            const float2 f = p.scratch[i];
            total += f.x;
            amax_z = fmaxf(amax_z, f.y);
        }
        total = wave_sum_f(total);
        amax_z = wave_max(amax_z);
        if (lane == 0) { s_tot[wave] = total; s_amax[wave] = amax_z; }
        __syncthreads();
        total = (s_tot[0] + s_tot[1]) + (s_tot[2] + s_tot[3]);
        amax_z = fmaxf(fmaxf(s_amax[0], s_amax[1]), fmaxf(s_amax[2], s_amax[3]));
    } else {
        const float2* part = p.scratch + (int64_t)blockIdx.y * kWideMaxSlices;
        for (int g = 0; g < slices; ++g) {      // the same order in every workgroup
            const float2 f = part[g];
            total += f.x;
            amax_z = fmaxf(amax_z, f.y);
        }
    }
    const float r = 1.0f / sqrtf(total / (float)K + p.eps);
    float inv, scale;
    quant_scales(amax_z * r, inv, scale);
    int8_t* qrow = p.q ? p.q + (int64_t)blockIdx.y * p.Kp : nullptr;
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int k = slice * kWideSlice + (tid + i * kWideThreads) * 4;
        float x[4], g[4] = {1.0f, 1.0f, 1.0f, 1.0f};
        if constexpr (MODE != BL_NORM_PREMULTIPLIED) load4<VEC>(p.gamma, k, K, g);
        wide_inputs<MODE, VEC>(p, row, k, K, true, x);
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = MODE == BL_NORM_PREMULTIPLIED ? x[j] * r : (x[j] * g[j]) * r;
            const int v = quant_one(x[j], inv);
            sum += v;
            word |= (uint32_t)(v & 0xff) << (8 * j);
        }
        if (p.y) store4<VEC>(p.y + row, k, K, x);
        if (qrow && k < K) *reinterpret_cast<uint32_t*>(qrow + k) = word;
    }
    if (!qrow) return;   // uniform
    if (slice == slices - 1)
        for (int k = (K + 3) / 4 * 4 + tid * 4; k < p.Kp; k += kWideThreads * 4) *reinterpret_cast<uint32_t*>(qrow + k) = 0;
    sum = wave_sum(sum);
    if (lane == 0) s_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        const int part = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
        if constexpr (MODE == BL_NORM_PREMULTIPLIED) {
            // no earlier launch of this call could zero sum(q), so the slices meet in one 64-bit word behind the
            // pieces: slice count in the high bits, signed sum in the low 40; the slice that completes the count
            // writes the total and puts the word back to zero (it is zero before the first call)
            if (p.q_sum) {
                unsigned long long* word = reinterpret_cast<unsigned long long*>(p.scratch + p.pieces);
                const unsigned long long add = (1ull << 40) + (unsigned long long)(long long)part;
                const unsigned long long now =
                    __hip_atomic_fetch_add(word, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
                const long long sum = (long long)(now << 24) >> 24;
                if ((long long)((now - (unsigned long long)sum) >> 40) == slices) {
                    p.q_sum[0] = (int)sum;
                    __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        } else if (p.q_sum) {
            atomicAdd(p.q_sum + blockIdx.y, part);
        }
        if (slice == 0) p.a_scale[blockIdx.y] = scale;
    }
}

// The pre-multiplied form: the figures of the first launch are there already (a gated product's epilogue left them).
hipError_t launch_norm_premultiplied(const NormArgs& p, bool vec, hipStream_t s) {
    const dim3 grid((unsigned)((p.K + kWideSlice - 1) / kWideSlice), 1u), block(kWideThreads);
    if (vec) norm_wide_quant_kernel<BL_NORM_PREMULTIPLIED, true><<<grid, block, 0, s>>>(p);
    else norm_wide_quant_kernel<BL_NORM_PREMULTIPLIED, false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_norm_wide(const NormArgs& p, int M, bool vec, hipStream_t s) {
    const dim3 grid((unsigned)((p.K + kWideSlice - 1) / kWideSlice), (unsigned)M), block(kWideThreads);
    if (vec) norm_wide_stats_kernel<MODE, true><<<grid, block, 0, s>>>(p);
    else norm_wide_stats_kernel<MODE, false><<<grid, block, 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (vec) norm_wide_quant_kernel<MODE, true><<<grid, block, 0, s>>>(p);
    else norm_wide_quant_kernel<MODE, false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

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
static_assert(kChunk == kWave, "the chunk's softmax runs in one wavefront");

struct AttnArgs {
    const float*   q_lin;
    const float*   k_lin;
    const float*   v_lin;
    const int32_t* pos;
    const float2*  rope;
    uint16_t*      k_cache;
    uint16_t*      v_cache;
    float*         out;
    float*         scratch;     // per query [n_heads][chunks][head_dim + 2] (weighted values, maximum, sum), then n_heads counters
    int32_t        n_heads, head_dim, max_pos, chunks;
    // several consecutive tokens (a prompt): pos is null, query z has position pos0 + z, its own row of q_lin and out
    // and its own part of scratch; keys and values are in the cache already (kv_append_kernel)
    int32_t        pos0;
    int64_t        scratch_stride;   // floats per query
};

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {   // nearest, ties to even; finite inputs
    const uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// W bf16 values as one register vector: 128 bits for W = 8, 64 bits for W = 4.
template <int W> struct CacheVec;
template <> struct CacheVec<8> { typedef uint4 type; };
template <> struct CacheVec<4> { typedef uint2 type; };

template <int W>
__device__ __forceinline__ void unpack_bf16(const typename CacheVec<W>::type& u, float (&f)[W]) {
    const uint32_t* w = reinterpret_cast<const uint32_t*>(&u);
#pragma unroll
    for (int i = 0; i < W / 2; ++i) {
        f[2 * i] = bf16_to_f32(w[i] & 0xffffu);
        f[2 * i + 1] = bf16_to_f32(w[i] >> 16);
    }
}

// One head's chunks merged by one workgroup: out = sum_c f_c o_c / sum_c f_c l_c with f_c = exp(m_c - max m) over the
// chunks that hold rows 0 .. pos.  The chunks' maxima and sums are read one per thread; the factors go through LDS.
// A value another workgroup of this launch has published (see publish below): read where it was deposited, by a
// device-scope atomic load (it does not take its value from this die's cache).
__device__ __forceinline__ float read_published(float* at) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<unsigned int*>(at), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

__device__ __forceinline__ void attn_merge(const AttnArgs& p, float* scratch, float* out, int head, int used, float* s_f,
                                           float* s_red) {
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int d = p.head_dim;
    float* base = scratch + (int64_t)head * p.chunks * (d + 2);
    const auto src = [&](int i) { return read_published(base + i); };
    float m = -INFINITY;
    for (int c = tid; c < used; c += kAttnThreads) m = fmaxf(m, src(c * (d + 2) + d));
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    static_assert(kAttnWaves == 4, "four partial maxima");
    float l = 0.0f, o = 0.0f;
    for (int c0 = 0; c0 < used; c0 += kAttnThreads) {   // one pass unless the context exceeds 256 chunks
        __syncthreads();                                // s_f and s_red of the previous pass have been read
        const int c = c0 + tid;
        float f = 0.0f, fl = 0.0f;
        if (c < used) {
            f = expf(src(c * (d + 2) + d) - m);
            fl = f * src(c * (d + 2) + d + 1);
        }
        s_f[tid] = f;
        fl = wave_sum_f(fl);
        if (lane == 0) s_red[wave] = fl;
        __syncthreads();
        l += (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
        const int n = min(kAttnThreads, used - c0);
        if (tid < d) {
#pragma unroll 4
            for (int i = 0; i < n; ++i) o += s_f[i] * src((c0 + i) * (d + 2) + tid);
        }
    }
    if (tid < d) out[head * d + tid] = o / l;
}

// A chunk is 64 cache rows.  Its keys and values (64 x head_dim bf16 each) are requested as W values per thread and
// request, MAXD / W consecutive lanes on one row; while they travel the query is rotated (and, in the chunk that
// holds the token's own row, key and value are rotated, rounded and appended).  A wave keeps everything about its 16
// rows to itself: the partial dot products of a row meet by lane exchanges, the wave takes its own maximum, weights
// and sum, multiplies its value vectors in registers and adds them up across its rows by lane exchanges again; only
// the four waves' figures (maximum, sum, head_dim weighted values each) meet in LDS.  Two barriers per chunk.
// MAXD: the largest head size of this instance (128 or 256) -- registers and LDS are sized by it, and the smaller one
// lets twice as many workgroups share a compute unit.
template <int W, int MAXD>
__global__ __launch_bounds__(kAttnThreads) void attn_chunk_kernel(const AttnArgs p) {
    typedef typename CacheVec<W>::type vec_t;
    constexpr int kMaxLanesPerRow = MAXD / W;
    constexpr int kVecs = kChunk * kMaxLanesPerRow / kAttnThreads;            // requests per thread at most
    __shared__ __attribute__((aligned(16))) float s_q[MAXD];                  // rotated query / sqrt(head_dim)
    __shared__ __attribute__((aligned(16))) float s_newk[MAXD];               // the token's own key and value as cached
    __shared__ __attribute__((aligned(16))) float s_newv[MAXD];
    __shared__ float s_ow[kAttnWaves][MAXD];            // per wave: weighted values of its rows
    __shared__ float s_mw[kAttnWaves], s_lw[kAttnWaves];   // per wave: maximum and sum
    __shared__ float s_w[kChunk];                       // the merge's partial results
    __shared__ float s_o[kAttnThreads];                 // the merge's factors
    const int tid = threadIdx.x;
    const int head = blockIdx.x, chunk = blockIdx.y;
    const int d = p.head_dim, half = d / 2;
    const int hidden = p.n_heads * d;
    const int query = blockIdx.z;                       // 0 unless a prompt's tokens are processed together
    const bool appended = p.pos == nullptr;             // uniform: the prompt form, keys and values already cached
    const float* q_lin = p.q_lin + (int64_t)query * hidden;
    float* out = p.out + (int64_t)query * hidden;
    float* scratch = p.scratch + (int64_t)query * p.scratch_stride;
    // the token's projections do not depend on the position: requested before the position is waited for
    float qa = 0.0f, qb = 0.0f, ka = 0.0f, kb = 0.0f, va = 0.0f, vb = 0.0f;
    if (tid < half) {
        qa = q_lin[head * d + tid]; qb = q_lin[head * d + tid + half];
        if (!appended) {
            ka = p.k_lin[head * d + tid]; kb = p.k_lin[head * d + tid + half];
            va = p.v_lin[head * d + tid]; vb = p.v_lin[head * d + tid + half];
        }
    }
    const int pos = appended ? p.pos0 + query : *p.pos;
    if (pos < 0 || pos >= p.max_pos) return;            // uniform
    // Workgroup y of a head takes the chunks y, y + G, y + 2G, ... (G = workgroups per head in this launch) that hold
    // rows up to the token's: one chunk each while the context is short, several once it outgrows the launch -- then
    // a workgroup folds its chunks into ONE running maximum, sum and weighted values before it deposits anything.
    const int groups = (int)gridDim.y;
    const int last_chunk = pos / kChunk;
    if (chunk > last_chunk) return;                     // uniform: nothing cached this far yet
    const bool owner = !appended && last_chunk % groups == chunk;   // uniform: one of this workgroup's chunks holds the row this launch appends
    constexpr int L = kMaxLanesPerRow;                  // lanes per cache row: a power of two; those beyond head_dim / W idle
    constexpr int kRowsPerStep = kAttnThreads / L;      // rows the workgroup takes per request
    const int lane = tid % kWave, wave = tid / kWave;
    const int grp = tid / L, cc = tid % L;
    const bool active = cc * W < d;

    // rows beyond the token's are read as the token's row (always inside the cache) and never used; the token's own
    // row may be read while this workgroup writes it and is replaced by the values kept in LDS
    vec_t kv[kVecs], vv[kVecs];
    const auto request = [&](int c, bool keys) {
#pragma unroll
        for (int i = 0; i < kVecs; ++i) {
            if (active) {
                const int64_t at = (int64_t)min(c * kChunk + grp + i * kRowsPerStep, pos) * hidden + head * d + cc * W;
                if (keys) kv[i] = *reinterpret_cast<const vec_t*>(p.k_cache + at);
                else vv[i] = *reinterpret_cast<const vec_t*>(p.v_cache + at);
            }
        }
    };
    request(chunk, true);
    request(chunk, false);

    const float scale = 1.0f / sqrtf((float)d);
    if (tid < half) {
        const float2 cs = p.rope[(int64_t)pos * half + tid];
        s_q[tid] = (qa * cs.x - qb * cs.y) * scale;
        s_q[tid + half] = (qa * cs.y + qb * cs.x) * scale;
        if (owner) {
            const uint16_t k0 = f32_to_bf16(ka * cs.x - kb * cs.y), k1 = f32_to_bf16(ka * cs.y + kb * cs.x);
            const uint16_t v0 = f32_to_bf16(va), v1 = f32_to_bf16(vb);
            uint16_t* krow = p.k_cache + (int64_t)pos * hidden + head * d;
            uint16_t* vrow = p.v_cache + (int64_t)pos * hidden + head * d;
            krow[tid] = k0; krow[tid + half] = k1;
            vrow[tid] = v0; vrow[tid + half] = v1;
            s_newk[tid] = bf16_to_f32(k0); s_newk[tid + half] = bf16_to_f32(k1);
            s_newv[tid] = bf16_to_f32(v0); s_newv[tid + half] = bf16_to_f32(v1);
        }
    }

    float run_m = -INFINITY, run_l = 0.0f, run_o = 0.0f;   // over the chunks so far (run_o: element tid, tid < d)
    for (int c = chunk; c <= last_chunk; c += groups) {
        const int j0 = c * kChunk;
        const int rows = min(kChunk, pos + 1 - j0);
        const bool holds_token = owner && c == last_chunk;   // uniform
        const bool more = c + groups <= last_chunk;          // uniform
        __syncthreads();                                // s_q and the token's row are there; the previous chunk's figures have been read
        float score[kVecs];
#pragma unroll
        for (int i = 0; i < kVecs; ++i) {
            const int row = grp + i * kRowsPerStep;
            const bool own = holds_token && j0 + row == pos;   // this launch appends that row: its values are in LDS
            float acc = 0.0f;
            if (active) {
                float k[W];
                unpack_bf16<W>(kv[i], k);
#pragma unroll
                for (int x = 0; x < W; ++x) acc += s_q[cc * W + x] * (own ? s_newk[cc * W + x] : k[x]);
            }
#pragma unroll
            for (int off = 1; off < L; off <<= 1) acc += __shfl_xor(acc, off);
            score[i] = row < rows ? acc : -INFINITY;
        }
        if (more) request(c + groups, true);            // the next chunk travels while this one is worked on
        float m_w = score[0];
#pragma unroll
        for (int i = 1; i < kVecs; ++i) m_w = fmaxf(m_w, score[i]);
#pragma unroll
        for (int off = L; off < kWave; off <<= 1) m_w = fmaxf(m_w, __shfl_xor(m_w, off));
        float l_w = 0.0f, o_w[W];
#pragma unroll
        for (int x = 0; x < W; ++x) o_w[x] = 0.0f;
#pragma unroll
        for (int i = 0; i < kVecs; ++i) {
            const int row = grp + i * kRowsPerStep;
            const bool own = holds_token && j0 + row == pos;
            const float w = m_w == -INFINITY ? 0.0f : expf(score[i] - m_w);   // a wave without rows adds nothing
            l_w += w;
            if (active) {
                float v[W];
                unpack_bf16<W>(vv[i], v);
                // rows beyond the token's are selected out, not multiplied out: their registers hold whatever the cache
                // held before (row `pos` is requested before this launch writes it; a caller's cache need not be finite)
                const bool counts = row < rows;
#pragma unroll
                for (int x = 0; x < W; ++x) o_w[x] += counts ? w * (own ? s_newv[cc * W + x] : v[x]) : 0.0f;
            }
        }
        if (more) request(c + groups, false);
#pragma unroll
        for (int off = L; off < kWave; off <<= 1) {
            l_w += __shfl_xor(l_w, off);
#pragma unroll
            for (int x = 0; x < W; ++x) o_w[x] += __shfl_xor(o_w[x], off);
        }
        if (lane < L && active) {
#pragma unroll
            for (int x = 0; x < W; ++x) s_ow[wave][cc * W + x] = o_w[x];
        }
        if (lane == 0) { s_mw[wave] = m_w; s_lw[wave] = l_w; }
        __syncthreads();
        // the four waves' figures into the chunk's, and the chunk into the running ones
        static_assert(kAttnWaves == 4, "four waves' figures");
        const float m_c = fmaxf(fmaxf(s_mw[0], s_mw[1]), fmaxf(s_mw[2], s_mw[3]));   // finite: the chunk has a row
        float f_w[kAttnWaves], l_c = 0.0f;
#pragma unroll
        for (int q = 0; q < kAttnWaves; ++q) {
            f_w[q] = s_mw[q] == -INFINITY ? 0.0f : expf(s_mw[q] - m_c);
            l_c += f_w[q] * s_lw[q];
        }
        const float m_new = fmaxf(run_m, m_c);
        const float f_run = expf(run_m - m_new), f_c = expf(m_c - m_new);
        if (tid < d) {
            float t = 0.0f;
#pragma unroll
            for (int q = 0; q < kAttnWaves; ++q) t += f_w[q] * s_ow[q][tid];
            run_o = run_o * f_run + t * f_c;
        }
        run_l = run_l * f_run + l_c * f_c;
        run_m = m_new;
    }

    // The head's workgroups are merged by whichever of them finishes last.  Nobody waits for anybody: every
    // workgroup DEPOSITS its figures with device-scope atomic exchanges (performed where every compute unit's atomics
    // meet, not in a cache of this die), then draws a ticket from the head's counter the same way; the one that draws
    // the last ticket reads all deposits with device-scope loads, merges, and puts the counter back to zero for the
    // next launch.  Data that crosses workgroups inside this launch travels through these operations only -- no cache
    // write-back or invalidation is involved (a device-wide fence here cost 8-35 us per layer).
    // What orders a deposit before the ticket: the exchange RETURNS a value, so it is counted as outstanding until
    // it has been performed; EVERY publishing wave waits for its own outstanding memory operations (vmcnt(0), below)
    // before the barrier, and the ticket is drawn after the barrier.  A workgroup barrier alone does not wait for
    // memory operations in flight, so the wait is explicit, and it is in every wave, not only in the one that draws.
    const int used = min(groups, last_chunk + 1);       // workgroups of this head that get this far
    const bool alone = used == 1;                       // uniform
    float* dst = scratch + ((int64_t)head * p.chunks + chunk) * (d + 2);
    unsigned int sink = 0;
    const auto publish = [&](float* at, float v) {
        sink ^= __hip_atomic_exchange(reinterpret_cast<unsigned int*>(at), __float_as_uint(v), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    };
    if (alone) {
        if (tid < d) out[head * d + tid] = run_o / run_l;   // the only workgroup: nothing is deposited
    } else {
        if (tid < d) publish(dst + tid, run_o);
        if (tid == 0) {
            publish(dst + d, run_m);
            publish(dst + d + 1, run_l);
        }
    }
    if (alone) return;                                  // uniform
    __shared__ unsigned int s_ticket;
    // every lane consumes what its exchanges returned (so they stay returning atomics) and waits until none of this
    // wave's memory operations is outstanding
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(sink) : "memory");
    __syncthreads();                                    // all deposits of this workgroup have been performed (and s_o, s_w read)
    unsigned int* counter = reinterpret_cast<unsigned int*>(scratch + (int64_t)p.n_heads * p.chunks * (d + 2)) + head;
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != (unsigned)(used - 1)) return;       // uniform
    attn_merge(p, scratch, out, head, used, s_o, s_w);
    if (tid == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A prompt's keys and values into the cache, ahead of its attention: one token per workgroup, the rotation and
// rounding of attn_chunk_kernel's own append.  A thread takes two neighbouring elements of a head's lower half and
// their partners in the upper half (head_dim is a multiple of 4), so that it loads 8 bytes and stores 4 at a time.
__global__ __launch_bounds__(256) void kv_append_kernel(const AttnArgs p) {
    const int token = blockIdx.x;
    const int d = p.head_dim, half = d / 2, quarter = half / 2, hidden = p.n_heads * d;
    const int pos = p.pos0 + token;
    if (pos < 0 || pos >= p.max_pos) return;
    const float* k_lin = p.k_lin + (int64_t)token * hidden;
    const float* v_lin = p.v_lin + (int64_t)token * hidden;
    uint32_t* krow = reinterpret_cast<uint32_t*>(p.k_cache + (int64_t)pos * hidden);
    uint32_t* vrow = reinterpret_cast<uint32_t*>(p.v_cache + (int64_t)pos * hidden);
    const float2* cs_row = p.rope + (int64_t)pos * half;
    const auto pack = [](float lo, float hi) { return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16); };
    for (int i = threadIdx.x; i < p.n_heads * quarter; i += 256) {
        const int head = i / quarter, t = 2 * (i - head * quarter);
        const int lo = head * d + t, hi = lo + half;                    // even element indices
        const float2 ka = *reinterpret_cast<const float2*>(k_lin + lo), kb = *reinterpret_cast<const float2*>(k_lin + hi);
        const float2 va = *reinterpret_cast<const float2*>(v_lin + lo), vb = *reinterpret_cast<const float2*>(v_lin + hi);
        const float2 c0 = cs_row[t], c1 = cs_row[t + 1];
        krow[lo / 2] = pack(ka.x * c0.x - kb.x * c0.y, ka.y * c1.x - kb.y * c1.y);
        krow[hi / 2] = pack(ka.x * c0.y + kb.x * c0.x, ka.y * c1.y + kb.y * c1.x);
        vrow[lo / 2] = pack(va.x, va.y);
        vrow[hi / 2] = pack(vb.x, vb.y);
    }
}

// A prompt's attention on the matrix cores: one workgroup per (head, block of 64 consecutive prompt tokens), 16 queries
// per wave.  The block walks the cache's 64-row chunks up to its last token's; per chunk a wave forms its 16 x 64
// scores S = Q K^T and then O += P V with 16x16x32 bf16 products, keeping the running maximum, sum and output of
// every query in registers (the usual rescaling by 2^(old maximum - new maximum); the scores carry log2(e), so the
// weights are plain powers of two).  Keys and values are bf16 in the cache already; the fp32 queries enter as the
// sum of three bf16 numbers (the value rounded, then the remainder, then its remainder: all 24 bits, since a score's
// error is multiplied by the scores' size) and the weights, which lie in [0, 1], as the sum of two (about 17 bits);
// each part takes one product, and everything is accumulated in fp32.  Operand layouts of the product, per lane: A
// holds row lane%16 and eight consecutive contraction indices chosen by lane/16, B holds column lane%16 and the same
// eight indices, the result holds rows 4*(lane/16) .. +3 of column lane%16.  The contraction index has to be the
// register-contiguous one on both sides: K rows serve as they are, V is transposed on its way into LDS, and the
// weights pass through LDS (each wave its own part) to turn from the result layout into the A layout.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlockQ = 64;          // queries per workgroup
constexpr int kBlockThreads = 256;   // four waves of 16 queries

// nearest-even bf16 of a finite float, by the hardware's conversion
__device__ __forceinline__ short bf16_bits(float v) { return __builtin_bit_cast(short, (__bf16)v); }
__device__ __forceinline__ float bf16_value(short b) { return __uint_as_float((uint32_t)(uint16_t)b << 16); }

__device__ __forceinline__ f32x4 mfma_bf16(const s16x8& a, const s16x8& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// max / sum over the 16 lanes of a row of the wave, on the vector ALU's lane rotations; every lane gets the result
#define BL_ROW_ROR(x, n) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (x)), 0x120 + (n), 0xf, 0xf, false))
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, BL_ROW_ROR(v, 8));
    v = fmaxf(v, BL_ROW_ROR(v, 4));
    v = fmaxf(v, BL_ROW_ROR(v, 2));
    return fmaxf(v, BL_ROW_ROR(v, 1));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += BL_ROW_ROR(v, 8);
    v += BL_ROW_ROR(v, 4);
    v += BL_ROW_ROR(v, 2);
    return v + BL_ROW_ROR(v, 1);
}

template <int D16>   // head_dim rounded up to 16, in sixteens; the columns beyond head_dim are zero
__global__ __launch_bounds__(kBlockThreads) void attn_block_kernel(const AttnArgs p, const int M) {
    constexpr int D32 = (D16 + 1) / 2;   // steps of the scores' contraction over the head's elements
    constexpr int kKS = 32 * D32 + 8;    // bf16 elements per key row in LDS: 16 bytes of padding spread the rows over the banks
    constexpr int kVS = kChunk + 8;      // the same for a row of the transposed values
    constexpr int kPS = kChunk + 4;      // floats per row of weights
    __shared__ __align__(16) uint16_t s_k[kChunk * kKS];
    __shared__ __align__(16) uint16_t s_vt[16 * D16 * kVS];
    __shared__ __align__(16) float s_p[kBlockThreads / kWave][16][kPS];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    // a later block walks more chunks: those are launched first
    const int head = blockIdx.x, block = (int)(gridDim.y - 1 - blockIdx.y);
    const int d = p.head_dim, half = d / 2, hidden = p.n_heads * d;
    const int l16 = lane % 16, g = lane / 16;
    const int m_last = min(block * kBlockQ + kBlockQ - 1, M - 1);      // the block's last token
    const int last_pos = p.pos0 + M - 1;                               // the last cached row

    // the padding beyond head_dim (key columns up to a multiple of 32, value rows up to a multiple of 16) must read as zero
    if (d != 32 * D32)
        for (int i = tid; i < kChunk * kKS / 2; i += kBlockThreads) reinterpret_cast<uint32_t*>(s_k)[i] = 0;
    if (d != 16 * D16)
        for (int i = tid; i < 16 * D16 * kVS / 2; i += kBlockThreads) reinterpret_cast<uint32_t*>(s_vt)[i] = 0;

    // the wave's queries, rotated, scaled by log2(e) / sqrt(head_dim), as A operands: row l16, elements 32 ks + 8 g .. + 7
    s16x8 q_hi[D32], q_mid[D32], q_lo[D32];
    {
        const int m = min(block * kBlockQ + wave * 16 + l16, M - 1);   // rows beyond the prompt repeat its last one
        const float* q = p.q_lin + (int64_t)m * hidden + head * d;
        const float2* cs_row = p.rope + (int64_t)(p.pos0 + m) * half;
        const float scale = 1.4426950408889634f / sqrtf((float)d);
#pragma unroll
        for (int ks = 0; ks < D32; ++ks) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // element e of the rotated query: pairs (e, e + half); no branches, so that all loads go out together
                const int e = 32 * ks + 8 * g + j;
                const bool low = e < half, valid = e < d;
                const int ea = valid ? (low ? e : e - half) : 0;
                const float a = q[ea], b = q[ea + half];
                const float2 cs = cs_row[ea];
                float v = low ? a * cs.x - b * cs.y : a * cs.y + b * cs.x;
                v = valid ? v * scale : 0.0f;
                const short hi = bf16_bits(v);
                const float r1 = v - bf16_value(hi);
                const short mid = bf16_bits(r1);
                q_hi[ks][j] = hi; q_mid[ks][j] = mid; q_lo[ks][j] = bf16_bits(r1 - bf16_value(mid));
            }
        }
    }

    f32x4 o[D16];
#pragma unroll
    for (int t = 0; t < D16; ++t) o[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    float run_m[4], run_l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { run_m[i] = -INFINITY; run_l[i] = 0.0f; }
    const int q_wave0 = p.pos0 + block * kBlockQ + wave * 16;          // position of the wave's first query
    const int q_pos0 = q_wave0 + 4 * g;                                // position of result row 0 of this lane

    // A chunk's keys and values travel cache -> registers -> LDS in pieces of 4 rows x 4 elements (head_dim is a
    // multiple of 4), 8 x 8 pieces per wave and step: the values are transposed inside the piece, so that either matrix
    // is written as 8-byte words, two lanes to a bank at worst.  The next chunk's pieces are requested before this
    // one's products start, so that their way from memory is covered by the arithmetic.
    constexpr int kSteps = (2 * ((D16 + 1) / 2) + 3) / 4;   // wave steps: 2 row halves x ceil(elements / 32), over 4 waves
    const int c_count = d / 4, c_blocks = (c_count + 7) / 8;
    const int c_last = (p.pos0 + m_last) / kChunk;
    uint2 kreg[kSteps][4], vreg[kSteps][4];
    const auto piece = [&](int i, int& c, int& rg) {       // false: nothing to do in this step
        const int wt = wave + 4 * i;
        const int cb = wt % c_blocks, rb = wt / c_blocks;
        c = cb * 8 + lane % 8;
        rg = rb * 8 + lane / 8;
        return rb < 2 && c < c_count;
    };
    const auto request = [&](int chunk) {
        const int j0 = chunk * kChunk;
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            int c, rg;
            if (piece(i, c, rg)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t at = (int64_t)min(j0 + 4 * rg + j, last_pos) * hidden + head * d + c * 4;
                    kreg[i][j] = *reinterpret_cast<const uint2*>(p.k_cache + at);
                    vreg[i][j] = *reinterpret_cast<const uint2*>(p.v_cache + at);
                }
            }
        }
    };
    request(0);
    for (int chunk = 0; chunk <= c_last; ++chunk) {
        const int j0 = chunk * kChunk;
        __syncthreads();                               // the previous chunk's tiles have been used (and the zero fill is done)
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            int c, rg;
            if (piece(i, c, rg)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<uint2*>(s_k + (4 * rg + j) * kKS + c * 4) = kreg[i][j];
                const uint2* v = vreg[i];
                uint2 t[4];
                t[0] = make_uint2((v[0].x & 0xffffu) | (v[1].x << 16), (v[2].x & 0xffffu) | (v[3].x << 16));
                t[1] = make_uint2((v[0].x >> 16) | (v[1].x & 0xffff0000u), (v[2].x >> 16) | (v[3].x & 0xffff0000u));
                t[2] = make_uint2((v[0].y & 0xffffu) | (v[1].y << 16), (v[2].y & 0xffffu) | (v[3].y << 16));
                t[3] = make_uint2((v[0].y >> 16) | (v[1].y & 0xffff0000u), (v[2].y >> 16) | (v[3].y & 0xffff0000u));
#pragma unroll
                for (int e = 0; e < 4; ++e) *reinterpret_cast<uint2*>(s_vt + (c * 4 + e) * kVS + 4 * rg) = t[e];
            }
        }
        if (chunk < c_last) request(chunk + 1);
        __syncthreads();

        // a wave whose queries all lie before this chunk has nothing to add (the block's last chunks; uniform per wave)
        if (j0 > q_wave0 + 15) continue;
        // scores of the wave's 16 queries against the chunk's 64 keys: four 16 x 16 tiles; consecutive products go to
        // different tiles, so that none waits for the one before it
        f32x4 sc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) sc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < D32; ++ks) {
            s16x8 b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) b[t] = *reinterpret_cast<const s16x8*>(s_k + (16 * t + l16) * kKS + 32 * ks + 8 * g);
#pragma unroll
            for (int t = 0; t < 4; ++t) sc[t] = mfma_bf16(q_lo[ks], b[t], sc[t]);
#pragma unroll
            for (int t = 0; t < 4; ++t) sc[t] = mfma_bf16(q_mid[ks], b[t], sc[t]);
#pragma unroll
            for (int t = 0; t < 4; ++t) sc[t] = mfma_bf16(q_hi[ks], b[t], sc[t]);
        }
        // a query sees the keys up to its own position (only the chunks around the wave's own positions need the
        // test); chunk 0 holds key 0, which every query sees, so the running maximum is finite from there on
        if (j0 + kChunk - 1 > q_wave0) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (j0 + 16 * t + l16 > q_pos0 + i) sc[t][i] = -INFINITY;
        }
        float f[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float mx = fmaxf(fmaxf(sc[0][i], sc[1][i]), fmaxf(sc[2][i], sc[3][i]));
            const float m_new = fmaxf(run_m[i], row16_max(mx));
            f[i] = __builtin_amdgcn_exp2f(run_m[i] - m_new);
            float sum = 0.0f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float w = __builtin_amdgcn_exp2f(sc[t][i] - m_new);
                sum += w;
                s_p[wave][4 * g + i][16 * t + l16] = w;
            }
            run_l[i] = run_l[i] * f[i] + row16_sum(sum);
            run_m[i] = m_new;
        }
#pragma unroll
        for (int t = 0; t < D16; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) o[t][i] *= f[i];
        // the weights are read back by this wave only: LDS serves a wave's requests in their order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const float4 w0 = *reinterpret_cast<const float4*>(&s_p[wave][l16][32 * ks + 8 * g]);
            const float4 w1 = *reinterpret_cast<const float4*>(&s_p[wave][l16][32 * ks + 8 * g + 4]);
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            s16x8 w_hi, w_lo;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                w_hi[j] = bf16_bits(w[j]);
                w_lo[j] = bf16_bits(w[j] - bf16_value(w_hi[j]));
            }
            s16x8 b[D16];
#pragma unroll
            for (int t = 0; t < D16; ++t) b[t] = *reinterpret_cast<const s16x8*>(s_vt + (16 * t + l16) * kVS + 32 * ks + 8 * g);
#pragma unroll
            for (int t = 0; t < D16; ++t) o[t] = mfma_bf16(w_lo, b[t], o[t]);
#pragma unroll
            for (int t = 0; t < D16; ++t) o[t] = mfma_bf16(w_hi, b[t], o[t]);
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = block * kBlockQ + wave * 16 + 4 * g + i;
        if (m >= M) continue;
        float* out = p.out + (int64_t)m * hidden + head * d;
        const float inv = 1.0f / run_l[i];
#pragma unroll
        for (int t = 0; t < D16; ++t)
            if (16 * t + l16 < d) out[16 * t + l16] = o[t][i] * inv;
    }
}

template <int D16>
hipError_t launch_attn_block(const AttnArgs& p, int M, hipStream_t s) {
    const dim3 grid((unsigned)p.n_heads, (unsigned)((M + kBlockQ - 1) / kBlockQ));
    attn_block_kernel<D16><<<grid, dim3(kBlockThreads), 0, s>>>(p, M);
    return hipGetLastError();
}

__global__ void pos_advance_kernel(int32_t* pos) {
    if (threadIdx.x == 0) *pos = *pos + 1;
}

}  // namespace

constexpr int kAttnTargetWorkgroups = 1024;   // of bl_attn_decode: four per compute unit (measured best on 32 heads of 128)
constexpr int kAttnMaxGroups = 32;            // per head, however few heads there are (16 heads of 96: 32 beat 64)
int g_attn_groups = 0;                        // forced workgroups per head (0: automatic)

hipError_t launch_norm_quant(const bl_norm_quant_args& a, hipStream_t s) {
    NormArgs p;
    p.a = a.a_dev; p.b = a.b_dev; p.h = a.h_dev; p.gamma = a.gamma_dev;
    p.q = a.q_dev; p.a_scale = a.a_scale_dev; p.q_sum = a.q_sum_dev; p.y = a.y_dev;
    p.K = (int32_t)a.K; p.Kp = (int32_t)a.Kp; p.eps = a.eps;
    p.scratch = static_cast<float2*>(a.scratch_dev);
    auto ok16 = [](const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; };
    const bool vec = a.K % 4 == 0 && ok16(a.a_dev) && ok16(a.b_dev) && ok16(a.h_dev) && ok16(a.gamma_dev) && ok16(a.y_dev);
    p.pieces = a.pieces;
    if (a.mode == BL_NORM_PREMULTIPLIED) return launch_norm_premultiplied(p, vec, s);
    if (a.scratch_dev && a.K >= kWideMinK && a.M <= 65535) {
        switch (a.mode) {
            case BL_NORM_PLAIN: return launch_norm_wide<BL_NORM_PLAIN>(p, a.M, vec, s);
            case BL_NORM_RESIDUAL: return launch_norm_wide<BL_NORM_RESIDUAL>(p, a.M, vec, s);
            case BL_NORM_GATED: return launch_norm_wide<BL_NORM_GATED>(p, a.M, vec, s);
        }
    }
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

static void launch_attn_chunks(const AttnArgs& p, const dim3& grid, hipStream_t s) {
    const dim3 block(kAttnThreads);
    if (p.head_dim % 8 == 0) {
        if (p.head_dim <= 128) attn_chunk_kernel<8, 128><<<grid, block, 0, s>>>(p);
        else attn_chunk_kernel<8, BL_ATTN_MAX_HEAD_DIM><<<grid, block, 0, s>>>(p);
    } else {
        if (p.head_dim <= 128) attn_chunk_kernel<4, 128><<<grid, block, 0, s>>>(p);
        else attn_chunk_kernel<4, BL_ATTN_MAX_HEAD_DIM><<<grid, block, 0, s>>>(p);
    }
}

hipError_t launch_attn_decode(const bl_attn_args& a, hipStream_t s) {
    AttnArgs p;
    p.q_lin = a.q_lin_dev; p.k_lin = a.k_lin_dev; p.v_lin = a.v_lin_dev; p.pos = a.pos_dev;
    p.rope = reinterpret_cast<const float2*>(a.rope_table_dev);
    p.k_cache = a.k_cache_dev; p.v_cache = a.v_cache_dev; p.out = a.out_dev;
    p.scratch = static_cast<float*>(a.scratch_dev);
    p.n_heads = a.n_heads; p.head_dim = a.head_dim; p.max_pos = a.max_pos; p.chunks = attn_chunks(a.max_pos);
    p.pos0 = 0; p.scratch_stride = 0;
    // Workgroups per head: one per chunk while that keeps the launch within a few workgroups per compute unit; a longer
    // cache is walked by that many workgroups, several chunks each (a deposit per workgroup, not per chunk).
    int groups = g_attn_groups > 0 ? g_attn_groups : min(kAttnMaxGroups, (kAttnTargetWorkgroups + a.n_heads - 1) / a.n_heads);
    if (groups > p.chunks) groups = p.chunks;
    const dim3 grid((unsigned)a.n_heads, (unsigned)groups);
    launch_attn_chunks(p, grid, s);
    return hipGetLastError();
}

void set_attn_groups(int groups) { g_attn_groups = groups; }

int64_t attn_scratch_floats(int n_heads, int head_dim, int max_pos) {   // per query
    return (int64_t)n_heads * attn_chunks(max_pos) * (head_dim + 2) + n_heads;
}

hipError_t launch_attn_prefill(const bl_attn_prefill_args& a, hipStream_t s) {
    AttnArgs p;
    p.q_lin = a.q_lin_dev; p.k_lin = a.k_lin_dev; p.v_lin = a.v_lin_dev; p.pos = nullptr;
    p.rope = reinterpret_cast<const float2*>(a.rope_table_dev);
    p.k_cache = a.k_cache_dev; p.v_cache = a.v_cache_dev; p.out = a.out_dev;
    p.scratch = static_cast<float*>(a.scratch_dev);
    p.n_heads = a.n_heads; p.head_dim = a.head_dim; p.max_pos = a.max_pos;
    p.pos0 = a.pos0;
    // a prompt's queries never look beyond its last token: chunks up to that one only
    p.chunks = attn_chunks(a.pos0 + a.M);
    p.scratch_stride = (int64_t)a.n_heads * p.chunks * (a.head_dim + 2) + a.n_heads;
    kv_append_kernel<<<dim3((unsigned)a.M), dim3(256), 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // head sizes up to 128 take the matrix-core kernel (a block of 64 tokens per workgroup); larger ones go token by token
    static_assert(BL_ATTN_BLOCK_MAX_HEAD_DIM == 128, "the dispatch below covers head sizes up to 8 sixteens");
    switch ((a.head_dim + 15) / 16) {
        case 1: return launch_attn_block<1>(p, a.M, s);
        case 2: return launch_attn_block<2>(p, a.M, s);
        case 3: return launch_attn_block<3>(p, a.M, s);
        case 4: return launch_attn_block<4>(p, a.M, s);
        case 5: return launch_attn_block<5>(p, a.M, s);
        case 6: return launch_attn_block<6>(p, a.M, s);
        case 7: return launch_attn_block<7>(p, a.M, s);
        case 8: return launch_attn_block<8>(p, a.M, s);
        default: break;
    }
    const dim3 grid((unsigned)a.n_heads, (unsigned)p.chunks, (unsigned)a.M);
    launch_attn_chunks(p, grid, s);
    return hipGetLastError();
}

hipError_t launch_pos_advance(int32_t* pos, hipStream_t s) {
    pos_advance_kernel<<<dim3(1), dim3(64), 0, s>>>(pos);
    return hipGetLastError();
}

}  // namespace bl
