// Device-side pieces shared by the decode kernels: the per-tile multiply-accumulate over packed
// codes and the in-kernel activation quantizers (Section 2 of arXiv 2410.16144, I2_S form).
#pragma once
#include "bl_quant_device.hpp"

namespace bl {

struct FirstWgs {   // host side
    int v[BL_MAX_BATCH];
    explicit FirstWgs(const DecodeBatch& b) {
        for (int i = 0; i < BL_MAX_BATCH; ++i) v[i] = i < b.count ? b.p[i].first_wg : INT32_MAX;
    }
};

constexpr int kWaves = 16;            // waves per workgroup
constexpr int kThreads = kWaves * kWave;
constexpr int kInFlight = 8;          // weight tiles a wave keeps in flight

// One lane's 16 bytes of a packed weight tile.  STREAM: a streaming (nontemporal) load -- the decode kernels read every
// weight byte exactly once per launch, and telling the memory system so is worth 10-15 % of HBM bandwidth on MI355X (a
// read-only streaming kernel over 462 MB: 6.0 TB/s with ordinary loads, 6.8 TB/s with these).  Not STREAM: an ordinary
// load, for launches so small that the whole model may live in the 256 MB memory-side cache from token to token
// (a 700M-shape token loop measured 8 % slower when its weights were streamed past that cache).
template <bool STREAM>
__device__ __forceinline__ uint4 load_weight_tile(const uint4* p) {
    if constexpr (STREAM) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        return make_uint4(v[0], v[1], v[2], v[3]);
    } else {
        return *p;
    }
}

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

// ---- layout version 2: the paper's TL2 code (Table 3), six 5-bit codes per 32-bit word, 72 k per tile --------
//
// The paper's TL2 kernel looks up partial sums of ACTIVATION triples by weight code; that replaces multiplies, which
// the dot-product units give for free here.  What carries over is the code: three weights in 5 bits, so the stream
// from HBM is shorter.  The table is the other way round: 32 entries, code -> the three weights as int8 (fourth
// byte zero), one 32-bit word each, in LDS.  32 words lie in 32 different banks, so the lookups of a wavefront
// never conflict, whatever the codes.  Per group of three weights: a shift and a mask (table address), one LDS
// read, one v_dot4_i32_i8 against the three activations -- 1.0 vector operation per weight against 0.56 for the
// 2-bit layout, for 11 % fewer bytes.  Signed weights come out of the table, so there is no sum(q) correction.
constexpr int kTl2GroupsPerWord = 6;
constexpr int kTl2QWords = BL_TL2_TILE_K / 4;   // a tile's 72 activations as 18 words

// code -> the three weights: balanced-ternary digits of the index (most significant first), negated if the sign
// bit is set.  Codes that Table 3 does not use give zeros.
__device__ __forceinline__ void tl2_weights(int code, int (&w)[3]) {
    int v = code & 15;
    const bool neg = code & 16;
    w[0] = w[1] = w[2] = 0;
    if (v > 13 || (neg && v == 0)) return;
#pragma unroll
    for (int j = 2; j >= 0; --j) {     // least significant digit first; digits are -1, 0, +1
        int d = (v + 1) % 3 - 1;       // v mod 3 mapped to {0, 1, -1}
        w[j] = d;
        v = (v - d) / 3;
    }
    if (neg) { w[0] = -w[0]; w[1] = -w[1]; w[2] = -w[2]; }
}

// The table: threads 0..31 write one entry each; a workgroup barrier must follow before the first lookup.
__device__ __forceinline__ void tl2_fill_table(int* lut, int tid) {
    if (tid < 32) {
        int t[3];
        tl2_weights(tid, t);
        lut[tid] = (t[0] & 0xff) | (t[1] & 0xff) << 8 | (t[2] & 0xff) << 16;
    }
}

// The three activations that meet group g (0..23) of a tile, as the low three bytes of a word; the fourth byte is
// whatever follows and meets the table entry's zero byte.  qk: the tile's 72 activations (wave-uniform: scalar
// loads, scalar shifts).  They are read as 64-bit pairs (a tile's activations start at a multiple of 8 bytes): from
// two separate 32-bit loads the compiler builds ONE unaligned 32-bit load for a group that straddles two words,
// which has to be a vector load, and waiting for that one drains the weight tiles in flight.
__device__ __forceinline__ int tl2_group_activations(const int32_t* __restrict__ qk, int g) {
    const int2* __restrict__ q2 = reinterpret_cast<const int2*>(qk);
    const int word = (3 * g) >> 2, off = (3 * g) & 3;
    const auto at = [&](int wd) { return (uint32_t)((wd & 1) ? q2[wd >> 1].y : q2[wd >> 1].x); };
    if (off == 0) return (int)at(word);
    if (off == 1) return (int)(at(word) >> 8);
    const uint64_t pair = at(word) | ((uint64_t)at(word + 1) << 32);
    return (int)(uint32_t)(pair >> (8 * off));
}

// One 64 x 72 tile of the version-2 layout, one token: w = this lane's 16 bytes, qk = the tile's activations.
__device__ __forceinline__ void tl2_tile_mac(const uint4& w, const int32_t* __restrict__ qk, const int* lut, int& acc) {
    const uint32_t word[4] = {w.x, w.y, w.z, w.w};
    int part[3] = {0, 0, 0};   // independent sums: the dot products of a word do not wait for one another
    int e[2][kTl2GroupsPerWord];   // the table entries of a word are fetched while the previous word's dot products run
#pragma unroll
    for (int i = 0; i < kTl2GroupsPerWord; ++i) e[0][i] = lut[(word[0] >> (5 * i)) & 31];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (s < 3) {
#pragma unroll
            for (int i = 0; i < kTl2GroupsPerWord; ++i) e[(s + 1) & 1][i] = lut[(word[s + 1] >> (5 * i)) & 31];
        }
#pragma unroll
        for (int i = 0; i < kTl2GroupsPerWord; ++i)
            part[i % 3] = __builtin_amdgcn_sdot4(e[s & 1][i], tl2_group_activations(qk, kTl2GroupsPerWord * s + i),
                                                 part[i % 3], false);
    }
    acc += part[0] + part[1] + part[2];
}

// Quantize M token rows into LDS; per-token scale and partial sums of q are left in s_f / s_i (LDS).
// General form: the rows are read twice (the second read hits L1/L2).  Both passes walk the rows R at a
// time with the R loads of a step issued together, so a pass costs one memory round trip per step
// instead of one per row.
// LONG (one token): rows of up to kLongVectors * 8192 elements take the single-read path below.
template <int M, bool BF16, bool VEC, bool LONG = false>
__device__ __forceinline__ void quantize_rows_to_lds(const DecodeProblem& p, int8_t* lds_q, float* s_f, int* s_i,
                                                     int tid, int lane, int wave) {
    const int K = p.K, Kp = p.KC * kTileK;
    const char* x = static_cast<const char*>(p.x);
    const int64_t row_bytes = p.ldx * (BF16 ? 2 : 4);
    constexpr int R = !VEC ? 1 : M < (BF16 ? 4 : 2) ? M : (BF16 ? 4 : 2);   // rows whose vectors are in registers together
    // One token with a long row (the 100B-shape down projection: 33792 elements): all of a thread's vectors are requested
    // together and stay in registers between the two passes -- ONE memory round trip where the loops below take one per
    // 8192 elements and pass, ten for such a row, during which the workgroup streams no weights.
    constexpr int kLongVectors = BF16 ? 5 : 3;        // per thread: 20 (bf16) or 24 (fp32) registers
    if constexpr (M == 1 && VEC && LONG) {
        if (K <= kLongVectors * kThreads * 8) {       // uniform
            Raw8<BF16> r[kLongVectors];
            float am = 0.0f;
#pragma unroll
            for (int j = 0; j < kLongVectors; ++j) {
                const int k = (tid + j * kThreads) * 8;
                r[j] = load_raw8<BF16>(x, k < K ? k : 0);   // beyond the row: a valid address, the values unused
            }
#pragma unroll
            for (int j = 0; j < kLongVectors; ++j) {
                if ((tid + j * kThreads) * 8 < K) {
                    float v[8];
                    unpack_raw8<BF16>(r[j], v);
                    am = fmaxf(am, absmax8(v));
                }
            }
            am = wave_max(am);
            if (lane == 0) s_f[wave] = am;
            __syncthreads();
            am = s_f[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) am = fmaxf(am, s_f[w]);
            float inv, scale;
            quant_scales(am, inv, scale);
            if (tid == 0) s_f[kWaves] = scale;
            int sum = 0;
#pragma unroll
            for (int j = 0; j < kLongVectors; ++j) {
                const int k = (tid + j * kThreads) * 8;
                if (k < K) {
                    float v[8];
                    unpack_raw8<BF16>(r[j], v);
                    sum += quantize8(v, inv, lds_q + k);
                }
            }
            for (int k = K + tid; k < Kp; k += kThreads) lds_q[k] = 0;   // layout padding
            sum = wave_sum(sum);
            if (lane == 0) s_i[wave] = sum;
            __syncthreads();
            return;
        }
    }
    float amax[M];
#pragma unroll
    for (int m = 0; m < M; ++m) amax[m] = 0.0f;
    if constexpr (VEC) {
        for (int k = tid * 8; k < K; k += kThreads * 8) {
#pragma unroll
            for (int m0 = 0; m0 < M; m0 += R) {
                Raw8<BF16> r[R];
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if (m0 + j < M) r[j] = load_raw8<BF16>(x + (m0 + j) * row_bytes, k);
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    if (m0 + j < M) {
                        float v[8];
                        unpack_raw8<BF16>(r[j], v);
                        amax[m0 + j] = fmaxf(amax[m0 + j], absmax8(v));
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < M; ++m) amax[m] = thread_absmax<BF16, false>(x + m * row_bytes, K, tid, kThreads);
    }
#pragma unroll
    for (int m = 0; m < M; ++m) amax[m] = wave_max(amax[m]);
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) s_f[m * kWaves + wave] = amax[m];
    }
    __syncthreads();
    float inv[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        float am = s_f[m * kWaves];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) am = fmaxf(am, s_f[m * kWaves + w]);
        float scale;
        quant_scales(am, inv[m], scale);
        if (tid == 0) s_f[M * kWaves + m] = scale;
    }
    int sum[M];
#pragma unroll
    for (int m = 0; m < M; ++m) sum[m] = 0;
    if constexpr (VEC) {
        for (int k = tid * 8; k < K; k += kThreads * 8) {
#pragma unroll
            for (int m0 = 0; m0 < M; m0 += R) {
                Raw8<BF16> r[R];
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if (m0 + j < M) r[j] = load_raw8<BF16>(x + (m0 + j) * row_bytes, k);
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    if (m0 + j < M) {
                        float v[8];
                        unpack_raw8<BF16>(r[j], v);
                        sum[m0 + j] += quantize8(v, inv[m0 + j], lds_q + (m0 + j) * Kp + k);
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m)
            for (int k = K + tid; k < Kp; k += kThreads) lds_q[m * Kp + k] = 0;   // layout padding
    } else {
#pragma unroll
        for (int m = 0; m < M; ++m)
            sum[m] = thread_quantize<BF16, false>(x + m * row_bytes, K, Kp, inv[m], lds_q + m * Kp, tid, kThreads);
    }
#pragma unroll
    for (int m = 0; m < M; ++m) sum[m] = wave_sum(sum[m]);
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < M; ++m) s_i[m * kWaves + wave] = sum[m];
    }
    __syncthreads();
}

// One token whose row fits two 8-element vectors per thread (K <= 16384, vector-loadable): the raw
// inputs are loaded by the caller BEFORE the weight tiles (loads retire in order, so waiting for x
// then leaves the 8 weight loads in flight) and stay in registers between the two passes.
//
// The row is held by as FEW leading waves as can hold it with two vectors per thread: the waves of a
// workgroup issue their loads one after another, so the row's loads are at the head of the compute unit's
// queue only if they come from its first waves; a load issued by wave 12 waits behind the weight tiles of
// waves 0-11, and the whole workgroup waits for it at the quantizer's first barrier.
__device__ __forceinline__ int row_threads(int K) {   // multiple of 64
    return min(kThreads, (((K + 7) / 8 + 1) / 2 + kWave - 1) / kWave * kWave);
}

// First half, run by the waves that hold the row: this wave's absolute maximum to s_f[wave].  A workgroup barrier
// follows (every wave takes it).
template <bool BF16>
__device__ __forceinline__ void row_absmax_to_lds(const Raw8<BF16>& r0, const Raw8<BF16>& r1, bool h0, bool h1,
                                                  float* s_f, int lane, int wave) {
    float v[8];
    unpack_raw8<BF16>(r0, v);
    float am = h0 ? absmax8(v) : 0.0f;
    unpack_raw8<BF16>(r1, v);
    am = fmaxf(am, h1 ? absmax8(v) : 0.0f);
    am = wave_max(am);
    if (lane == 0) s_f[wave] = am;
}

// Second half, run by the same waves after that barrier: the row's int8 values to lds_q (the padding up to Kp
// included), this wave's part of sum(q) to s_i[wave], the scale to s_f[kWaves].  Another barrier follows.
template <bool BF16>
__device__ __forceinline__ void row_quantize_to_lds(const Raw8<BF16>& r0, const Raw8<BF16>& r1, bool h0, bool h1,
                                                    int k0, int k1, int holders, int K, int Kp, int8_t* lds_q,
                                                    float* s_f, int* s_i, int tid, int lane, int wave) {
    float am = s_f[0];
    for (int w = 1; w < holders / kWave; ++w) am = fmaxf(am, s_f[w]);
    float inv, scale;
    quant_scales(am, inv, scale);
    int sum = 0;
    float v[8];
    unpack_raw8<BF16>(r0, v);
    if (h0) sum += quantize8(v, inv, lds_q + k0);
    unpack_raw8<BF16>(r1, v);
    if (h1) sum += quantize8(v, inv, lds_q + k1);
    for (int k = K + tid; k < Kp; k += holders) lds_q[k] = 0;
    sum = wave_sum(sum);
    if (tid == 0) s_f[kWaves] = scale;
    if (lane == 0) s_i[wave] = sum;
}

// RMSNorm folded into the fused quantizer (one token, fp32 row in the registers of the holder waves).  The norm's
// scalar r = 1 / sqrt(mean(x'^2) + eps) is positive and common to the whole row, so it passes through the absmax
// quantizer unchanged: quantize(r * z) has the codes of quantize(z) and r times its scale.  The row therefore becomes
// z = x' * gamma with x' = x + delta (one fp32 operation each), is quantized as it is, and r multiplies the
// activation scale -- no second pass over the row, no extra barrier.
//
// On entry r0 / r1 hold x; on exit they hold z.  Returns this thread's part of sum(x'^2).  write_h (uniform): also
// store x' to p.h_out.
__device__ __forceinline__ float norm_fold(Raw8<false>& r0, Raw8<false>& r1, const Raw8<false>& g0, const Raw8<false>& g1,
                                           const Raw8<false>& d0, const Raw8<false>& d1, bool h0, bool h1, int k0, int k1,
                                           bool has_delta, float* h_out) {
    float ss = 0.0f;
    auto one = [&](Raw8<false>& r, const Raw8<false>& g, const Raw8<false>& d, bool held, int k) {
        float x[8], gm[8], dl[8];
        unpack_raw8<false>(r, x);
        unpack_raw8<false>(g, gm);
        unpack_raw8<false>(d, dl);
        uint32_t z[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (has_delta) x[i] += dl[i];
            if (held) ss += x[i] * x[i];
            z[i] = __float_as_uint(x[i] * gm[i]);
        }
        if (h_out && held) {
            float4* dst = reinterpret_cast<float4*>(h_out + k);
            dst[0] = make_float4(x[0], x[1], x[2], x[3]);
            dst[1] = make_float4(x[4], x[5], x[6], x[7]);
        }
        r.a = make_uint4(z[0], z[1], z[2], z[3]);
        r.b = make_uint4(z[4], z[5], z[6], z[7]);
    };
    one(r0, g0, d0, h0, k0);
    one(r1, g1, d1, h1, k1);
    return ss;
}

// The row arrives multiplied by its norm weight already and sum(x^2) in `count` pieces: this holder thread's share of
// the pieces (the holder waves' shares then meet in LDS like the sums of norm_fold).
__device__ __forceinline__ float norm_pieces(const float2* __restrict__ pieces, int count, int tid, int holders) {
    float ss = 0.0f;
    for (int i = tid; i < count; i += holders) ss += pieces[i].x;   // .y, the pieces' absmax, is for consumers that cannot hold the row
    return ss;
}

// The norm's scalar from the holder waves' partial sums (every thread computes the same value).
__device__ __forceinline__ float norm_scalar(const float* s_ss, int holding_waves, int K, float eps) {
    float total = 0.0f;
    for (int w = 0; w < holding_waves; ++w) total += s_ss[w];
    return 1.0f / sqrtf(total / (float)K + eps);
}

// Both halves with their barriers, for a caller whose waves all arrive together.  Only the waves that hold the
// row run the arithmetic; the others go from barrier to barrier: the waves of a compute unit share four
// instruction issuers, so sixteen waves stepping through the quantizer's few hundred instructions cost four
// times what four waves do.  Afterwards sum(q) = s_i[0] + ... + s_i[kWaves - 1].
template <bool BF16>
__device__ __forceinline__ void quantize_row_from_regs(const Raw8<BF16>& r0, const Raw8<BF16>& r1, bool h0, bool h1,
                                                       int k0, int k1, int holders, int K, int Kp, int8_t* lds_q,
                                                       float* s_f, int* s_i, int tid, int lane, int wave) {
    const bool holder = wave * kWave < holders;   // uniform per wave
    if (holder) row_absmax_to_lds<BF16>(r0, r1, h0, h1, s_f, lane, wave);
    __syncthreads();
    if (holder) row_quantize_to_lds<BF16>(r0, r1, h0, h1, k0, k1, holders, K, Kp, lds_q, s_f, s_i, tid, lane, wave);
    else if (lane == 0) s_i[wave] = 0;
    __syncthreads();
}

// Copies n16 16-byte vectors from global memory straight into LDS at byte offset lds_dst (no staging
// registers: global_load_lds_dwordx4 writes lane i's 16 bytes at base + 16 i, which for a linear copy is exactly
// where they belong).  Asynchronous: the loads count in vmcnt like any other, in issue order; the caller waits
// with wait_lds_copy(younger) where `younger` is the number of vector loads it has issued since, and then
// synchronizes the workgroup.  Written as assembly because a global->LDS load the compiler can see makes it wait
// for ALL outstanding loads at the next dependency.  M0 carries the LDS address for this instruction only.
__device__ __forceinline__ void copy_to_lds_async(const void* src, uint32_t lds_dst, int n16, int tid, int wave) {
    for (int i0 = 0; i0 < n16; i0 += kThreads) {
        const int idx = i0 + tid;
        if (idx < n16) {
            const char* from = static_cast<const char*>(src) + (int64_t)idx * 16;
            const uint32_t to = lds_dst + (uint32_t)(i0 + wave * kWave) * 16;   // wave-uniform
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(to), "v"(from) : "memory", "m0");
#pragma clang diagnostic pop
        }
    }
}

template <int YOUNGER>
__device__ __forceinline__ void wait_lds_copy() {
    static_assert(YOUNGER >= 0 && YOUNGER < 16, "fits the low vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0f70 | YOUNGER);   // vmcnt(YOUNGER); the other counters untouched
}

// ---- matrix-core operand helpers (2..8 tokens) ----------------------------------------------
__device__ __forceinline__ void regroup16(const uint4& w, uint32_t (&t)[4]) {
    auto s02 = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
    auto s13 = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
    auto a = __builtin_amdgcn_permlane16_swap(s02[0], s13[0], false, false);
    auto c = __builtin_amdgcn_permlane16_swap(s02[1], s13[1], false, false);
    t[0] = a[0]; t[1] = a[1]; t[2] = c[0]; t[3] = c[1];
}

}  // namespace bl
