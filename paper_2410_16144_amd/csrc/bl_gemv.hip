// bl_gemv / bl_gemv_batch / bl_decode_batch: the decode product (1..8 tokens) over 2-bit packed
// ternary weights (Section 2 of arXiv 2410.16144, I2_S: codes back to weights in registers, then
// multiply-add), optionally fused with the per-token absmax int8 quantization of its input.
//
// Mapping.  A workgroup is 16 waves.  Lane r of a wave owns row r of a 64-row block; the K tiles
// of a row block are dealt round-robin to a group of G = 1,2,4,8 or 16 waves (G chosen per matrix
// so that a wave gets about 8 tiles), so a workgroup covers 16/G row blocks.  Per tile a wave
// issues ONE 128-bit load per lane (1 KiB, fully coalesced), 8 tiles in flight at a time.
// The tile's 64 int8 activations are the same for all lanes: in the plain kernel they arrive by
// scalar loads and feed v_dot4_i32_i8 as scalar operands; in the fused kernel the workgroup first
// quantizes its token row into LDS (while its first weight tiles are already in flight) and the
// activations are LDS broadcast reads.  There is no cross-lane reduction: the G partial sums of
// a row meet once in LDS at the end.  These are the row-block kernels: a workgroup owns whole
// 64-row blocks and shares nothing with other workgroups.  One-token launches of medium size
// that come with a workspace take the work-balanced kernel of bl_decode_sk.hip instead; the
// choice is made in launch_decode below.
//
// Arithmetic.  Codes c = w+1 in {0,1,2} are used as they are: sum_k q*w = sum_k q*c - sum_k q.
// A packed word holds 16 codes; masking with 0x03030303 gives four byte codes, masking with
// 0x0c0c0c0c gives four codes times 4 (still int8), so a word costs 1 shift + 4 ands + 4 dot4 per
// token, the x4 group being kept in its own accumulator and divided out exactly at the end.
#include "bl_decode_device.hpp"
#include "bl_gemm_ring.hpp"

namespace bl {

namespace {

// XBF16: dtype of the raw activations (fused form only).  LAYOUT 2: tiles of the TL2-coded layout (one token, plain
// form): same streaming structure, tl2_tile_mac instead of tile_mac, no sum(q) correction.
// NORM (one token, fp32 rows): 1 = RMSNorm folded into the fused quantizer, 2 = the row is already multiplied by its norm
// weight and sum(x^2) arrives in pieces.  GLU: gated epilogue (see DecodeProblem).
// STREAM: weight tiles by streaming (nontemporal) loads, see load_weight_tile.
template <int M, bool FUSED, bool XBF16, int LAYOUT, int NORM, bool GLU, bool STREAM>
__global__ __launch_bounds__(kThreads, 8) void decode_kernel(BL_FIRST_WG_PARAMS, const DecodeBatch b) {
    static_assert(NORM == 0 || (M == 1 && FUSED && !XBF16 && LAYOUT == 1), "the norm is folded into the one-token fused quantizer of fp32 rows");
    static_assert(!GLU || (M == 1 && LAYOUT == 1), "the gated epilogue is for one token");
    static_assert(LAYOUT == 1 || (LAYOUT == 2 && M == 1 && !FUSED), "the TL2 layout has the one-token plain form only");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int tl2_lut[LAYOUT == 2 ? 32 : 1];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // which problem does this workgroup belong to (uniform)
    const int blk = blockIdx.x;
    const DecodeProblem& p = b.p[BL_PROBLEM_OF(blk)];
    const int wg = blk - p.first_wg;

    const int wlog2 = p.wlog2, G = 1 << wlog2;
    const int ks = wave & (G - 1);
    const int rb = wg * (kWaves >> wlog2) + (wave >> wlog2);
    const bool active = rb < p.row_blocks;
    const int KC = p.KC;
    const int Kp = KC * kTileK;
    const uint4* __restrict__ wp = p.packed + (int64_t)(active ? rb : 0) * KC * kWave + lane;

    // LDS carve-up: [quantized activations (fused only)] [partial sums] [small per-token scalars]
    int8_t* lds_q = reinterpret_cast<int8_t*>(smem);
    int* red = reinterpret_cast<int*>(smem + (FUSED ? M * Kp : 0));
    float* s_f = reinterpret_cast<float*>(red + kWaves * M * kWave);   // [M][16] maxima, then [M] scales
    int* s_i = reinterpret_cast<int*>(s_f + M * kWaves + M);           // [M][16] partial sum(q)
    float* s_ss = reinterpret_cast<float*>(s_i + M * kWaves);          // [16] partial sums of squares (norm form, M = 1)

    // first batch of weight tiles goes in flight before anything else
    uint4 w[kInFlight];
    // How the G waves of a row block share its KC tiles.  Fused form: dealt round-robin (wave ks takes tiles ks, ks + G,
    // ...), so that the group's loads in flight cover one contiguous window of memory.  Plain one-token form: one
    // contiguous piece per wave -- measured 1.6 to 3.1 % faster there on 70B- and 100B-shape layers (100B shape: 72.0 ->
    // 70.4 us), and 0.6 to 2 % SLOWER in the fused form, which therefore keeps the deal.
    constexpr bool kPieces = !FUSED && M == 1 && LAYOUT == 1;
    const int k_per = (KC + G - 1) >> wlog2;
    const int k_begin = min(ks * k_per, KC - 1);                                     // a valid tile also for a wave without any
    const int k_end = kPieces ? max(min(k_begin + k_per, KC), k_begin + 1) : KC;     // one past this wave's last tile
    const bool has_tiles = !kPieces || ks * k_per < KC;
    const int k_start = kPieces ? k_begin : ks, k_stride = kPieces ? 1 : G;
    auto load_part = [&](int kc0, int first, int last) {
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            if (u >= first && u < last) {
                const int k = kc0 + u * k_stride;
                w[u] = load_weight_tile<STREAM>(wp + (int64_t)(k < k_end ? k : k_end - 1) * kWave);   // clamped: always a valid tile
            }
        }
    };
    auto load_batch = [&](int kc0) { load_part(kc0, 0, kInFlight); };
    if constexpr (!FUSED) {
        load_batch(k_start);   // waves without a row block load (valid) block 0: no branch, exact wait counts
    } else {
        const bool vec = p.x_flags & 2;
        bool fast = false;
        if constexpr (M == 1) fast = vec && p.K <= 2 * kThreads * 8;   // uniform
        if (fast) {
            if constexpr (M == 1) {
                const int holders = row_threads(p.K);
                const int k0 = tid * 8, k1 = k0 + holders * 8;
                const bool h0 = tid < holders && k0 < p.K, h1 = tid < holders && k1 < p.K;
                Raw8<XBF16> r0 = {}, r1 = {};
                if (tid < holders) {   // uniform per wave
                    r0 = load_raw8<XBF16>(p.x, h0 ? k0 : 0);
                    r1 = load_raw8<XBF16>(p.x, h1 ? k1 : 0);
                }
                // half of the weight tiles go in flight behind the activations (loads retire in order, so the
                // quantizer's wait for x leaves them outstanding); the other half follows the quantizer, which
                // keeps its register footprint small
                bool folded = false;
                if constexpr (NORM == 2) {
                    if (tid < holders) {   // uniform per wave
                        const float ss = wave_sum_f(norm_pieces(p.ss_in, p.ss_count, tid, holders));
                        if (lane == 0) s_ss[wave] = ss;
                    }
                } else if constexpr (NORM == 1) {
                    if (tid < holders) {   // uniform per wave
                        const Raw8<false> g0 = load_raw8<false>(p.gamma, h0 ? k0 : 0), g1 = load_raw8<false>(p.gamma, h1 ? k1 : 0);
                        Raw8<false> d0 = g0, d1 = g1;
                        if (p.delta) {
                            d0 = load_raw8<false>(p.delta, h0 ? k0 : 0);
                            d1 = load_raw8<false>(p.delta, h1 ? k1 : 0);
                        }
                        folded = true;   // gamma and delta take the registers of the early tiles: none here
                        float ss = norm_fold(r0, r1, g0, g1, d0, d1, h0, h1, k0, k1, p.delta != nullptr,
                                             wg == 0 ? p.h_out : nullptr);
                        ss = wave_sum_f(ss);
                        if (lane == 0) s_ss[wave] = ss;
                    }
                }
                // (the waves that hold gamma and delta as well have no registers for early tiles; the others do)
                if (!folded) load_part(k_start, 0, kInFlight / 2);
                quantize_row_from_regs<XBF16>(r0, r1, h0, h1, k0, k1, holders, p.K, Kp, lds_q, s_f, s_i, tid, lane, wave);
                load_part(k_start, folded ? 0 : kInFlight / 2, kInFlight);
            }
        } else {
            // general form: quantize first (its loads would otherwise have to wait for the weight tiles too)
            if (vec) quantize_rows_to_lds<M, XBF16, true, M == 1>(p, lds_q, s_f, s_i, tid, lane, wave);
            else quantize_rows_to_lds<M, XBF16, false>(p, lds_q, s_f, s_i, tid, lane, wave);
            load_batch(k_start);   // waves without a row block load (valid) block 0: no branch, exact wait counts
        }
        if (wg == 0 && p.q_out) {   // optional copy-out of the quantized activations
            for (int i = tid; i < M * Kp / 4; i += kThreads)
                reinterpret_cast<int32_t*>(p.q_out)[i] = reinterpret_cast<const int32_t*>(lds_q)[i];
        }
    }

    Acc<M> a;
#pragma unroll
    for (int m = 0; m < M; ++m) a.lo[m] = a.hi[m] = 0;
    if constexpr (LAYOUT == 2) {
        tl2_fill_table(tl2_lut, tid);
        __syncthreads();
    }

    if (active) {
        for (int kc0 = k_start;;) {
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int k = kc0 + u * k_stride;
                if (k < k_end && has_tiles) {
                    if constexpr (LAYOUT == 2) tl2_tile_mac(w[u], p.q + k * kTl2QWords, tl2_lut, a.lo[0]);
                    else if constexpr (FUSED) tile_mac<M>(w[u], reinterpret_cast<const int32_t*>(lds_q) + k * 16, Kp / 4, a);
                    else tile_mac<M>(w[u], p.q + k * 16, Kp / 4, a);
                }
                // keep the activation reads of later tiles from piling up in registers (the TL2 form wants the
                // opposite: the next tile's table lookups under this tile's dot products)
                if constexpr (LAYOUT == 1) __builtin_amdgcn_sched_barrier(0);
            }
            kc0 += k_stride * kInFlight;
            if (kc0 >= k_end) break;
            load_batch(kc0);
        }
    }

#pragma unroll
    for (int m = 0; m < M; ++m) red[(wave * M + m) * kWave + lane] = a.lo[m] + (a.hi[m] >> 2);  // hi: exact multiple of 4
    __syncthreads();

    const int row = rb * kTileN + lane;
    for (int m = ks; m < M; m += G) {
        int qsum;
        float scale;
        if constexpr (FUSED) {
            qsum = 0;
#pragma unroll
            for (int w16 = 0; w16 < kWaves; ++w16) qsum += s_i[m * kWaves + w16];
            scale = s_f[M * kWaves + m];
            if constexpr (NORM != 0) scale *= norm_scalar(s_ss, row_threads(p.K) / kWave, p.K, p.eps);
            if (wg == 0 && wave == m % G && lane == 0) {
                if (p.a_scale_out) p.a_scale_out[m] = scale;
                if (p.q_sum_out) p.q_sum_out[m] = qsum;
            }
        } else {
            qsum = LAYOUT == 2 ? 0 : p.q_sum[m];
            scale = p.a_scale[m];
        }
        int v = -qsum;
        for (int g = 0; g < G; ++g) v += red[((wave - ks + g) * M + m) * kWave + lane];
        if constexpr (GLU) {
            // lanes 0-31: gate rows, lanes 32-63: the up rows of the same 32 outputs (the whole wave is here: ks == 0)
            const float val = (float)v * ((lane < 32 ? p.w_scale : p.w_scale2) * scale);
            const float up = __shfl_xor(val, 32);
            const int n = rb * 32 + (lane & 31);
            float x = 0.0f, z = 0.0f;
            if (lane < 32 && active && n < p.N / 2) {
                x = silu(val) * up;
                z = x * p.glu_gamma[n];
                p.out[n] = z;
            }
            const float ss = wave_sum_f(x * x), zmax = wave_max(fabsf(z));
            if (lane == 0 && active) p.ss_out[rb] = make_float2(ss, zmax);
            if (p.acc && active && row < p.N) p.acc[row] = v;
        } else if (active && row < p.N) {
            p.out[(int64_t)m * p.N + row] = (float)v * (p.w_scale * scale);
            if (p.acc) p.acc[(int64_t)m * p.N + row] = v;
        }
    }
}


// ---------------------------------------------------------------------------------------------
// 2..8 tokens: the same streaming structure, but the products run on the matrix cores.
// With M tokens the dot4 formulation costs 20 + 16*M vector ops per tile and becomes VALU-bound
// beyond M = 2; v_mfma_i32_16x16x64_i8 (A = 16 token rows x 64 k, B = 64 k x 16 weight rows)
// takes the products off the vector ALU, which is left with unpacking only (32 ops per tile).
// A tile's four packed words of lane r (row r, k-pieces 0..3) are regrouped by a 4x4 transpose
// of 16-lane blocks (two v_permlane32_swap + two v_permlane16_swap) so that lane (j, g) holds
// k-piece g of row 16t+j: the B-operand shape for the t-th group of 16 weight rows.
// ---------------------------------------------------------------------------------------------
constexpr int kMaxStagedBytes = 64 * 1024;            // largest activation matrix the plain matrix-core kernel copies into LDS
constexpr int kMfmaInFlightDirect = 4;                 // ... when it is prefetched from global memory with the tiles
constexpr int kMfmaInFlightLds = 6;                    // weight tiles in flight when the A operand is in LDS
constexpr int kMfmaRedBytes = kWaves * 16 * 32 * 4;   // per wave: 16 accumulator registers x 32 useful lanes

// ---- publishing form: every distinct input is quantized ONCE per launch -------------------------------------------
// The fused matrix-core kernel above makes every workgroup quantize all M token rows for itself, which is bound by the
// vector ALU from a few tokens on.  In the publishing form the launch's FIRST workgroups are quantizers, one per
// (distinct input, token row): each writes its row's int8 values, scale and sum to the caller's buffers with
// device-scope stores (they go through to memory, past this die's cache), waits until those stores have completed,
// and adds one to its input's "rows ready" counter.  All other workgroups request their first weight tiles, then
// wait -- a bounded number of polls -- until their input's counter says M, and read the rows like a launch that was
// given quantized activations.  Workgroups are dispatched in index order, so the quantizers are running before any
// waiter can occupy a compute unit: nobody waits for a workgroup that has no place to run.  A waiter whose polls run
// out sets the status word and goes on with whatever the buffers hold (every wave reaches the kernel's end); the
// last waiter past its wait puts the counters back to zero.
template <bool BF16>
__device__ __forceinline__ void publish_row(const DecodeBatch& b, int M, int blk, float* s_f, int* s_i) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int input = blk / M, m = blk - input * M;
    const DecodeProblem& p = b.p[b.pub_src[input]];
    const int K = p.K, Kp = p.KC * kTileK;
    const char* row = static_cast<const char*>(p.x) + (int64_t)m * p.ldx * (BF16 ? 2 : 4);
    unsigned long long* qrow = reinterpret_cast<unsigned long long*>(p.q_out + (int64_t)m * Kp);
    const bool in_regs = K <= 2 * kThreads * 8;   // uniform: two vectors per thread hold the row between the passes
    const int k0 = tid * 8, k1 = k0 + kThreads * 8;
    Raw8<BF16> r0 = {}, r1 = {};
    float amax = 0.0f;
    if (in_regs) {
        r0 = load_raw8<BF16>(row, k0 < K ? k0 : 0);
        r1 = load_raw8<BF16>(row, k1 < K ? k1 : 0);
        float v[8];
        unpack_raw8<BF16>(r0, v);
        if (k0 < K) amax = absmax8(v);
        unpack_raw8<BF16>(r1, v);
        if (k1 < K) amax = fmaxf(amax, absmax8(v));
    } else {
        amax = thread_absmax<BF16, true>(row, K, tid, kThreads);
    }
    amax = wave_max(amax);
    if (lane == 0) s_f[wave] = amax;
    __syncthreads();
    amax = s_f[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) amax = fmaxf(amax, s_f[w]);
    float inv, scale;
    quant_scales(amax, inv, scale);
    int sum = 0;
    const auto put = [&](int k, const float (&v)[8]) {
        uint32_t lo, hi;
        sum += quantize8_packed(v, inv, lo, hi);
        __hip_atomic_store(qrow + k / 8, (unsigned long long)lo | ((unsigned long long)hi << 32), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    };
    if (in_regs) {
        float v[8];
        unpack_raw8<BF16>(r0, v);
        if (k0 < K) put(k0, v);
        unpack_raw8<BF16>(r1, v);
        if (k1 < K) put(k1, v);
    } else {
        for (int k = tid * 8; k < K; k += kThreads * 8) {
            float v[8];
            load8<BF16>(row, k, v);
            put(k, v);
        }
    }
    for (int k = K + tid * 8; k < Kp; k += kThreads * 8)   // layout padding (K is a multiple of 8 in this form)
        __hip_atomic_store(qrow + k / 8, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum = wave_sum(sum);
    if (lane == 0) s_i[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += s_i[w];
        __hip_atomic_store(p.a_scale_out + m, scale, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(p.q_sum_out + m, total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // every thread's stores have been performed before the workgroup says so: stores count as outstanding vector
    // memory operations until they are acknowledged, and a workgroup barrier alone does not wait for them
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
    __syncthreads();
    if (tid < kPubCopies)
        __hip_atomic_fetch_add(b.pub_ctr + kPubReady + (input * kPubCopies + tid) * kPubStride, 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
}

// The waiters' side: thread 0 polls, everybody leaves together.
__device__ __forceinline__ void wait_for_published_rows(const DecodeBatch& b, int M, int input, int tid) {
    if (tid == 0) {
        unsigned int* ready = b.pub_ctr + kPubReady + (input * kPubCopies + (int)(blockIdx.x % kPubCopies)) * kPubStride;
        int polls = 0;
        unsigned int have = __hip_atomic_load(ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while (have < (unsigned)M && ++polls < b.pub_limit) {
            __builtin_amdgcn_s_sleep(8);
            have = __hip_atomic_load(ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (have < (unsigned)M) __hip_atomic_store(b.pub_ctr + kPubStatus, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
}

// At the END of a waiting workgroup (thread 0, nobody waits for it): count the workgroups that are through; the last one
// puts the counters back to zero.  Not at the wait itself: a returning update of ONE word by every workgroup at the
// moment the rows become ready queued them up for 8 us.
__device__ __forceinline__ void leave_published_launch(const DecodeBatch& b) {
    const unsigned int past = __hip_atomic_fetch_add(b.pub_ctr + kPubDone, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
    if (past == (unsigned)(b.total_wgs - b.pub_rows)) {   // every waiter is past its wait: counters back to zero
        for (int i = 0; i < BL_MAX_BATCH * kPubCopies; ++i)
            __hip_atomic_store(b.pub_ctr + kPubReady + i * kPubStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(b.pub_ctr + kPubDone, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// QMODE: where the int8 activations (the A operand) come from
//   0 = straight from global memory, prefetched with the weight tiles (any size)
//   1 = copied once per workgroup from global memory into LDS (when M*Kp fits)
//   2 = quantized by the workgroup into LDS (fused form)
// PUB: the publishing form (QMODE 0 or 1; XBF16 is then the dtype of the raw activations the quantizers read).
template <int M, int QMODE, bool XBF16, bool STREAM, bool PUB = false>
__global__ __launch_bounds__(kThreads, 8) void decode_mfma_kernel(BL_FIRST_WG_PARAMS, const DecodeBatch b) {
    static_assert(!PUB || QMODE == 0 || QMODE == 1, "waiters read published rows like given ones");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kLdsQ = QMODE != 0;
    constexpr int U = kLdsQ ? kMfmaInFlightLds : kMfmaInFlightDirect;   // weight tiles in flight per wave
    // fused form: the quantizer's own registers leave no room for tiles in flight beside it (with two to four
    // tokens they would fit, at the price of a spill or of a longer wait in the quantizer: measured slower)
    constexpr bool kTilesAfterQuant = QMODE == 2 && M > 1;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x;
    if constexpr (PUB) {
        if (blk < b.pub_rows) {   // uniform: a quantizer workgroup
            float* q_f = reinterpret_cast<float*>(smem);
            publish_row<XBF16>(b, M, blk, q_f, reinterpret_cast<int*>(q_f + kWaves));
            return;
        }
    }
    const DecodeProblem& p = b.p[BL_PROBLEM_OF(blk)];   // (the problems' first workgroups lie behind the quantizers)
    const int wg = blk - p.first_wg;

    const int wlog2 = p.wlog2, G = 1 << wlog2;
    const int ks = wave & (G - 1);
    const int rb = wg * (kWaves >> wlog2) + (wave >> wlog2);
    const bool active = rb < p.row_blocks;
    const int KC = p.KC;
    const int Kp = KC * kTileK;
    const uint4* __restrict__ wp = p.packed + (int64_t)(active ? rb : 0) * KC * kWave + lane;

    int8_t* lds_q = reinterpret_cast<int8_t*>(smem);
    int* red = reinterpret_cast<int*>(smem + (kLdsQ ? M * Kp : 0));
    float* s_f = reinterpret_cast<float*>(red + kMfmaRedBytes / 4);
    int* s_i = reinterpret_cast<int*>(s_f + M * kWaves + M);

    // this lane's share of the A operand: token row (lane % 16), k-piece (lane / 16)
    const int mrow = lane & 15, piece = lane >> 4;
    const bool has_row = mrow < M;
    const int a_off = (has_row ? mrow : 0) * Kp + piece * 16;   // byte offset inside the activation matrix

    uint4 w[U];
    v4i av[kLdsQ ? 1 : U];
    auto load_batch_part = [&](int kc0, bool weights, bool activations) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = kc0 + u * G;
            const int kk = k < KC ? k : KC - 1;   // clamped: always a valid tile
            if (weights) w[u] = load_weight_tile<STREAM>(wp + (int64_t)kk * kWave);
            if constexpr (!kLdsQ) {
                if (activations) {
                    av[u] = v4i{0, 0, 0, 0};
                    if (has_row) av[u] = *reinterpret_cast<const v4i*>(reinterpret_cast<const int8_t*>(p.q) + a_off + kk * kTileK);
                }
            }
        }
    };
    auto load_batch = [&](int kc0) { load_batch_part(kc0, true, true); };

    if constexpr (PUB) {
        // the weight tiles do not depend on the token: they are on their way while the quantizers work
        load_batch_part(ks, true, false);
        wait_for_published_rows(b, M, p.input, tid);
        if constexpr (QMODE == 1) {
            copy_to_lds_async(p.q, (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds_q, M * Kp / 16, tid, wave);
            wait_lds_copy<0>();   // the copy is this thread's youngest request: everything has landed, the tiles too
            __syncthreads();
        } else {
            load_batch_part(ks, false, true);
        }
    } else if constexpr (QMODE == 1) {
        // activations first, straight into LDS (loads retire in order: waiting for them leaves the weight tiles in flight)
        copy_to_lds_async(p.q, (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds_q, M * Kp / 16, tid, wave);
        load_batch(ks);
        wait_lds_copy<LdsCopyWait<U>::kYounger>();   // the U weight tiles just requested may stay in flight; the copy may not
        __syncthreads();
    } else if constexpr (!kTilesAfterQuant) {
        load_batch(ks);   // waves without a row block load (valid) block 0: no branch, exact wait counts
    }

    if constexpr (QMODE == 2) {
        if (p.x_flags & 2) quantize_rows_to_lds<M, XBF16, true>(p, lds_q, s_f, s_i, tid, lane, wave);
        else quantize_rows_to_lds<M, XBF16, false>(p, lds_q, s_f, s_i, tid, lane, wave);
        if constexpr (kTilesAfterQuant) load_batch(ks);
        if (wg == 0 && p.q_out) {
            for (int i = tid; i < M * Kp / 4; i += kThreads)
                reinterpret_cast<int32_t*>(p.q_out)[i] = reinterpret_cast<const int32_t*>(lds_q)[i];
        }
    }

    v4i acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = v4i{0, 0, 0, 0};

    if (active) {
        for (int kc0 = ks;;) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = kc0 + u * G;
                if (k < KC) {
                    v4i a_op;
                    if constexpr (kLdsQ) {
                        a_op = v4i{0, 0, 0, 0};
                        if (has_row) a_op = *reinterpret_cast<const v4i*>(lds_q + a_off + k * kTileK);
                    } else {
                        a_op = av[u];
                    }
                    uint32_t t[4];
                    regroup16(w[u], t);
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_op, expand_codes(t[g]), acc[g], 0, 0, 0);
                }
            }
            kc0 += G * U;
            if (kc0 >= KC) break;
            load_batch(kc0);
        }
    }

    // accumulator register r of group t, lane (j, g): token 4g + r, weight row 16t + j.  Tokens < 8 live in lanes 0..31.
    if (lane < 32) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(wave * 16 + t * 4 + r) * 32 + lane] = acc[t][r];
    }
    __syncthreads();

    if (active && lane < 32) {
        for (int idx = ks; idx < 16; idx += G) {
            const int t = idx >> 2, r = idx & 3;
            const int m = 4 * (lane >> 4) + r;
            const int n = rb * kTileN + 16 * t + (lane & 15);
            if (m < M && n < p.N) {
                int qsum;
                float scale;
                if constexpr (QMODE == 2) {
                    qsum = 0;
#pragma unroll
                    for (int w16 = 0; w16 < kWaves; ++w16) qsum += s_i[m * kWaves + w16];
                    scale = s_f[M * kWaves + m];
                } else {
                    qsum = p.q_sum[m];
                    scale = p.a_scale[m];
                }
                int v = -qsum;
                for (int g = 0; g < G; ++g) v += red[((wave - ks + g) * 16 + idx) * 32 + lane];
                p.out[(int64_t)m * p.N + n] = (float)v * (p.w_scale * scale);
                if (p.acc) p.acc[(int64_t)m * p.N + n] = v;
            }
        }
    }
    if constexpr (PUB) {
        if (tid == 0) leave_published_launch(b);
    }
    if constexpr (QMODE == 2) {
        if (wg == 0 && tid < M) {   // optional copy-out of the quantizer's scalars
            int qsum = 0;
            for (int w16 = 0; w16 < kWaves; ++w16) qsum += s_i[tid * kWaves + w16];
            if (p.a_scale_out) p.a_scale_out[tid] = s_f[M * kWaves + tid];
            if (p.q_sum_out) p.q_sum_out[tid] = qsum;
        }
    }
}

// One launch of one kernel (a template argument, so that every kernel has its own LdsCeiling).
template <auto Kernel>
hipError_t launch_kernel(const DecodeBatch& b, size_t lds_bytes, hipStream_t s) {
    static LdsCeiling ceiling;
    const hipError_t e = ceiling.ensure(reinterpret_cast<const void*>(Kernel));
    if (e != hipSuccess) return e;
    const FirstWgs first(b);
    Kernel<<<dim3((unsigned)b.total_wgs), dim3(kThreads), lds_bytes, s>>>(BL_FIRST_WG_ARGS(first), b);
    return hipGetLastError();
}

// decode_kernel by its template arguments, with the note for bl_last_kernel; the streaming form by b.stream
template <int M, bool FUSED, bool XBF16, int LAYOUT = 1, int NORM = 0, bool GLU = false>
hipError_t launch_dot(const DecodeBatch& b, size_t lds_bytes, hipStream_t s) {
    note_kernel("decode_kernel<%d, %b, %b, %d, %d, %b, %b>", b.total_wgs, M, FUSED, XBF16, LAYOUT, NORM, GLU, b.stream != 0);
    return b.stream ? launch_kernel<&decode_kernel<M, FUSED, XBF16, LAYOUT, NORM, GLU, true>>(b, lds_bytes, s)
                    : launch_kernel<&decode_kernel<M, FUSED, XBF16, LAYOUT, NORM, GLU, false>>(b, lds_bytes, s);
}

template <int M, int QMODE, bool XBF16>
hipError_t launch_mfma(const DecodeBatch& b, size_t lds_bytes, hipStream_t s) {
    note_kernel("decode_mfma_kernel<%d, %d, %b, %b>", b.total_wgs, M, QMODE, XBF16, b.stream != 0);
    return b.stream ? launch_kernel<&decode_mfma_kernel<M, QMODE, XBF16, true>>(b, lds_bytes, s)
                    : launch_kernel<&decode_mfma_kernel<M, QMODE, XBF16, false>>(b, lds_bytes, s);
}

template <int M, int QMODE, bool XBF16>
hipError_t launch_pub(const DecodeBatch& b, size_t lds_bytes, hipStream_t s) {
    note_kernel("decode_mfma_kernel<%d, %d, %b, %b, true>", b.total_wgs, M, QMODE, XBF16, b.stream != 0);
    return b.stream ? launch_kernel<&decode_mfma_kernel<M, QMODE, XBF16, true, true>>(b, lds_bytes, s)
                    : launch_kernel<&decode_mfma_kernel<M, QMODE, XBF16, false, true>>(b, lds_bytes, s);
}

// KIND: 0 = dot-product kernel, plain; 1 = dot-product kernel, fused; 2..4 = matrix-core kernel with QMODE 0..2;
// 5, 6 = publishing form of the matrix-core kernel with QMODE 0, 1
template <int M, int KIND, bool XBF16>
hipError_t launch_one(const DecodeBatch& b, size_t lds_bytes, hipStream_t s) {
    if constexpr (KIND == 0) return launch_dot<M, false, true>(b, lds_bytes, s);
    else if constexpr (KIND == 1) return launch_dot<M, true, XBF16>(b, lds_bytes, s);
    else if constexpr (KIND == 2) return launch_mfma<M, 0, true>(b, lds_bytes, s);
    else if constexpr (KIND == 3) return launch_mfma<M, 1, true>(b, lds_bytes, s);
    else if constexpr (KIND == 4) return launch_mfma<M, 2, XBF16>(b, lds_bytes, s);
    else if constexpr (M == 1) return hipErrorInvalidValue;   // the publishing form is for 2..8 tokens
    else if constexpr (KIND == 5) return launch_pub<M, 0, XBF16>(b, lds_bytes, s);
    else return launch_pub<M, 1, XBF16>(b, lds_bytes, s);
}

template <int KIND, bool XBF16>
hipError_t launch_m(const DecodeBatch& b, int M, size_t lds, hipStream_t s) {
    switch (M) {
        case 1: return launch_one<1, KIND, XBF16>(b, lds, s);
        case 2: return launch_one<2, KIND, XBF16>(b, lds, s);
        case 3: return launch_one<3, KIND, XBF16>(b, lds, s);
        case 4: return launch_one<4, KIND, XBF16>(b, lds, s);
        case 5: return launch_one<5, KIND, XBF16>(b, lds, s);
        case 6: return launch_one<6, KIND, XBF16>(b, lds, s);
        case 7: return launch_one<7, KIND, XBF16>(b, lds, s);
        case 8: return launch_one<8, KIND, XBF16>(b, lds, s);
    }
    return hipErrorInvalidValue;
}

int g_force_waves = 0;
int g_force_path = 0;   // 0 auto, 1 dot4, 2 mfma
int g_force_stage = 0;  // 1: never stage the activations in LDS (matrix-core kernel, plain form)
int g_force_stream = 0; // weight tiles by streaming loads: 0 automatic, 1 always, -1 never
int g_publish = 0;      // publishing form of fused launches of 2..8 tokens: 0 when possible, -1 never
int g_wait_limit = 0;   // polls before a waiter gives up; 0: kDefaultWaitLimit
constexpr int kDefaultWaitLimit = 1 << 18;   // a poll is a round trip to memory plus a short sleep, about a microsecond

// Whether a fused launch can take the publishing form: a workspace for the counters, vector-loadable rows, and
// buffers for the quantized rows of every problem (that is where they are published).
bool can_publish(const DecodeBatch& b, int M) {
    if (g_publish < 0 || M < 2 || !b.ws) return false;
    for (int i = 0; i < b.count; ++i) {
        const DecodeProblem& p = b.p[i];
        if (!p.q_out || !p.a_scale_out || !p.q_sum_out || !(p.x_flags & 2) || p.gamma || p.ss_in || p.glu_gamma) return false;
    }
    return true;
}

// Numbers the distinct inputs (same rows, same destination buffers) and puts the quantizers in front of the grid.
void plan_publish(DecodeBatch& b, int M) {
    int inputs = 0;
    for (int i = 0; i < b.count; ++i) {
        DecodeProblem& p = b.p[i];
        int found = -1;
        for (int j = 0; j < inputs && found < 0; ++j) {
            const DecodeProblem& o = b.p[b.pub_src[j]];
            if (o.x == p.x && o.ldx == p.ldx && o.K == p.K && o.x_flags == p.x_flags && o.q_out == p.q_out &&
                o.a_scale_out == p.a_scale_out && o.q_sum_out == p.q_sum_out)
                found = j;
        }
        if (found < 0) {
            found = inputs;
            b.pub_src[inputs++] = i;
        }
        p.input = found;
        // the waiters read what the quantizers publish
        p.q = reinterpret_cast<const int32_t*>(p.q_out);
        p.a_scale = p.a_scale_out;
        p.q_sum = p.q_sum_out;
    }
    b.pub_rows = inputs * M;
    for (int i = 0; i < b.count; ++i) b.p[i].first_wg += b.pub_rows;
    b.total_wgs += b.pub_rows;
    b.pub_limit = g_wait_limit > 0 ? g_wait_limit : kDefaultWaitLimit;
    b.pub_ctr = reinterpret_cast<unsigned int*>(reinterpret_cast<char*>(b.ws) + BL_WORKSPACE_BYTES - kPubBytes);
}

// Launches whose weights could not stay in the 256 MB memory-side cache anyway stream them (nontemporal loads); small
// launches, as the token loops of the smallest models make them, use ordinary loads so that the model may stay cached
// from token to token.  The launch's packed bytes are all the library knows of the model's size: 4 MiB is the line
// (every launch of the Appendix-A models up to 1B, 233 MB of packed weights in all, lies below it; every launch of
// the models from 2.5B up, whose weights do not fit that cache, above).
constexpr int64_t kStreamBytes = 4 << 20;
bool want_stream(const DecodeBatch& b) {
    if (g_force_stream) return g_force_stream > 0;
    int64_t tiles = 0;
    for (int i = 0; i < b.count; ++i) tiles += (int64_t)b.p[i].row_blocks * b.p[i].KC;
    return tiles * kTileBytes >= kStreamBytes;
}

bool use_mfma(int M) { return g_force_path ? g_force_path == 2 : M >= 2; }

}  // namespace

void set_gemv_waves(int waves) { g_force_waves = waves; }
void set_decode_path(int path) { g_force_path = path; }
void set_decode_stage(int v) { g_force_stage = v; }
void set_decode_stream(int v) { g_force_stream = v; }
void set_decode_publish(int v) { g_publish = v; }
void set_decode_wait_limit(int v) { g_wait_limit = v; }

// LDS bytes of one launch; q_in_lds: the quantized activations live in LDS (fused, or staged copy)
static size_t lds_bytes_for(int M, int64_t max_Kp, bool q_in_lds) {
    const size_t red = use_mfma(M) ? (size_t)kMfmaRedBytes : (size_t)kWaves * M * kWave * 4;
    return (size_t)(q_in_lds ? M * max_Kp : 0) + red + (size_t)(2 * M * kWaves + M + kWaves) * 4;
}

size_t decode_lds_bytes(int M, int64_t max_Kp, bool fused) { return lds_bytes_for(M, max_Kp, fused); }

// Fill in the launch geometry: waves per row block for each problem (so that a wave gets about one
// batch of `tiles_per_wave` tiles) and the workgroup prefix.  Problems are put in order of falling
// work per workgroup: workgroups are dispatched in index order, so the long ones start first and
// the short ones fill in behind them instead of the other way round.
static void plan_decode(DecodeBatch& b, int tiles_per_wave) {
    int64_t work[BL_MAX_BATCH];
    for (int i = 0; i < b.count; ++i) {
        DecodeProblem& p = b.p[i];
        int g = 1, lg = 0;
        while (g < kWaves && g * tiles_per_wave < p.KC) { g *= 2; ++lg; }
        if (g_force_waves) {
            lg = 0;
            while ((1 << lg) < g_force_waves) ++lg;
        }
        p.wlog2 = lg;
    }
    // A launch with fewer workgroups than compute units is pure latency: spread it over more units by letting
    // more waves share a row block (shorter pieces per wave, more workgroups), widest pieces first.
    if (!g_force_waves) {
        const int cus = compute_unit_count();
        for (;;) {
            int total = 0, widest = -1;
            for (int i = 0; i < b.count; ++i) {
                const DecodeProblem& p = b.p[i];
                total += (p.row_blocks + (kWaves >> p.wlog2) - 1) >> (4 - p.wlog2);
                if (p.wlog2 < 4 && (p.KC >> (p.wlog2 + 1)) >= 1 &&   // every wave keeps at least one tile
                    (widest < 0 || (p.KC >> p.wlog2) > (b.p[widest].KC >> b.p[widest].wlog2)))
                    widest = i;
            }
            if (total >= cus || widest < 0) break;
            ++b.p[widest].wlog2;
        }
        // The gated launch quantizes its input in every workgroup.  With more row blocks than compute units, two row
        // blocks per workgroup halve the workgroups and their quantizations; between one and two row blocks per unit
        // they also even out the turns (some units had two workgroups, the rest one).
        for (int i = 0; i < b.count; ++i) {
            DecodeProblem& p = b.p[i];
            if (b.count == 1 && p.glu_gamma && p.wlog2 == 4 && p.row_blocks > cus) p.wlog2 = 3;
        }
    }
    for (int i = 0; i < b.count; ++i) work[i] = (int64_t)(kWaves >> b.p[i].wlog2) * b.p[i].KC;   // tiles per workgroup
    for (int i = 1; i < b.count; ++i) {   // insertion sort, stable
        const DecodeProblem p = b.p[i];
        const int64_t w = work[i];
        int j = i;
        for (; j > 0 && work[j - 1] < w; --j) {
            b.p[j] = b.p[j - 1];
            work[j] = work[j - 1];
        }
        b.p[j] = p;
        work[j] = w;
    }
    int total = 0;
    for (int i = 0; i < b.count; ++i) {
        DecodeProblem& p = b.p[i];
        p.first_wg = total;
        const int rbs_per_wg = kWaves >> p.wlog2;
        total += (p.row_blocks + rbs_per_wg - 1) / rbs_per_wg;
    }
    b.total_wgs = total;
}

hipError_t launch_decode(const DecodeBatch& batch, int M, bool fused, hipStream_t s) {
    DecodeBatch b = batch;
    b.stream = want_stream(b);
    if (b.layout == 2) {   // TL2-coded tiles: one token, plain form, dot-product kernels only
        if (M != 1 || fused) return hipErrorInvalidValue;
        int tiles_per_wave = 0;
        if (plan_decode_split(b, false, tiles_per_wave)) return launch_decode_split(b, tiles_per_wave, false, s);
        plan_decode(b, kInFlight);
        return launch_dot<1, false, true, 2>(b, lds_bytes_for(1, 0, false), s);
    }
    int64_t max_Kp = 0;
    for (int i = 0; i < b.count; ++i) max_Kp = (int64_t)b.p[i].KC * kTileK > max_Kp ? (int64_t)b.p[i].KC * kTileK : max_Kp;
    const bool bf16 = b.p[0].x_flags & 1;   // the fused form requires one activation dtype per launch
    if (use_mfma(M)) {
        if (fused && can_publish(b, M)) {
            // every distinct input quantized once by a leading workgroup; the rest of the launch is the plain form
            const bool staged = (size_t)M * max_Kp <= (size_t)kMaxStagedBytes && g_force_stage != 1;
            // twice the tiles per wave of the plain form: half the workgroups, so that (nearly) all of them are resident
            // from the start and wait ONCE, together, instead of a second round paying start-up, wait and copy again
            plan_decode(b, 2 * (staged ? kMfmaInFlightLds : kMfmaInFlightDirect));
            plan_publish(b, M);
            const size_t lds = lds_bytes_for(M, max_Kp, staged);
            if (staged) return bf16 ? launch_m<6, true>(b, M, lds, s) : launch_m<6, false>(b, M, lds, s);
            return bf16 ? launch_m<5, true>(b, M, lds, s) : launch_m<5, false>(b, M, lds, s);
        }
        if (fused) {
            const size_t lds = lds_bytes_for(M, max_Kp, true);
            if (lds > (size_t)kMaxDecodeLds) return hipErrorInvalidValue;
            plan_decode(b, kMfmaInFlightLds);
            return bf16 ? launch_m<4, true>(b, M, lds, s) : launch_m<4, false>(b, M, lds, s);
        }
        // plain form: stage the activations in LDS when they fit, else fetch them per tile from global memory
        if ((size_t)M * max_Kp <= (size_t)kMaxStagedBytes && g_force_stage != 1) {
            plan_decode(b, kMfmaInFlightLds);
            return launch_m<3, true>(b, M, lds_bytes_for(M, max_Kp, true), s);
        }
        plan_decode(b, kMfmaInFlightDirect);
        return launch_m<2, true>(b, M, lds_bytes_for(M, max_Kp, false), s);
    }
    if (M == 1) {   // with a workspace: equal work per workgroup, row blocks cut across workgroups
        int tiles_per_wave = 0;
        if (plan_decode_split(b, fused, tiles_per_wave)) return launch_decode_split(b, tiles_per_wave, fused, s);
    }
    const size_t lds = lds_bytes_for(M, max_Kp, fused);
    if (lds > (size_t)kMaxDecodeLds) return hipErrorInvalidValue;
    plan_decode(b, kInFlight);
    if (!fused) return launch_m<0, true>(b, M, lds, s);
    if (b.p[0].gamma) {   // RMSNorm folded into the quantizer: one token, fp32 rows (checked by the entry point)
        if (M != 1 || bf16) return hipErrorInvalidValue;
        if (b.p[0].glu_gamma) return launch_dot<1, true, false, 1, 1, true>(b, lds, s);
        return launch_dot<1, true, false, 1, 1>(b, lds, s);
    }
    if (b.p[0].ss_in) {   // the row is already multiplied by its norm weight; sum(x^2) in pieces
        if (M != 1 || bf16) return hipErrorInvalidValue;
        return launch_dot<1, true, false, 1, 2>(b, lds, s);
    }
    return bf16 ? launch_m<1, true>(b, M, lds, s) : launch_m<1, false>(b, M, lds, s);
}

}  // namespace bl
