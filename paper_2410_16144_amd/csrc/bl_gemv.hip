// bl_gemv / bl_gemv_batch: the decode product (1..8 tokens) over 2-bit packed ternary weights
// (Section 2 of arXiv 2410.16144, I2_S: codes back to weights in registers, then multiply-add).
//
// Mapping.  One workgroup owns one 64-row block of one matrix; lane r of every wave owns row r.
// The workgroup's waves take the K tiles of that row block round-robin.  Per tile a wave issues
// ONE 128-bit load per lane (1 KiB, fully coalesced) for the weights; the matching 64 int8
// activations are the same for all lanes, so they are fetched with scalar loads and fed to the
// dot instruction as scalar operands.  No cross-lane reduction is needed at all: partial sums
// of the waves meet once in LDS at the end.
//
// Arithmetic.  Codes c = w+1 in {0,1,2} are used as they are: sum_k q*w = sum_k q*c - sum_k q,
// and sum_k q comes from bl_quant_act.  A packed word holds 16 codes; masking with 0x03030303
// gives four byte codes, masking with 0x0c0c0c0c gives four codes times 4 (still int8), so a
// word costs 1 shift + 4 ands + 4 v_dot4_i32_i8 per token, with the x4 group kept in its own
// accumulator and divided out exactly at the end.
#include "bl_internal.hpp"

namespace bl {

namespace {

template <int M>
struct Acc {
    int lo[M];  // sums of q * code
    int hi[M];  // sums of q * (4 * code)
};

// One 64x64 tile: w = this lane's 16 bytes (4 words), qk = tile's activations (16 words per token row).
template <int M>
__device__ __forceinline__ void tile_mac(const uint4& w, const int32_t* __restrict__ qk, int q_stride_words,
                                         Acc<M>& a) {
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
            const int32_t* qm = qk + m * q_stride_words + 4 * s;
            a.lo[m] = __builtin_amdgcn_sdot4(c0, qm[0], a.lo[m], false);
            a.hi[m] = __builtin_amdgcn_sdot4(c1, qm[1], a.hi[m], false);
            a.lo[m] = __builtin_amdgcn_sdot4(c2, qm[2], a.lo[m], false);
            a.hi[m] = __builtin_amdgcn_sdot4(c3, qm[3], a.hi[m], false);
        }
    }
}

template <int M, int WAVES, int UNROLL>
__global__ __launch_bounds__(WAVES* kWave) void gemv_kernel(const GemvBatch b) {
    __shared__ int red[WAVES > 1 ? WAVES : 1][M][kWave];

    // which problem does this workgroup belong to (uniform)
    const int blk = blockIdx.x;
    int pi = 0;
#pragma unroll
    for (int i = 1; i < BL_MAX_BATCH; ++i) pi += (blk >= b.first_block[i]) ? 1 : 0;
    const GemvProblem& p = b.p[pi];
    const int rb = blk - b.first_block[pi];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KC = p.KC;
    const int qsw = KC * (kTileK / 4);  // activation row stride in words
    const uint4* __restrict__ wp = p.packed + (int64_t)rb * KC * kWave + lane;
    const int32_t* __restrict__ q = p.q;

    Acc<M> a;
#pragma unroll
    for (int m = 0; m < M; ++m) a.lo[m] = a.hi[m] = 0;

    int kc = wave;
    for (; kc + (UNROLL - 1) * WAVES < KC; kc += UNROLL * WAVES) {
        uint4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) w[u] = wp[(int64_t)(kc + u * WAVES) * kWave];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) tile_mac<M>(w[u], q + (kc + u * WAVES) * (kTileK / 4), qsw, a);
    }
    for (; kc < KC; kc += WAVES) {
        uint4 w = wp[(int64_t)kc * kWave];
        tile_mac<M>(w, q + kc * (kTileK / 4), qsw, a);
    }

    int part[M];
#pragma unroll
    for (int m = 0; m < M; ++m) part[m] = a.lo[m] + (a.hi[m] >> 2);  // hi is an exact multiple of 4

    const int row = rb * kTileN + lane;
    if constexpr (WAVES == 1) {
        if (row < p.N) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int v = part[m] - p.q_sum[m];
                p.out[(int64_t)m * p.N + row] = (float)v * (p.w_scale * p.a_scale[m]);
                if (p.acc) p.acc[(int64_t)m * p.N + row] = v;
            }
        }
    } else {
#pragma unroll
        for (int m = 0; m < M; ++m) red[wave][m][lane] = part[m];
        __syncthreads();
        for (int m = wave; m < M; m += WAVES) {
            int v = -p.q_sum[m];
#pragma unroll
            for (int w = 0; w < WAVES; ++w) v += red[w][m][lane];
            if (row < p.N) {
                p.out[(int64_t)m * p.N + row] = (float)v * (p.w_scale * p.a_scale[m]);
                if (p.acc) p.acc[(int64_t)m * p.N + row] = v;
            }
        }
    }
}

template <int M, int WAVES>
hipError_t launch_mw(const GemvBatch& b, int blocks, hipStream_t s) {
    gemv_kernel<M, WAVES, 4><<<dim3((unsigned)blocks), dim3(WAVES * kWave), 0, s>>>(b);
    return hipGetLastError();
}

template <int M>
hipError_t launch_m(const GemvBatch& b, int blocks, int waves, hipStream_t s) {
    switch (waves) {
        case 1: return launch_mw<M, 1>(b, blocks, s);
        case 2: return launch_mw<M, 2>(b, blocks, s);
        case 4: return launch_mw<M, 4>(b, blocks, s);
        case 8: return launch_mw<M, 8>(b, blocks, s);
        default: return launch_mw<M, 16>(b, blocks, s);
    }
}

int g_force_waves = 0;

}  // namespace

void set_gemv_waves(int waves) { g_force_waves = waves; }

hipError_t launch_gemv(const GemvBatch& b, int M, hipStream_t s) {
    const int blocks = b.first_block[BL_MAX_BATCH];
    int min_kc = b.p[0].KC;
    for (int i = 1; i < b.count; ++i) min_kc = b.p[i].KC < min_kc ? b.p[i].KC : min_kc;
    // Enough waves to cover the chip several times over, but never more waves than K tiles.
    int waves = 16;
    while (waves > 1 && ((int64_t)blocks * (waves / 2) >= 4096 || waves > min_kc)) waves /= 2;
    if (g_force_waves == 1 || g_force_waves == 2 || g_force_waves == 4 || g_force_waves == 8 || g_force_waves == 16)
        waves = g_force_waves;
    switch (M) {
        case 1: return launch_m<1>(b, blocks, waves, s);
        case 2: return launch_m<2>(b, blocks, waves, s);
        case 3: return launch_m<3>(b, blocks, waves, s);
        case 4: return launch_m<4>(b, blocks, waves, s);
        case 5: return launch_m<5>(b, blocks, waves, s);
        case 6: return launch_m<6>(b, blocks, waves, s);
        case 7: return launch_m<7>(b, blocks, waves, s);
        case 8: return launch_m<8>(b, blocks, waves, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace bl
