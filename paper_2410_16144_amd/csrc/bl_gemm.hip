// bl_gemm: the prefill product (any number of tokens) on the int8 matrix cores.
//
// Same mathematics as the decode kernel (Section 2 of arXiv 2410.16144, I2_S: codes back to
// weights, multiply-add), but M is large, so this is a real dense contraction and runs on
// v_mfma_i32_32x32x32_i8:  D[m][n] += sum_k A[m][k] * B[k][n],  A = int8 activations,
// B = weight codes (w+1) as int8; sum_k q is subtracted in the epilogue.
//
// Tiling.  Workgroup = 4 waves side by side along N = (32*MB) tokens x (256*NB) weight rows; each
// wave owns (32*MB) x (64*NB), i.e. MB x 2NB MFMA tiles.  (Variant WK = 2 for small M x N, where
// that grid would leave compute units idle: 2 waves along N x 2 along K, the two K groups take
// alternate packed tiles and add their accumulators through LDS at the end, so the workgroup tile
// is half as wide and the grid twice as large.)  K advances one packed tile (64) per step:
//   - activations: the (32*MB) x 64 int8 tile goes global -> registers (three steps ahead) -> LDS
//     through a ring of stages (rows padded to 80 bytes so the 128-bit operand reads are
//     bank-conflict free).  With at least three stages the operands of step i+1 are read from
//     LDS while the MFMAs of step i run, and one barrier per step is enough;
//   - weights: each wave loads its own packed 64 x 64 tile straight into registers (one 128-bit
//     load per lane, four steps ahead).  Lane r holds row r; v_permlane32_swap regroups two 16-k
//     pieces so that lanes 0-31 / 32-63 hold k-halves of the same 32 rows -- exactly the MFMA
//     B-operand shape -- and 7 VALU ops expand a word of codes into the 16 int8 of one operand.
//     Weights never touch LDS and stay 2 bits wide all the way from HBM into the register file.
// The loop body is branch-free (out-of-range rows and row blocks are clamped to valid memory and
// their results dropped in the epilogue) so that the accumulators never leave their registers.
#include <type_traits>

#include "bl_internal.hpp"

namespace bl {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kWaves = 4;         // waves per workgroup
#ifndef BL_LDS_ROW
#define BL_LDS_ROW 80
#endif
constexpr int kLdsRow = BL_LDS_ROW;   // bytes per activation row in LDS (64 + 16 pad)
constexpr int kStages = 4;       // LDS ring; 4 = the period of every register ring below, so the loop unrolls by 4 without copies

__device__ __forceinline__ v4i expand_codes(uint32_t word) {
    v4i r;
    r[0] = (int)(word & 0x03030303u);
    r[1] = (int)((word >> 2) & 0x03030303u);
    r[2] = (int)((word >> 4) & 0x03030303u);
    r[3] = (int)((word >> 6) & 0x03030303u);
    return r;
}

template <int MB, int NB, int WK>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const GemvProblem p, const int M) {
    static_assert(WK == 1 || (WK == 2 && MB % 2 == 0), "K groups exchange halves of the token tile");
    constexpr int WN = kWaves / WK;       // waves along N
    constexpr int BM = 32 * MB;
    constexpr int kTileBytesA = BM * kLdsRow;
    constexpr int kStageBytes = WK * kTileBytesA;   // one activation tile per K group
    constexpr int NLD = (BM + 63) / 64;   // 16-byte pieces each thread moves per tile (256 threads x 16 B = 64 rows)
    constexpr int kExchangeBytes = WK == 1 ? 0 : WN * MB * 2 * NB * 16 * 64 * 4;
    constexpr int kLdsBytes = kStages * kStageBytes > kExchangeBytes ? kStages * kStageBytes : kExchangeBytes;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    __shared__ float s_scale[BM];   // w_scale * a_scale[m] of the workgroup's tokens (read in the epilogue)
    __shared__ int s_qsum[BM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KC = p.KC;
    const int steps = (KC + WK - 1) / WK;             // step i covers packed tiles WK*i .. WK*i + WK-1, one per K group
    const int wave_n = wave % WN, kg = wave / WN;     // position along N, K group
    const int m0 = blockIdx.y * BM;
    const int rb0 = (blockIdx.x * WN + wave_n) * NB;  // this wave's first 64-row block of W (it owns NB of them)
    const int64_t qs = (int64_t)KC * kTileK;          // activation row stride in bytes
    const uint8_t* qbase = reinterpret_cast<const uint8_t*>(p.q);

    // global -> LDS staging: thread t moves 16 bytes at column 16*(t%4) of rows t/4 (+64)
    const int a_row = tid >> 2, a_col = (tid & 3) * 16;
    const uint8_t* a_src[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int m = min(m0 + a_row + 64 * i, M - 1);   // clamped rows compute garbage that is never stored
        a_src[i] = qbase + (int64_t)m * qs + a_col;
    }
    struct Staged { uint4 v[WK * NLD]; };   // passed by value so that it lives in registers
    auto gload = [&](int step_i) {
        Staged t;
#pragma unroll
        for (int g = 0; g < WK; ++g) {
            const int kc = step_i * WK + g;
            const int k = min(kc, KC - 1);
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                t.v[g * NLD + i] = *reinterpret_cast<const uint4*>(a_src[i] + k * kTileK);
                // a K group's tile beyond the last one must add nothing (only an odd tile count with WK = 2 gets here
                // inside the loop; reads beyond the loop's end are never used)
                if (WK > 1 && kc >= KC) t.v[g * NLD + i] = make_uint4(0, 0, 0, 0);
            }
        }
        return t;
    };
    auto lstore = [&](int stage, const Staged t) {
#pragma unroll
        for (int g = 0; g < WK; ++g)
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                if (BM >= 64 || a_row < BM)
                    *reinterpret_cast<uint4*>(&lds[stage * kStageBytes + g * kTileBytesA + (a_row + 64 * i) * kLdsRow + a_col]) =
                        t.v[g * NLD + i];
    };
    const int op_row = lane & 31, op_g = lane >> 5;
    const int a_read = kg * kTileBytesA + op_row * kLdsRow + op_g * 16;
    // operands of one 32-k half step: MB registers quadruples
    auto lread_half = [&](int stage, int ks, v4i (&a)[MB]) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            a[mb] = *reinterpret_cast<const v4i*>(&lds[stage * kStageBytes + mb * 32 * kLdsRow + a_read + ks * 32]);
    };
    struct WTiles { uint4 v[NB]; };    // by value: registers
    const uint4* wp[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)   // row blocks beyond the matrix are clamped to a valid one and dropped in the epilogue
        wp[j] = p.packed + (int64_t)min(rb0 + j, p.row_blocks - 1) * KC * kWave + lane;
    auto wload = [&](int step_i) {
        WTiles t;
#pragma unroll
        for (int j = 0; j < NB; ++j) t.v[j] = wp[j][(int64_t)min(step_i * WK + kg, KC - 1) * kWave];
        return t;
    };

    v16i c[MB][2 * NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < 2 * NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0;

    if (tid < BM) {   // published by the prologue's barrier
        const int m = min(m0 + tid, M - 1);
        s_scale[tid] = p.w_scale * p.a_scale[m];
        s_qsum[tid] = p.q_sum[m];
    }
    // prologue: LDS stages 0 and 1 filled, first-half operands of step 0 in registers; activation tiles of
    // steps 2..3 and weight tiles of steps 0..2 in flight
    lstore(0, gload(0));
    lstore(1, gload(1));
    // register rings, indexed by (step mod ring size) with compile-time phases: no copies when the loop advances
    WTiles w[4];     // packed weight tiles of steps i .. i+3
    Staged g[2];     // activation tiles of steps i+2, i+3 on their way to LDS
    w[0] = wload(0);
    w[1] = wload(1);
    w[2] = wload(2);
    g[0] = gload(2);
    g[1] = gload(3);
    __syncthreads();
    v4i a_lo[2][MB], a_hi[MB];
    lread_half(0, 0, a_lo[0]);

    // B operands of one 32-k half step: per packed tile, after v_permlane32_swap, [0] = rows 0-31 and [1] = rows
    // 32-63 of the tile.  They are expanded one half step AHEAD of the MFMAs that use them, so that the vector
    // ALU work of the expansion has independent matrix work to hide under.
    struct BOps { v4i v[NB][2]; };
    auto unpack_half = [&](const WTiles& w, int half) {
        BOps b;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            auto s = half ? __builtin_amdgcn_permlane32_swap(w.v[j].z, w.v[j].w, false, false)    // k 32..63
                          : __builtin_amdgcn_permlane32_swap(w.v[j].x, w.v[j].y, false, false);   // k 0..31
            b.v[j][0] = expand_codes(s[0]);
            b.v[j][1] = expand_codes(s[1]);
        }
        return b;
    };
    auto mfma_half = [&](const v4i (&a)[MB], const BOps& b) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                c[mb][2 * j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mb], b.v[j][0], c[mb][2 * j], 0, 0, 0);
                c[mb][2 * j + 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mb], b.v[j][1], c[mb][2 * j + 1], 0, 0, 0);
            }
    };
    // scheduling hint for one half step: each MFMA is followed by a share of the independent vector ALU work
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < 2 * NB * MB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, (16 * NB + 2 * NB * MB - 1) / (2 * NB * MB) + 1, 0);   // VALU
        }
    };
    BOps b_lo = unpack_half(w[0], 0);

    // One K step in two 32-k halves.  While the MFMAs of the first half run, the second half's operands are read
    // from the current LDS stage and expanded; while the second half runs, the first-half operands of the NEXT
    // step are read from the next stage (published by the barrier that ended the previous step) and expanded.
    // P = step mod 4 picks the ring slots at compile time.
    auto step = [&](auto phase, int kc) {
        constexpr int P = decltype(phase)::value;
        constexpr int st = P % kStages, st1 = (P + 1) % kStages, st2 = (P + 2) % kStages;
        lstore(st2, g[P % 2]);   // tile of step kc+2 (loaded two steps ago); stage st2 was last read two steps ago
        lread_half(st, 1, a_hi);
        g[P % 2] = gload(kc + 4);
        w[(P + 3) % 4] = wload(kc + 3);
        __builtin_amdgcn_sched_barrier(0);   // keep the fetches above the MFMAs they overlap with
        const BOps b_hi = unpack_half(w[P], 1);
        mfma_half(a_lo[P % 2], b_lo);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        lread_half(st1, 0, a_lo[(P + 1) % 2]);
        __builtin_amdgcn_sched_barrier(0);
        b_lo = unpack_half(w[(P + 1) % 4], 0);
        mfma_half(a_hi, b_hi);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    using P3 = std::integral_constant<int, 3>;
    static_assert(kStages == 4, "the unrolled loop assumes every ring has period 4");

    int kc = 0;
    for (; kc + 4 <= steps; kc += 4) {
        step(P0{}, kc);
        step(P1{}, kc + 1);
        step(P2{}, kc + 2);
        step(P3{}, kc + 3);
    }
    if (kc < steps) step(P0{}, kc);
    if (kc + 1 < steps) step(P1{}, kc + 1);
    if (kc + 2 < steps) step(P2{}, kc + 2);

    if constexpr (WK == 2) {
        // the two K groups swap halves of the token tile: group g keeps the 32-token blocks mb with mb % 2 == g and
        // adds the other group's accumulators for them (the loop's last barrier has released the staging ring)
        int* ex = reinterpret_cast<int*>(lds);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if ((mb & 1) != kg) {
#pragma unroll
                for (int nb = 0; nb < 2 * NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        ex[(((wave_n * MB + mb) * 2 * NB + nb) * 16 + r) * 64 + lane] = c[mb][nb][r];
            }
        }
        __syncthreads();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if ((mb & 1) == kg) {
#pragma unroll
                for (int nb = 0; nb < 2 * NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        c[mb][nb][r] += ex[(((wave_n * MB + mb) * 2 * NB + nb) * 16 + r) * 64 + lane];
            }
        }
    }

    // epilogue: register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        if (WK == 2 && (mb & 1) != kg) continue;   // the other K group finishes this block
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ml = mb * 32 + 8 * (r >> 2) + 4 * op_g + (r & 3);
            const int m = m0 + ml;
            if (m < M) {
                const int qsum = s_qsum[ml];
                const float sc = s_scale[ml];
#pragma unroll
                for (int nb = 0; nb < 2 * NB; ++nb) {
                    const int n = rb0 * kTileN + nb * 32 + op_row;   // n >= N covers padding rows and clamped row blocks
                    if (n < p.N) {
                        const int v = c[mb][nb][r] - qsum;
                        p.out[(int64_t)m * p.N + n] = (float)v * sc;
                        if (p.acc) p.acc[(int64_t)m * p.N + n] = v;
                    }
                }
            }
        }
    }
}

int g_force_mb = 0;

}  // namespace

void set_gemm_mb(int mb) { g_force_mb = mb; }

hipError_t launch_gemm(const GemvProblem& p, int64_t M, hipStream_t s) {
    // wave tile = (32*MB) tokens x (64*NB) weight rows; workgroup = 4 waves, 4/WK along N and WK along K.
    // Choice by workgroup count: 64 x 128 wave tiles (half the LDS traffic per MFMA) when the grid still gives
    // every compute unit two workgroups; 64 x 64 otherwise; and the K-split form when even that grid would
    // leave compute units without work.  Forced value: 100*WK' + 10*MB + NB with WK' = 0 for WK = 1, 1 for WK = 2.
    const int64_t tiles_m = (M + 63) / 64;
    const auto wgs = [&](int wn, int nb) { return tiles_m * ((p.row_blocks + wn * nb - 1) / (wn * nb)); };
    int mb = 2, nb = 1, wk = 1;
    if (wgs(4, 2) >= 512) nb = 2;
    else if (wgs(4, 1) < 256) wk = 2;
    if (g_force_mb) { wk = g_force_mb / 100 + 1; mb = g_force_mb / 10 % 10; nb = g_force_mb % 10; }
    const int wn = kWaves / wk;
    const int64_t gx = (p.row_blocks + wn * nb - 1) / (wn * nb);
    const int64_t gy = (M + 32 * mb - 1) / (32 * mb);
    if (gy > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(256);
    if (wk == 2 && mb == 2 && nb == 1) gemm_kernel<2, 1, 2><<<grid, block, 0, s>>>(p, (int)M);
    else if (wk == 2) return hipErrorInvalidValue;
    else if (mb == 2 && nb == 1) gemm_kernel<2, 1, 1><<<grid, block, 0, s>>>(p, (int)M);
    else if (mb == 4 && nb == 1) gemm_kernel<4, 1, 1><<<grid, block, 0, s>>>(p, (int)M);
    else if (mb == 2 && nb == 2) gemm_kernel<2, 2, 1><<<grid, block, 0, s>>>(p, (int)M);
    else if (mb == 1 && nb == 2) gemm_kernel<1, 2, 1><<<grid, block, 0, s>>>(p, (int)M);
    else if (mb == 1 && nb == 1) gemm_kernel<1, 1, 1><<<grid, block, 0, s>>>(p, (int)M);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace bl
