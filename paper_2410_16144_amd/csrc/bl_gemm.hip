// bl_gemm: the prefill product (any number of tokens) on the int8 matrix cores.
//
// Same mathematics as the decode kernel (Section 2 of arXiv 2410.16144, I2_S: codes back to
// weights, multiply-add), but M is large, so this is a real dense contraction and runs on
// v_mfma_i32_32x32x32_i8:  D[m][n] += sum_k A[m][k] * B[k][n],  A = int8 activations,
// B = weight codes (w+1) as int8; sum_k q is subtracted in the epilogue.
//
// Tiling.  Workgroup = 4 waves = 128 tokens x 256 weight rows; each wave owns 128 x 64, i.e.
// 4 x 2 MFMA tiles (128 accumulator registers).  K advances one packed tile (64) per step:
//   - activations: the 128 x 64 int8 tile goes global -> registers -> LDS (double buffered,
//     rows padded to 80 bytes so the 128-bit operand reads are bank-conflict free);
//   - weights: each wave loads its own packed 64 x 64 tile straight into registers (one 128-bit
//     load per lane).  Lane r holds row r; v_permlane32_swap regroups two 16-k pieces so that
//     lanes 0-31 / 32-63 hold k-halves of the same 32 rows -- exactly the MFMA B-operand shape --
//     and 7 VALU ops expand a word of codes into the 16 int8 of one operand.  Weights never
//     touch LDS, and stay 2 bits wide all the way from HBM into the register file.
#include "bl_internal.hpp"

namespace bl {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBM = 128;          // tokens per workgroup
constexpr int kWavesN = 4;        // waves along N
constexpr int kLdsRow = 80;       // bytes per activation row in LDS (64 + 16 pad)
constexpr int kMB = kBM / 32;     // MFMA tiles along M per wave

__device__ __forceinline__ v4i expand_codes(uint32_t word) {
    v4i r;
    r[0] = (int)(word & 0x03030303u);
    r[1] = (int)((word >> 2) & 0x03030303u);
    r[2] = (int)((word >> 4) & 0x03030303u);
    r[3] = (int)((word >> 6) & 0x03030303u);
    return r;
}

__global__ __launch_bounds__(256) void gemm_kernel(const GemvProblem p, const int M) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][kBM * kLdsRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KC = p.KC;
    const int m0 = blockIdx.y * kBM;
    const int rb = blockIdx.x * kWavesN + wave;       // this wave's 64-row block of W
    const bool wave_active = rb < p.row_blocks;
    const int64_t qs = (int64_t)KC * kTileK;          // activation row stride in bytes
    const uint8_t* qbase = reinterpret_cast<const uint8_t*>(p.q);

    // global -> LDS staging of the activation tile: thread t moves rows t/4 and t/4 + 64, 16 bytes at column 16*(t%4)
    const int a_row = tid >> 2, a_col = (tid & 3) * 16;
    auto load_a = [&](int kc, uint4 (&v)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m0 + a_row + 64 * i;
            v[i] = make_uint4(0, 0, 0, 0);
            if (m < M) v[i] = *reinterpret_cast<const uint4*>(qbase + (int64_t)m * qs + kc * kTileK + a_col);
        }
    };
    auto store_a = [&](int buf, const uint4 (&v)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<uint4*>(&lds[buf][(a_row + 64 * i) * kLdsRow + a_col]) = v[i];
    };
    const uint4* wp = p.packed + (int64_t)(wave_active ? rb : 0) * KC * kWave + lane;

    v16i c[kMB][2];
#pragma unroll
    for (int i = 0; i < kMB; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0;

    uint4 a_next[2];
    load_a(0, a_next);
    uint4 w_cur = wp[0];
    store_a(0, a_next);
    __syncthreads();

    const int op_row = lane & 31, op_g = lane >> 5;
    for (int kc = 0; kc < KC; ++kc) {
        const int buf = kc & 1;
        uint4 w_next = w_cur;
        const bool more = kc + 1 < KC;
        if (more) {
            load_a(kc + 1, a_next);
            w_next = wp[(int64_t)(kc + 1) * kWave];
        }
        if (wave_active) {
            // regroup: after the swaps, x0/x1 hold rows 0-31 / 32-63 for k 0..31, y0/y1 for k 32..63
            auto s01 = __builtin_amdgcn_permlane32_swap(w_cur.x, w_cur.y, false, false);
            auto s23 = __builtin_amdgcn_permlane32_swap(w_cur.z, w_cur.w, false, false);
            const uint32_t bw[2][2] = {{s01[0], s01[1]}, {s23[0], s23[1]}};  // [kstep][n-block]
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const v4i b0 = expand_codes(bw[ks][0]);
                const v4i b1 = expand_codes(bw[ks][1]);
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) {
                    const v4i av = *reinterpret_cast<const v4i*>(
                        &lds[buf][(mb * 32 + op_row) * kLdsRow + ks * 32 + op_g * 16]);
                    c[mb][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, b0, c[mb][0], 0, 0, 0);
                    c[mb][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, b1, c[mb][1], 0, 0, 0);
                }
            }
        }
        if (more) store_a(buf ^ 1, a_next);
        __syncthreads();
        w_cur = w_next;
    }

    if (!wave_active) return;
    // epilogue: register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + mb * 32 + 8 * (r >> 2) + 4 * op_g + (r & 3);
            if (m < M) {
                const int qsum = p.q_sum[m];
                const float sc = p.w_scale * p.a_scale[m];
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const int n = rb * kTileN + nb * 32 + op_row;
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

}  // namespace

hipError_t launch_gemm(const GemvProblem& p, int64_t M, hipStream_t s) {
    const int64_t gx = (p.row_blocks + kWavesN - 1) / kWavesN;
    const int64_t gy = (M + kBM - 1) / kBM;
    if (gy > 65535) return hipErrorInvalidValue;
    gemm_kernel<<<dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s>>>(p, (int)M);
    return hipGetLastError();
}

}  // namespace bl
