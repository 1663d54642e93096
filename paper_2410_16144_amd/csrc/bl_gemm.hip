// bl_gemm: the prefill product (any number of tokens) on the int8 matrix cores.
//
// Same mathematics as the decode kernel (Section 2 of arXiv 2410.16144, I2_S: codes back to
// weights, multiply-add), but M is large, so this is a real dense contraction and runs on
// v_mfma_i32_32x32x32_i8:  D[m][n] += sum_k A[m][k] * B[k][n],  A = int8 activations,
// B = weight codes (w+1) as int8; sum_k q is subtracted in the epilogue.
//
// Tiling.  Workgroup = WN x WK waves (4 or 8): WN side by side along N, WK along K; its tile is (32*MB) tokens x
// (32*H*WN) weight rows; each wave owns (32*MB) x (32*H), i.e. MB x H MFMA tiles, H = 2, 3 or 4.  (With H = 3 a wave's 96 rows are one
// packed 64-row tile and half of another, which it shares with its neighbour: both load it, each expands
// its own half.  The form was built for its workgroup count -- where 128-row wave tiles leave the last round of
// workgroups mostly empty, 96-row tiles fill it -- and measured no faster: the kernel runs at the chip's power
// limit, and compute units that idle let the others clock higher.  It stays selectable.)  (Variant WK = 2 for small M x N, where
// that grid would leave compute units idle: 2 waves along N x 2 along K, the two K groups take
// alternate packed tiles and add their accumulators through LDS at the end, so the workgroup tile
// is half as wide and the grid twice as large.)  K advances one packed tile (64) per step:
//   - activations: the (32*MB) x 64 int8 tile goes from global memory STRAIGHT into LDS
//     (global_load_lds_dwordx4: no registers, no LDS store instruction), several steps ahead, into
//     a ring of stages.  That instruction writes lane i's 16 bytes at base + 16 i, so the LDS
//     image is lane-linear; the 16-byte chunks of a row are XOR-swizzled by the row number (each
//     lane simply fetches the chunk that belongs at its position) so that the 128-bit operand
//     reads stay bank-conflict free without padding.  One barrier per step; the wait before it
//     names exactly how many younger loads may still be in flight;
//   - weights: each wave loads its own packed 64 x 64 tile straight into registers (one 128-bit
//     load per lane, into a ring of 8 steps, 4 with two tiles per step).  Lane r holds row r; v_permlane32_swap regroups two 16-k
//     pieces so that lanes 0-31 / 32-63 hold k-halves of the same 32 rows -- exactly the MFMA
//     B-operand shape -- and 7 VALU ops expand a word of codes into the 16 int8 of one operand.
//     Weights never touch LDS and stay 2 bits wide all the way from HBM into the register file.
// The loop body is branch-free (out-of-range rows and row blocks are clamped to valid memory and
// their results dropped in the epilogue) so that the accumulators never leave their registers.
#include <type_traits>

#include "bl_gemm_ring.hpp"
#include "bl_internal.hpp"

namespace bl {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;   // workgroup i runs on accelerator die i % 8, each die with its own L2

// Dynamic LDS of one form: the activation ring (reused for the K groups' final exchange), then the workgroup's per-token
// scales and sums.
template <int MB, int H, int WK, int WN>
constexpr int gemm_lds_bytes() {
    using Ring = GemmRing<MB, H, WK, WN>;
    const int ring = Ring::kStages * WK * 32 * MB * kTileK;
    const int exchange = WK == 1 ? 0 : WN * (WK - 1) * (MB * H / WK) * 16 * 64 * 4;
    return (ring > exchange ? ring : exchange) + 32 * MB * 8;
}

// One workgroup's tile of one product: tokens 32*MB*tile_y .. and the weight rows of N position tile_x.  WN waves along
// N, WK along K (the K groups take alternate packed tiles and add their accumulators through LDS at the end).  Eight
// waves give every SIMD two waves from ONE workgroup: what a launch of few, large tiles needs to keep the matrix cores
// fed while a wave waits at the step's barrier or for its operands.
template <int MB, int H, int WK, int WN>
__device__ __forceinline__ void gemm_tile(const GemmProblem& p, const int M, const int tile_x, const int tile_y) {
    static_assert(WK == 1 || (MB * H) % WK == 0, "the K groups share out the wave's MFMA tiles for the final sum");
    static_assert(H >= 2 && H <= 4, "32-row blocks per wave");
    using Ring = GemmRing<MB, H, WK, WN>;   // ring depths and wait counts: bl_gemm_ring.hpp, checked by a host-side model
    constexpr int NT = Ring::kNT;         // packed 64-row tiles a wave loads per step
    constexpr int kWaves = WN * WK;
    constexpr int BM = 32 * MB;
    constexpr int kTileBytesA = BM * kTileK;        // unpadded: 64 bytes per token row
    constexpr int kStageBytes = WK * kTileBytesA;   // one activation tile per K group
    constexpr int kStages = Ring::kStages;          // LDS ring
    constexpr int kLead = Ring::kLead;              // the tile of step i + kLead is requested during step i
    constexpr int kRQ = Ring::kRQ;                  // global -> LDS loads a loader thread issues per step
    constexpr int kSlabs = WK * BM / 16;            // 1 KiB pieces of a stage: 16 token rows of one K group, one wave-load each
    static_assert(BM <= 64, "a K group's tile is at most four slabs");
    constexpr int kExchangeBytes = WK == 1 ? 0 : WN * (WK - 1) * (MB * H / WK) * 16 * 64 * 4;   // one receiving group at a time
    constexpr int kRingBytes = kStages * kStageBytes > kExchangeBytes ? kStages * kStageBytes : kExchangeBytes;
    static_assert(gemm_lds_bytes<MB, H, WK, WN>() == kRingBytes + BM * 8, "the launcher's figure");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // ring (later the exchange area), then the two arrays below
    float* s_scale = reinterpret_cast<float*>(lds + kRingBytes);    // [BM] w_scale * a_scale[m] of the workgroup's tokens (read in the epilogue)
    int* s_qsum = reinterpret_cast<int*>(s_scale + BM);            // [BM]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KC = p.KC;
    const int steps = (KC + WK - 1) / WK;             // step i covers packed tiles WK*i .. WK*i + WK-1, one per K group
    const int wave_n = wave % WN, kg = wave / WN;     // position along N, K group
    const int m0 = tile_y * BM;
    const int row0 = (tile_x * WN + wave_n) * H * 32; // this wave's first row of W
    const int rb0 = row0 / kTileN;                    // the packed tile that row lies in
    const uint32_t upper_mask = (H % 2 != 0 && (row0 / 32) % 2 != 0) ? ~0u : 0u;   // uniform: the wave's rows start in the tile's upper half
    const int64_t qs = (int64_t)KC * kTileK;          // activation row stride in bytes
    const uint8_t* qbase = reinterpret_cast<const uint8_t*>(p.q);

    // global -> LDS: a stage is kSlabs slabs of 1 KiB (16 token rows x 64 bytes of one K group); wave w brings slabs
    // w, w + kWaves, ...: lane l fills the slab's 16-byte position l (row l / 4).  Position (row, c') holds the row's
    // chunk c = c' ^ swizzle(row), swizzle(row) = (row / 2) % 4.  A wave brings kRQ slabs or none (uniform).
    static_assert(kSlabs % kWaves == 0 || kSlabs < kWaves, "every loader wave issues the same number of requests");
    // (with a slab for every wave the test is a compile-time truth and the K loop has no branch in it: a step is then one
    // basic block, and the expansion of the next operands stays under the MFMAs where it is scheduled instead of
    // sinking behind the barrier into the block that uses it)
    constexpr bool kEveryWaveLoads = kSlabs >= kWaves;
    const bool a_loader = kEveryWaveLoads || wave < kSlabs;
    const uint8_t* a_src[kRQ];
    uint32_t a_dst[kRQ];       // offset inside a stage (wave-uniform)
    int a_group[kRQ];          // the K group whose tile the slab belongs to (wave-uniform)
#pragma unroll
    for (int j = 0; j < kRQ; ++j) {
        const int slab = (wave + j * kWaves) % kSlabs;                  // (% only keeps the idle waves' arithmetic in range)
        const int g = slab / (BM / 16), row = (slab % (BM / 16)) * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ ((row >> 1) & 3);
        a_group[j] = g;
        a_dst[j] = (uint32_t)(g * kTileBytesA + (slab % (BM / 16)) * 1024);
        a_src[j] = qbase + (int64_t)min(m0 + row, M - 1) * qs + chunk * 16;   // clamped rows: never stored
    }
    // The request is written as assembly on purpose: the compiler treats a global->LDS load it can see as an
    // access that may complete out of order and answers every later dependency with a wait for ALL outstanding
    // loads, which would undo the prefetching of both operands.  Unseen, the loads still count in vmcnt, in order
    // (this ISA has one counter for all of them); the compiler's own waits for the weight tiles then only err on
    // the strict side, and the wait that publishes a stage is written out in publish().
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    auto request_tile = [&](int step_i) {
        if (a_loader) {
            const int stage = step_i % kStages;
#pragma unroll
            for (int j = 0; j < kRQ; ++j) {
                const int k = min(step_i * WK + a_group[j], KC - 1);   // beyond the end: a valid tile, never used
                const uint8_t* src = a_src[j] + (int64_t)k * kTileK;
                const uint32_t dst = lds_base + stage * kStageBytes + a_dst[j];   // wave-uniform
                // M0 carries the LDS address of this instruction and of nothing else in this kernel (no other
                // instruction here reads M0); the compiler warns that it does not track M0 across assembly
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
#pragma clang diagnostic pop
            }
        }
    };
    // The barrier that ends step i publishes the tile of step i+2, requested during step i+2-kLead: the wait in front
    // of it names how many younger vector memory operations of this thread may still be in flight (Ring::kYounger in
    // the main loop, Ring::kYoungerTail in the unrolled tail, whose weight loads the compiler removes as dead).
    auto publish = [&](auto tail) {
        constexpr int kAllowed = decltype(tail)::value ? Ring::kYoungerTail : Ring::kYounger;
        __builtin_amdgcn_s_waitcnt(0x0f70 | kAllowed);   // vmcnt(kAllowed); LDS and scalar counters untouched
        __builtin_amdgcn_s_barrier();
    };
    const int op_row = lane & 31, op_g = lane >> 5;
    const int a_read = kg * kTileBytesA + op_row * kTileK + ((op_g ^ ((op_row >> 1) & 3)) * 16);
    // operands of one 32-k half step: MB register quadruples (the second half's chunk index differs in bit 1)
    auto lread_half = [&](int stage, int ks, v4i (&a)[MB]) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            a[mb] = *reinterpret_cast<const v4i*>(&lds[stage * kStageBytes + mb * 32 * kTileK + (a_read ^ (ks * 32))]);
    };
    struct WTiles { uint4 v[NT]; };    // by value: registers
    const uint4* wp[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)   // row blocks beyond the matrix are clamped to a valid one and dropped in the epilogue
        wp[j] = p.packed + (int64_t)min(rb0 + j, p.row_blocks - 1) * KC * kWave + lane;
    auto wload = [&](int step_i) {
        WTiles t;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            t.v[j] = wp[j][(int64_t)min(step_i * WK + kg, KC - 1) * kWave];
            // a K group's tile beyond the last one must add nothing: code 0 everywhere (only an odd tile count with
            // WK = 2 gets here inside the loop; fetches beyond the loop's end are never used)
            if (WK > 1 && step_i * WK + kg >= KC) t.v[j] = make_uint4(0, 0, 0, 0);
        }
        return t;
    };

    v16i c[MB][H];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < H; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0;

    if (tid < BM) {   // published by the prologue's barrier
        const int m = min(m0 + tid, M - 1);
        s_scale[tid] = p.w_scale * p.a_scale[m];
        s_qsum[tid] = p.q_sum[m];
    }
    // prologue: the first weight tiles and the activation tiles of steps 0..kLead-1 requested; wait for tiles 0 and 1
    // Register ring of packed weight tiles, steps i .. i+kWR-1, indexed by compile-time phases.  Eight deep where the
    // registers allow: the compiler's own wait for a weight tile (it counts the weight loads it can see) then
    // leaves the newest 6 loads in flight, which also covers the activation tiles requested since.
    constexpr int kWR = Ring::kWR;
    WTiles w[kWR];
#pragma unroll
    for (int j = 0; j < kWR - 1; ++j) w[j] = wload(j);
#pragma unroll
    for (int j = 0; j < kLead; ++j) request_tile(j);
    // Tiles 0, 1 AND 2 have landed; only the youngest requests may still be in flight (see Ring::kPrologueWait).
    __builtin_amdgcn_s_waitcnt(0x0f70 | Ring::kPrologueWait);
    __syncthreads();                                            // also publishes s_scale / s_qsum
    v4i a_lo[2][MB], a_hi[MB];
    lread_half(0, 0, a_lo[0]);

    // B operands of one 32-k half step: per packed tile, after v_permlane32_swap, [0] = rows 0-31 and [1] = rows
    // 32-63 of the tile.  They are expanded one half step AHEAD of the MFMAs that use them, so that the vector
    // ALU work of the expansion has independent matrix work to hide under.
    struct BOps { v4i v[H]; };         // one per 32-row block of the wave, in row order
    auto unpack_half = [&](const WTiles& w, int half) {
        uint32_t codes[2 * NT];        // per packed tile: words of its rows 0-31 and of its rows 32-63
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            auto s = half ? __builtin_amdgcn_permlane32_swap(w.v[j].z, w.v[j].w, false, false)    // k 32..63
                          : __builtin_amdgcn_permlane32_swap(w.v[j].x, w.v[j].y, false, false);   // k 0..31
            codes[2 * j] = s[0];
            codes[2 * j + 1] = s[1];
        }
        BOps b;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            // an odd number of 32-row blocks: the wave's rows start at the tile's lower or upper half.  Written as a
            // bit blend under a uniform mask (one v_bfi): a select between two elements of the array would become an
            // indexed access and move the array out of the registers
            if constexpr (H % 2 != 0) b.v[h] = expand_codes((codes[h + 1] & upper_mask) | (codes[h] & ~upper_mask));
            else b.v[h] = expand_codes(codes[h]);
        }
        return b;
    };
    auto mfma_half = [&](const v4i (&a)[MB], const BOps& b) {
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                c[mb][h] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mb], b.v[h], c[mb][h], 0, 0, 0);
    };
    // scheduling hint for one half step: each MFMA is followed by a share of the independent vector ALU work
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < H * MB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, (8 * H + H * MB - 1) / (H * MB) + 1, 0);   // VALU
        }
    };
    BOps b_lo = unpack_half(w[0], 0);

    // One K step in two 32-k halves.  While the MFMAs of the first half run, the second half's operands are read
    // from the current LDS stage and expanded; while the second half runs, the first-half operands of the NEXT
    // step are read from the next stage (published by the barrier that ended the previous step) and expanded.
    // P = step mod 8 picks the register-ring slots at compile time; the LDS stage index is scalar arithmetic.
    auto step = [&](auto phase, auto tail, int kc) {
        constexpr int P = decltype(phase)::value;
        const int st = kc % kStages, st1 = (kc + 1) % kStages;
        request_tile(kc + kLead);
        lread_half(st, 1, a_hi);
        w[(P + kWR - 1) % kWR] = wload(kc + kWR - 1);
        __builtin_amdgcn_sched_barrier(0);   // keep the fetches above the MFMAs they overlap with
        const BOps b_hi = unpack_half(w[P % kWR], 1);
        mfma_half(a_lo[P % 2], b_lo);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        lread_half(st1, 0, a_lo[(P + 1) % 2]);
        __builtin_amdgcn_sched_barrier(0);
        b_lo = unpack_half(w[(P + 1) % kWR], 0);
        mfma_half(a_hi, b_hi);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        publish(tail);
    };
    static_assert(Ring::kUnroll == 8, "the main loop below is written out for eight phases");
#define BL_STEP(P, KC) step(std::integral_constant<int, P>{}, std::false_type{}, KC)
#define BL_TAIL_STEP(P, KC) step(std::integral_constant<int, P>{}, std::true_type{}, KC)
    int kc = 0;
    for (; kc + 8 <= steps; kc += 8) {
        BL_STEP(0, kc);
        BL_STEP(1, kc + 1);
        BL_STEP(2, kc + 2);
        BL_STEP(3, kc + 3);
        BL_STEP(4, kc + 4);
        BL_STEP(5, kc + 5);
        BL_STEP(6, kc + 6);
        BL_STEP(7, kc + 7);
    }
    if (kc < steps) BL_TAIL_STEP(0, kc);
    if (kc + 1 < steps) BL_TAIL_STEP(1, kc + 1);
    if (kc + 2 < steps) BL_TAIL_STEP(2, kc + 2);
    if (kc + 3 < steps) BL_TAIL_STEP(3, kc + 3);
    if (kc + 4 < steps) BL_TAIL_STEP(4, kc + 4);
    if (kc + 5 < steps) BL_TAIL_STEP(5, kc + 5);
    if (kc + 6 < steps) BL_TAIL_STEP(6, kc + 6);
#undef BL_STEP
#undef BL_TAIL_STEP

    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): the tiles requested beyond the end have landed too
    if constexpr (WK > 1) {
        // The K groups add up their accumulators through LDS (the staging ring is free now).  MFMA tile t = mb * H + nb
        // of a wave is FINISHED by group t % WK: one receiving group at a time, the other groups write their partial
        // sums of its tiles, it adds them; every group ends up with the complete sums of its own share of the tiles.
        int* ex = reinterpret_cast<int*>(lds);
        constexpr int kShare = MB * H / WK;   // tiles a group finishes
#pragma unroll
        for (int owner = 0; owner < WK; ++owner) {
            __syncthreads();
            if (kg != owner) {
                const int sender = kg < owner ? kg : kg - 1;   // 0 .. WK-2
#pragma unroll
                for (int t = owner, i = 0; t < MB * H; t += WK, ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        ex[((((wave_n * (WK - 1) + sender) * kShare) + i) * 16 + r) * 64 + lane] = c[t / H][t % H][r];
            }
            __syncthreads();
            if (kg == owner) {
#pragma unroll
                for (int sender = 0; sender < WK - 1; ++sender)
#pragma unroll
                    for (int t = owner, i = 0; t < MB * H; t += WK, ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            c[t / H][t % H][r] += ex[((((wave_n * (WK - 1) + sender) * kShare) + i) * 16 + r) * 64 + lane];
            }
        }
    }

    // epilogue: register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ml = mb * 32 + 8 * (r >> 2) + 4 * op_g + (r & 3);
            const int m = m0 + ml;
            if (m < M) {
                const int qsum = s_qsum[ml];
                const float sc = s_scale[ml];
#pragma unroll
                for (int nb = 0; nb < H; ++nb) {
                    if (WK > 1 && (mb * H + nb) % WK != kg) continue;   // another K group finishes this tile
                    const int n = row0 + nb * 32 + op_row;   // n >= N covers padding rows and clamped row blocks
                    if (n < p.N) {
                        const int v = c[mb][nb][r] - qsum;
                        // streaming stores: tens of MB of output must not push the operands out of L2
                        __builtin_nontemporal_store((float)v * sc, &p.out[(int64_t)m * p.N + n]);
                        if (p.acc) __builtin_nontemporal_store(v, &p.acc[(int64_t)m * p.N + n]);
                    }
                }
            }
        }
    }
}

// Workgroup index -> tile, so that the die (index % 8) depends on the N position only: every die keeps ITS slice of
// the packed weights in its L2 for the whole launch, and consecutive workgroups (all dies) walk through the same
// token rows at the same time.  The grid is padded to a multiple of 8 along N; false for a padding workgroup.
__device__ __forceinline__ bool tile_of_workgroup(int gx, int& tile_x, int& tile_y) {
    const int gxh = (gx + kXcds - 1) / kXcds;
    const int rest = blockIdx.x / kXcds;
    tile_x = (rest % gxh) * kXcds + blockIdx.x % kXcds;
    tile_y = rest / gxh;
    return tile_x < gx;
}

template <int MB, int H, int WK, int WN>
__global__ __launch_bounds__(64 * WN * WK, WN * WK == 4 ? 2 : 1) void gemm_kernel(const GemmProblem p, const int M, const int gx) {
    int tile_x, tile_y;
    if (!tile_of_workgroup(gx, tile_x, tile_y)) return;   // uniform
    gemm_tile<MB, H, WK, WN>(p, M, tile_x, tile_y);
}

// Several products over the same M in one launch: their N positions side by side, `end[i]` the first position behind
// product i (INT32_MAX behind the last one in use).
struct GemmBatch {
    GemmProblem p[kMaxGemmBatch];
    int32_t     end[kMaxGemmBatch];
};

template <int MB, int H, int WK, int WN>
__global__ __launch_bounds__(64 * WN * WK, WN * WK == 4 ? 2 : 1) void gemm_batch_kernel(const GemmBatch b, const int M, const int gx) {
    int tile_x, tile_y;
    if (!tile_of_workgroup(gx, tile_x, tile_y)) return;   // uniform
    int item = 0, first = 0;
#pragma unroll
    for (int i = 0; i + 1 < kMaxGemmBatch; ++i)
        if (tile_x >= b.end[i]) { item = i + 1; first = b.end[i]; }
    gemm_tile<MB, H, WK, WN>(b.p[item], M, tile_x - first, tile_y);
}

int g_force_mb = 0;

// One tile form: wave tile (32*MB) tokens x (32*H) weight rows, WN waves along N and WK along K.
struct TileForm { int mb, h, wk, wn; };

// Forced value (bl_set_tuning "gemm_mb"): 100*(WK-1) + 10*MB + H; four waves per workgroup, WN = 4 / WK.
TileForm form_of_code(int code) {
    TileForm f;
    const int waves = 4;
    f.wk = code / 100 % 10 + 1;
    f.mb = code / 10 % 10;
    f.h = code % 10;
    f.wn = waves / f.wk;
    return f;
}

// Choice by workgroup count: 64 x 128 wave tiles (half the LDS traffic per MFMA) when the grid still gives
// every compute unit two workgroups; 64 x 64 otherwise; and 32 x 64 or the K-split form when even that grid would
// leave compute units without work.  `rows`: padded weight rows of the launch.
TileForm choose_tile(int64_t M, int64_t rows) {
    if (g_force_mb) return form_of_code(g_force_mb);
    const int64_t tiles_m = (M + 63) / 64;
    const auto wgs = [&](int wn, int hh) { return tiles_m * ((rows + wn * hh * 32 - 1) / (wn * hh * 32)); };
    TileForm f = {2, 2, 1, 4};
    if (wgs(4, 4) >= 512) f.h = 4;
    else if (wgs(4, 2) < 256) {
        // too few workgroups either way: 32-token tiles from 128 tokens up (measured 5-8 % ahead of the K split on
        // shapes from 1536^2 to 8192^2), the K split below
        if (M >= 128) f.mb = 1;
        else { f.wk = 2; f.wn = 2; }
    }
    return f;
}

// One LdsCeiling per kernel: the larger forms need more than the 64 KiB a kernel gets without asking.
template <typename Kernel, typename Arg>
hipError_t launch_form(Kernel kernel, size_t lds_bytes, int threads, unsigned grid, const Arg& arg, int M, int gx, hipStream_t s) {
    static LdsCeiling ceiling;   // per instantiation of this template, i.e. per kernel
    const hipError_t e = ceiling.ensure(reinterpret_cast<const void*>(kernel));
    if (e != hipSuccess) return e;
    kernel<<<dim3(grid), dim3((unsigned)threads), lds_bytes, s>>>(arg, M, gx);
    return hipGetLastError();
}

// The forms that are built.  Eight-wave workgroups (8 waves along N; 4 x 2 and 2 x 4 along N x K) were built on the same
// tile code, were bit-exact, and measured equal or slower on every benchmark shape (e.g. M = 512, K = 11008 -> N = 4096:
// 29.9 us with 2 x 4 waves against 30.1 us; M = 2048: 77 to 112 us against 75 us), so they are not instantiated.
#define BL_GEMM_FORMS(X) \
    X(1, 2, 1, 4) X(1, 4, 1, 4) X(2, 2, 1, 4) X(2, 3, 1, 4) X(2, 4, 1, 4) X(2, 2, 2, 2) X(2, 4, 2, 2)

}  // namespace

void set_gemm_mb(int mb) { g_force_mb = mb; }

bool gemm_form_exists(int code) {
    const TileForm f = form_of_code(code);
#define X(MB, H, WK, WN) if (f.mb == MB && f.h == H && f.wk == WK && f.wn == WN) return true;
    BL_GEMM_FORMS(X)
#undef X
    return false;
}

hipError_t launch_gemm(const GemmProblem& p, int64_t M, hipStream_t s) {
    const int64_t rows = (int64_t)p.row_blocks * kTileN;
    const TileForm f = choose_tile(M, rows);
    const int64_t gx = (rows + f.wn * f.h * 32 - 1) / (f.wn * f.h * 32);
    const int64_t gy = (M + 32 * f.mb - 1) / (32 * f.mb);
    const int64_t wgs_total = (gx + kXcds - 1) / kXcds * kXcds * gy;
    if (wgs_total > INT32_MAX) return hipErrorInvalidValue;
    note_kernel("gemm_kernel<%d, %d, %d, %d>", (int)wgs_total, f.mb, f.h, f.wk, f.wn);
#define X(MB, H, WK, WN)                                                                                                 \
    if (f.mb == MB && f.h == H && f.wk == WK && f.wn == WN)                                                              \
        return launch_form(&gemm_kernel<MB, H, WK, WN>, gemm_lds_bytes<MB, H, WK, WN>(), 64 * WN * WK, (unsigned)wgs_total, p, \
                           (int)M, (int)gx, s);
    BL_GEMM_FORMS(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_batch(const GemmProblem* ps, int count, int64_t M, hipStream_t s) {
    if (count == 1) return launch_gemm(ps[0], M, s);
    if (count < 1 || count > kMaxGemmBatch) return hipErrorInvalidValue;
    int64_t rows = 0;
    for (int i = 0; i < count; ++i) rows += (int64_t)ps[i].row_blocks * kTileN;
    const TileForm f = choose_tile(M, rows);
    GemmBatch b;
    int64_t gx = 0;
    for (int i = 0; i < kMaxGemmBatch; ++i) {
        b.p[i] = ps[i < count ? i : count - 1];
        if (i < count) gx += ((int64_t)ps[i].row_blocks * kTileN + f.wn * f.h * 32 - 1) / (f.wn * f.h * 32);
        b.end[i] = i + 1 < count ? (int32_t)gx : INT32_MAX;
    }
    const int64_t gy = (M + 32 * f.mb - 1) / (32 * f.mb);
    const int64_t wgs_total = (gx + kXcds - 1) / kXcds * kXcds * gy;
    if (wgs_total > INT32_MAX) return hipErrorInvalidValue;
    note_kernel("gemm_batch_kernel<%d, %d, %d, %d>", (int)wgs_total, f.mb, f.h, f.wk, f.wn);
#define X(MB, H, WK, WN)                                                                                                 \
    if (f.mb == MB && f.h == H && f.wk == WK && f.wn == WN)                                                              \
        return launch_form(&gemm_batch_kernel<MB, H, WK, WN>, gemm_lds_bytes<MB, H, WK, WN>(), 64 * WN * WK, (unsigned)wgs_total, b, \
                           (int)M, (int)gx, s);
    BL_GEMM_FORMS(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace bl
