// A 1.78-bit weight layout built on the paper's TL2 code (Section 2 and Table 3 of arXiv 2410.16144:
// three ternary weights -> one sign bit and a 4-bit index, index = |9 w0 + 3 w1 + w2|, sign = 1 iff
// that sum is negative), with its pack / unpack kernels and a one-token decode product.
//
// The paper's TL2 kernel looks up partial sums of ACTIVATION triples by weight code; that replaces
// multiplies, which a GPU's dot-product units give for free.  What carries over is the code: it
// stores three weights in 5 bits, so the stream from HBM -- the bound of the decode product -- is
// shorter.  Here the table is the other way round: 32 entries, code -> the three weights as int8
// (fourth byte zero), one 32-bit word each, in LDS.  32 words lie in 32 different banks, so the
// lookups of a wavefront never conflict, whatever the codes.  Per group of three weights the kernel
// spends a shift and a mask (table address), one LDS read and one v_dot4_i32_i8 against the three
// activations (the dot product's fourth byte meets the entry's zero): 1.0 vector operation per
// weight against 0.56 for the 2-bit layout, for 11 % fewer bytes.
//
// Layout (version 2).  Tiles of 64 rows x 72 k = 1 KiB, tile (rb, kc) at byte ((rb * KC) + kc) * 1024
// with KC = Kp / 72; the 16 bytes at offset 16 r belong to row 64 rb + r (one 128-bit load per lane,
// as in the 2-bit layout).  They are four 32-bit words; word s holds groups i = 0..5, group i =
// weights k = 72 kc + 18 s + 3 i + {0, 1, 2}, its code (sign << 4 | index) at bits [5 i, 5 i + 4];
// bits 30 and 31 are zero.  Rows beyond N and k beyond K are zero weights (code 0).
#include "bl_internal.hpp"

namespace bl {

namespace {

constexpr int kGroupsPerWord = 6;
constexpr int kWordsPerTile = 256;   // 64 lanes x 4 words
constexpr int kWaves = 16;
constexpr int kThreads = kWaves * kWave;
constexpr int kInFlight = 8;         // weight tiles a wave keeps in flight

// code -> the three weights, as the table of the decode kernel and of unpack: balanced-ternary digits of the
// index (most significant first), negated if the sign bit is set.  Codes that Table 3 does not use give zeros.
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

// word index of the blob -> (row, first k)
__device__ __forceinline__ void word_coords(int64_t word, int64_t KC, int64_t& row, int64_t& k0) {
    const int64_t tile = word / kWordsPerTile;
    const int in_tile = (int)(word - tile * kWordsPerTile);
    const int64_t rb = tile / KC, kc = tile - rb * KC;
    row = rb * kTileN + (in_tile >> 2);
    k0 = kc * BL_TL2_TILE_K + (in_tile & 3) * 3 * kGroupsPerWord;
}

__global__ __launch_bounds__(256) void tl2_pack_kernel(const int8_t* __restrict__ w, int64_t N, int64_t K, int64_t KC,
                                                       int64_t words, uint32_t* __restrict__ packed,
                                                       int32_t* __restrict__ bad_count) {
    const int64_t word = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (word >= words) return;
    int64_t row, k0;
    word_coords(word, KC, row, k0);
    uint32_t out = 0;
    int bad = 0;
#pragma unroll
    for (int i = 0; i < kGroupsPerWord; ++i) {
        int t[3];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int64_t k = k0 + 3 * i + j;
            t[j] = (row < N && k < K) ? w[row * K + k] : 0;
            if (t[j] < -1 || t[j] > 1) { t[j] = 0; ++bad; }
        }
        const int v = 9 * t[0] + 3 * t[1] + t[2];
        out |= (uint32_t)((v < 0 ? 16 : 0) | (v < 0 ? -v : v)) << (5 * i);
    }
    packed[word] = out;
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

__global__ __launch_bounds__(256) void tl2_unpack_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                         int64_t KC, int64_t words, int8_t* __restrict__ w) {
    const int64_t word = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (word >= words) return;
    int64_t row, k0;
    word_coords(word, KC, row, k0);
    if (row >= N) return;
    const uint32_t v = packed[word];
#pragma unroll
    for (int i = 0; i < kGroupsPerWord; ++i) {
        int t[3];
        tl2_weights((int)(v >> (5 * i)) & 31, t);
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int64_t k = k0 + 3 * i + j;
            if (k < K) w[row * K + k] = (int8_t)t[j];
        }
    }
}

// The three activations that meet group g (0..23) of a tile, as the low three bytes of a word.  qk: the tile's 72
// activations as 18 words (wave-uniform: scalar loads, scalar shifts); the fourth byte is whatever follows and
// meets the table entry's zero byte.
__device__ __forceinline__ int group_activations(const int32_t* __restrict__ qk, int g) {
    // read as 64-bit pairs (a tile's activations start at a multiple of 8 bytes): from two separate 32-bit loads
    // the compiler would build ONE unaligned 32-bit load for a group that straddles two words, which has to be a
    // vector load, and waiting for that one drains the weight tiles in flight
    const int2* __restrict__ q2 = reinterpret_cast<const int2*>(qk);
    const int word = (3 * g) >> 2, off = (3 * g) & 3;
    const auto at = [&](int wd) { return (uint32_t)((wd & 1) ? q2[wd >> 1].y : q2[wd >> 1].x); };
    if (off == 0) return (int)at(word);
    if (off == 1) return (int)(at(word) >> 8);
    const uint64_t pair = at(word) | ((uint64_t)at(word + 1) << 32);
    return (int)(uint32_t)(pair >> (8 * off));
}

// One-token decode product.  Workgroup = 16 waves; lane r of a wave owns row r of a 64-row block; the block's K
// tiles are dealt round-robin to G = 2^wlog2 waves, whose partial sums meet once in LDS.  Signed weights come
// out of the table, so there is no sum(q) correction.
__global__ __launch_bounds__(kThreads, 8) void tl2_gemv_kernel(const uint4* __restrict__ packed,
                                                               const int32_t* __restrict__ q,
                                                               const float* __restrict__ a_scale,
                                                               float* __restrict__ out, int32_t* __restrict__ acc_out,
                                                               int N, int KC, int row_blocks, float w_scale,
                                                               int wlog2) {
    __shared__ int lut[32];
    __shared__ int red[kWaves * kWave];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid < 32) {
        int t[3];
        tl2_weights(tid, t);
        lut[tid] = (t[0] & 0xff) | (t[1] & 0xff) << 8 | (t[2] & 0xff) << 16;
    }
    const int G = 1 << wlog2;
    const int ks = wave & (G - 1);
    const int rb = blockIdx.x * (kWaves >> wlog2) + (wave >> wlog2);
    const uint4* __restrict__ wp = packed + (int64_t)min(rb, row_blocks - 1) * KC * kWave + lane;   // clamped: valid memory
    uint4 w[kInFlight];
    auto load_batch = [&](int kc0) {
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) w[u] = wp[(int64_t)min(kc0 + u * G, KC - 1) * kWave];
    };
    load_batch(ks);
    __syncthreads();   // the table is in place
    int part[3] = {0, 0, 0};   // independent sums: the dot products of a word do not wait for one another
    for (int kc0 = ks; kc0 < KC; kc0 += G * kInFlight) {
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int kc = kc0 + u * G;
            if (kc < KC) {   // uniform
                const int32_t* __restrict__ qk = q + kc * (BL_TL2_TILE_K / 4);
                const uint32_t word[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
                // the table entries of a word are fetched while the previous word's dot products run
                int e[2][kGroupsPerWord];
#pragma unroll
                for (int i = 0; i < kGroupsPerWord; ++i) e[0][i] = lut[(word[0] >> (5 * i)) & 31];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    if (s < 3) {
#pragma unroll
                        for (int i = 0; i < kGroupsPerWord; ++i) e[(s + 1) & 1][i] = lut[(word[s + 1] >> (5 * i)) & 31];
                    }
#pragma unroll
                    for (int i = 0; i < kGroupsPerWord; ++i)
                        part[i % 3] = __builtin_amdgcn_sdot4(e[s & 1][i], group_activations(qk, kGroupsPerWord * s + i),
                                                             part[i % 3], false);
                }
            }
        }
        if (kc0 + G * kInFlight < KC) load_batch(kc0 + G * kInFlight);
    }
    const int acc = part[0] + part[1] + part[2];
    red[wave * kWave + lane] = acc;
    __syncthreads();
    if (ks == 0 && rb < row_blocks) {
        int total = 0;
        for (int g = 0; g < G; ++g) total += red[(wave + g) * kWave + lane];
        const int n = rb * kTileN + lane;
        if (n < N) {
            out[n] = (float)total * (w_scale * a_scale[0]);
            if (acc_out) acc_out[n] = total;
        }
    }
}

}  // namespace

hipError_t launch_tl2_pack(const int8_t* w, int64_t N, int64_t K, int64_t Np, int64_t Kp, uint32_t* packed,
                           int32_t* bad_count, hipStream_t s) {
    const int64_t KC = Kp / BL_TL2_TILE_K, words = (Np / kTileN) * KC * kWordsPerTile;
    const int64_t blocks = (words + 255) / 256;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    tl2_pack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(w, N, K, KC, words, packed, bad_count);
    return hipGetLastError();
}

hipError_t launch_tl2_unpack(const uint32_t* packed, int64_t N, int64_t K, int64_t Np, int64_t Kp, int8_t* w,
                             hipStream_t s) {
    const int64_t KC = Kp / BL_TL2_TILE_K, words = (Np / kTileN) * KC * kWordsPerTile;
    const int64_t blocks = (words + 255) / 256;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    tl2_unpack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(packed, N, K, KC, words, w);
    return hipGetLastError();
}

hipError_t launch_tl2_gemv(const uint4* packed, const int32_t* q, const float* a_scale, float* out, int32_t* acc,
                           int64_t N, int64_t Np, int64_t Kp, float w_scale, hipStream_t s) {
    const int KC = (int)(Kp / BL_TL2_TILE_K), row_blocks = (int)(Np / kTileN);
    // waves per row block: about 8 tiles per wave, then more waves per block until every compute unit has a workgroup
    int wlog2 = 0;
    while (wlog2 < 4 && (KC >> (wlog2 + 1)) >= kInFlight) ++wlog2;
    const int cus = compute_unit_count();
    while (wlog2 < 4 && (KC >> (wlog2 + 1)) >= 1 && (row_blocks + (kWaves >> wlog2) - 1) / (kWaves >> wlog2) < cus) ++wlog2;
    const int per_wg = kWaves >> wlog2;
    const int64_t grid = (row_blocks + per_wg - 1) / per_wg;
    if (grid > INT32_MAX) return hipErrorInvalidValue;
    tl2_gemv_kernel<<<dim3((unsigned)grid), dim3(kThreads), 0, s>>>(packed, q, a_scale, out, acc, (int)N, KC, row_blocks,
                                                                    w_scale, wlog2);
    return hipGetLastError();
}

}  // namespace bl
