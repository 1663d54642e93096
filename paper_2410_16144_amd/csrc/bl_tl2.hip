// A 1.78-bit weight layout built on the paper's TL2 code (Section 2 and Table 3 of arXiv 2410.16144:
// three ternary weights -> one sign bit and a 4-bit index, index = |9 w0 + 3 w1 + w2|, sign = 1 iff
// that sum is negative): its pack / unpack kernels.  The decode product over this layout is a form of the decode
// kernels (LAYOUT = 2 in bl_gemv.hip and bl_decode_sk.hip; the arithmetic is tl2_tile_mac in bl_decode_device.hpp).
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
#include "bl_decode_device.hpp"

namespace bl {

namespace {

constexpr int kGroupsPerWord = kTl2GroupsPerWord;
constexpr int kWordsPerTile = 256;   // 64 lanes x 4 words

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

}  // namespace bl
