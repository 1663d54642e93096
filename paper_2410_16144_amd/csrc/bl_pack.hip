// bl_pack_ternary / bl_unpack_ternary: the offline I2_S transformation (Table 1 of
// arXiv 2410.16144: -1 -> 00, 0 -> 01, +1 -> 10) into the 64x64-tiled layout that the
// decode and prefill kernels stream, and its inverse.
//
// One thread produces (or consumes) one 32-bit word = 16 weights of one row.  Consecutive
// threads own consecutive words of the blob, so blob accesses are fully coalesced; the
// row-major int8 matrix is touched in 64-byte runs.
#include "bl_internal.hpp"

namespace bl {

namespace {

// word index -> (row, first k) under the version-1 layout
__device__ __forceinline__ void word_coords(int64_t word, int64_t KC, int64_t& row, int64_t& k0) {
    int64_t tile = word >> 8;          // 256 words per 1 KiB tile
    int r = (int)(word & 255) >> 2;    // lane / row inside the tile
    int s = (int)(word & 3);           // which 16-k piece
    int64_t rb = tile / KC;
    int64_t kc = tile - rb * KC;
    row = rb * kTileN + r;
    k0 = kc * kTileK + s * 16;
}

// w_up == nullptr: rows of the packed matrix are rows of w.  Otherwise the gated form's interleave: packed row block b holds
// rows 32 b .. 32 b + 31 of w (gate) in its rows 0-31 and the same rows of w_up in its rows 32-63; N counts packed rows.
__global__ __launch_bounds__(256) void pack_kernel(const int8_t* __restrict__ w, const int8_t* __restrict__ w_up, int64_t N,
                                                   int64_t K, int64_t KC, int64_t words, uint32_t* __restrict__ packed,
                                                   int32_t* __restrict__ bad_count) {
    int64_t word = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (word >= words) return;
    int64_t row, k0;
    word_coords(word, KC, row, k0);
    const bool in_matrix = row < N;
    if (w_up) {
        if (row & 32) w = w_up;
        row = (row >> 6) * 32 + (row & 31);
    }
    uint32_t out = 0;
    int bad = 0;
    const bool fast = in_matrix && k0 + 16 <= K && ((reinterpret_cast<uintptr_t>(w) + row * K + k0) & 15) == 0;
    if (fast) {
        uint4 v = *reinterpret_cast<const uint4*>(w + row * K + k0);
        uint32_t src[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                int val = (int)(int8_t)(src[j] >> (8 * b));
                if (val < -1 || val > 1) { val = 0; ++bad; }
                out |= (uint32_t)(val + 1) << (8 * b + 2 * j);
            }
        }
    } else {
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            int val = 0;  // padding weight
            if (in_matrix && k0 + t < K) {
                val = w[row * K + k0 + t];
                if (val < -1 || val > 1) { val = 0; ++bad; }
            }
            out |= (uint32_t)(val + 1) << (8 * (t & 3) + 2 * (t >> 2));
        }
    }
    packed[word] = out;
    if (bad && bad_count) atomicAdd(bad_count, bad);
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                     int64_t KC, int64_t words, int8_t* __restrict__ w) {
    int64_t word = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (word >= words) return;
    int64_t row, k0;
    word_coords(word, KC, row, k0);
    if (row >= N) return;
    uint32_t v = packed[word];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        if (k0 + t < K) {
            int code = (v >> (8 * (t & 3) + 2 * (t >> 2))) & 3;
            w[row * K + k0 + t] = (int8_t)(code == 3 ? 0 : code - 1);
        }
    }
}

}  // namespace

hipError_t launch_pack(const int8_t* w, const int8_t* w_up, int64_t N, int64_t K, int64_t Np, int64_t Kp, uint32_t* packed,
                       int32_t* bad_count, hipStream_t s) {
    int64_t words = Np * Kp / 16;
    int64_t blocks = (words + 255) / 256;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    pack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(w, w_up, N, K, Kp / kTileK, words, packed, bad_count);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t* packed, int64_t N, int64_t K, int64_t Np, int64_t Kp, int8_t* w,
                         hipStream_t s) {
    int64_t words = Np * Kp / 16;
    int64_t blocks = (words + 255) / 256;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    unpack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(packed, N, K, Kp / kTileK, words, w);
    return hipGetLastError();
}

}  // namespace bl
