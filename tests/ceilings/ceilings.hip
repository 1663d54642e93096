// Measured denominators for the roofline fractions bench.py reports (test and benchmark infrastructure; NOT part of
// libbitlinear.so and never called by it).  Two questions, each answered by the simplest kernel that can answer it:
//
//   ceil_mfma_loop    how many int8 operations per second do the matrix cores deliver when nothing else is in the way?
//                     A register-only loop of independent v_mfma_i32_32x32x32_i8 (no memory, no LDS, no barrier),
//                     optionally with the prefill kernel's in-register expansion of 2-bit codes between the MFMAs.
//   ceil_stream_read  how fast can a kernel read N bytes from HBM once, with 128-bit loads and nothing to compute?
//                     Every wave walks 1 KiB chunks (64 lanes x 16 bytes, the decode kernels' load shape), U loads in
//                     flight, and folds what it reads into one register so that the loads cannot be dropped; with
//                     ordinary or streaming (nontemporal) loads, chunks dealt round-robin or in one range per wave.
//
// Both take a stream and return the hipError_t of the launch; timing is the caller's (events around graph replays).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ v4i codes_to_bytes(uint32_t word) {   // 16 two-bit codes -> 16 int8, as the prefill kernel does
    v4i r;
    r[0] = (int)(word & 0x03030303u);
    r[1] = (int)((word >> 2) & 0x03030303u);
    r[2] = (int)((word >> 4) & 0x03030303u);
    r[3] = (int)((word >> 6) & 0x03030303u);
    return r;
}

// EXPAND false: operands are loop constants.  EXPAND true: the B operands are expanded from loop-carried packed words
// (7 vector ALU operations per operand, two operands per four MFMAs: the prefill kernel's ratio).
template <bool EXPAND>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, int* out) {
    v4i a0 = {(int)threadIdx.x, 1, 2, 3}, a1 = {(int)threadIdx.x + 1, 1, 2, 3};
    v4i b0 = {4, 5, (int)blockIdx.x, 7}, b1 = {1, 2, 3, (int)blockIdx.x};
    uint32_t w0 = threadIdx.x * 2654435761u, w1 = w0 ^ 0x55555555u;
    v16i c[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) c[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if constexpr (EXPAND) {
                b0 = codes_to_bytes(w0);
                b1 = codes_to_bytes(w1);
                w0 = w0 * 3u + 1u;          // loop-carried, so the expansion cannot be hoisted out of the loop
                w1 += w0;
            }
            c[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, c[0], 0, 0, 0);
            c[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b1, c[1], 0, 0, 0);
            c[2] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b0, c[2], 0, 0, 0);
            c[3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, c[3], 0, 0, 0);
        }
    }
    int s = 0;
    for (int i = 0; i < 4; ++i) s += c[i][0] + c[i][15];
    if (s == 0x7fffffff) out[threadIdx.x] = s;   // keeps the loop alive; practically never true
}

// NT: streaming (nontemporal) loads.  RANGES: every wave reads one contiguous range of chunks instead of every
// (number of waves)-th chunk.
template <int U, bool NT, bool RANGES>
__global__ __launch_bounds__(1024) void stream_read_kernel(const uint4* __restrict__ src, int64_t chunks, uint32_t* out) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t waves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int64_t per = (chunks + waves - 1) / waves;
    const int64_t first = RANGES ? wave * per : wave, step = RANGES ? 1 : waves;
    const int64_t end = RANGES ? (first + per < chunks ? first + per : chunks) : chunks;
    uint32_t fold = 0;
    for (int64_t c = first; c < end; c += step * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t cc = c + u * step;
            const uint4* p = src + (cc < end ? cc : end - 1) * 64 + lane;   // beyond the end: the last chunk again (a cache hit)
            if constexpr (NT) {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
                v[u] = make_uint4(t[0], t[1], t[2], t[3]);
            } else {
                v[u] = *p;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) fold ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (fold == 0x12345678u) out[(wave * 64 + lane) & 1023] = fold;   // practically never: no store traffic
}

template <int U>
hipError_t launch_read(const uint4* src, int64_t chunks, uint32_t* out, int wgs, int threads, int flags, hipStream_t s) {
    switch (flags & 3) {
        case 0: stream_read_kernel<U, false, false><<<wgs, threads, 0, s>>>(src, chunks, out); break;
        case 1: stream_read_kernel<U, true, false><<<wgs, threads, 0, s>>>(src, chunks, out); break;
        case 2: stream_read_kernel<U, false, true><<<wgs, threads, 0, s>>>(src, chunks, out); break;
        default: stream_read_kernel<U, true, true><<<wgs, threads, 0, s>>>(src, chunks, out); break;
    }
    return hipGetLastError();
}

}  // namespace

extern "C" {

// 8 MFMAs of 2 * 32 * 32 * 32 operations per iteration and wave; blocks x 4 waves.  out_dev: at least 256 ints.
int ceil_mfma_ops_per_wave_iter(void) { return 8 * 2 * 32 * 32 * 32; }

int ceil_mfma_loop(int expand, int blocks, int iters, void* out_dev, void* stream) {
    if (blocks < 1 || iters < 1 || !out_dev) return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (expand) mfma_loop_kernel<true><<<blocks, 256, 0, s>>>(iters, static_cast<int*>(out_dev));
    else mfma_loop_kernel<false><<<blocks, 256, 0, s>>>(iters, static_cast<int*>(out_dev));
    return (int)hipGetLastError();
}

// Reads `bytes` (a multiple of 1024, 16-byte aligned) once.  threads: multiple of 64 up to 1024; unroll: 4, 8 or 16;
// flags: bit 0 = streaming (nontemporal) loads, bit 1 = one contiguous range per wave.  out_dev: at least 1024 words.
int ceil_stream_read(const void* src_dev, int64_t bytes, void* out_dev, int wgs, int threads, int unroll, int flags, void* stream) {
    if (!src_dev || !out_dev || bytes < 1024 || bytes % 1024 != 0 || wgs < 1 || threads < 64 || threads > 1024 ||
        threads % 64 != 0 || (reinterpret_cast<uintptr_t>(src_dev) & 15) != 0 || flags < 0 || flags > 3)
        return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint4* src = static_cast<const uint4*>(src_dev);
    uint32_t* out = static_cast<uint32_t*>(out_dev);
    const int64_t chunks = bytes / 1024;
    switch (unroll) {
        case 4: return (int)launch_read<4>(src, chunks, out, wgs, threads, flags, s);
        case 8: return (int)launch_read<8>(src, chunks, out, wgs, threads, flags, s);
        case 16: return (int)launch_read<16>(src, chunks, out, wgs, threads, flags, s);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // extern "C"
