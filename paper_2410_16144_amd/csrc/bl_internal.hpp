// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bitlinear.h"
#include "bitlinear_decoder.h"

namespace bl {

constexpr int kTileN = BL_TILE_N;            // rows per packed tile = lanes per wavefront
constexpr int kTileK = BL_TILE_K;            // k per packed tile
constexpr int kTileBytes = kTileN * kTileK / 4;  // 1 KiB: one 128-bit load per lane
constexpr int kWave = 64;

// 16 two-bit codes of a packed word -> 16 int8 (one matrix-core operand register quadruple): byte b of element j is
// the code at bits [8 b + 2 j, 8 b + 2 j + 1], i.e. k-offset 4 j + b of the word.
typedef int v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4i expand_codes(uint32_t word) {
    v4i r;
    r[0] = (int)(word & 0x03030303u);
    r[1] = (int)((word >> 2) & 0x03030303u);
    r[2] = (int)((word >> 4) & 0x03030303u);
    r[3] = (int)((word >> 6) & 0x03030303u);
    return r;
}

// One prefill product as the kernel sees it (all device pointers).
struct GemmProblem {
    const uint4*   packed;
    const int32_t* q;        // int8 activations viewed as 32-bit words, row stride Kp/4 words
    const float*   a_scale;
    const int32_t* q_sum;
    float*         out;
    int32_t*       acc;      // may be null
    int32_t        N;
    int32_t        KC;       // Kp / 64: tiles along K
    int32_t        row_blocks;  // Np / 64
    float          w_scale;
};

// One decode problem with its launch geometry; the fused form also carries the raw activations.
struct DecodeProblem {
    const uint4*   packed;
    const int32_t* q;            // plain form: int8 activations as 32-bit words, row stride Kp/4
    const float*   a_scale;      // plain form
    const int32_t* q_sum;        // plain form
    float*         out;
    int32_t*       acc;          // may be null
    const void*    x;            // fused form: [M, ldx] fp32 or bf16
    int64_t        ldx;
    int8_t*        q_out;        // fused form, optional copies of the quantizer's results
    float*         a_scale_out;
    int32_t*       q_sum_out;
    int32_t        N, K, KC, row_blocks;
    float          w_scale;
    int32_t        x_flags;      // bit 0: bf16, bit 1: 128-bit vector loads allowed
    int32_t        wlog2;        // log2(waves that share one row block)
    int32_t        first_wg;     // first workgroup of this problem in the grid
    int32_t        chunk;        // balanced form: tiles per workgroup
    int32_t        input;        // publishing form: which distinct input this problem reads
    // fused form with RMSNorm (one token, fp32 x, K <= 16384): activations = quantize((x + delta) * gamma); the norm's
    // scalar 1 / sqrt(mean((x + delta)^2) + eps) multiplies the activation scale instead of every element
    const float*   gamma;        // [K]; null: no norm
    const float*   delta;        // optional [K]
    float*         h_out;        // optional [K]: receives x + delta (written by the problem's first workgroup)
    float          eps;
    // ... or the row arrives already multiplied by its norm weight, with sum(x^2) in pieces (the gated epilogue below)
    const float2*  ss_in;        // [ss_count] pieces (sum of squares, absmax) as the gated epilogue leaves them; null unless this form
    int32_t        ss_count;
    // gated epilogue (row-block kernel, one token): the matrix holds gate and up rows interleaved by 32, lanes 0-31 of a
    // row block the gate rows, lanes 32-63 the up rows of the same 32 outputs; out[n] = silu(gate) * up * glu_gamma[n],
    // ss_out[row block] = (sum over its 32 outputs of (silu(gate) * up)^2, max over them of |out|)
    const float*   glu_gamma;    // [N / 2]; null: plain epilogue
    float2*        ss_out;       // [row_blocks]
    float          w_scale2;     // the up rows' weight scale (w_scale: the gate rows')
};

struct DecodeBatch {
    DecodeProblem p[BL_MAX_BATCH];
    int32_t       count;
    int32_t       total_wgs;
    unsigned long long* ws;      // balanced form: the caller's workspace (zero between launches), or null
    int32_t       layout;        // 1: 2-bit tiles of 64 k; 2: TL2 codes, tiles of 72 k (one token, plain form only)
    int32_t       stream;        // host side only: weight tiles by streaming (nontemporal) loads; set by launch_decode
    // publishing form (2..8 tokens, fused): the launch's first pub_rows workgroups quantize one token row of one distinct
    // input each and publish it; the others wait for their input's rows (see decode_mfma_kernel)
    int32_t       pub_rows;      // 0: not this form
    int32_t       pub_limit;     // polls before a waiting workgroup gives up
    int32_t       pub_src[BL_MAX_BATCH];   // distinct input i -> a problem that reads it
    unsigned int* pub_ctr;       // counters in the caller's workspace: see kPub* below
};

// DecodeBatch::pub_ctr: the last kPubBytes of the workspace, all zero between launches like the rest of it.  Hundreds
// of waiting workgroups polling ONE word queue up at one memory channel in front of the very update they are waiting
// for (measured: a 13 us launch took 33), so every "rows ready" counter exists in kPubCopies copies, kPubStride words
// apart: a quantizer adds to all of them, a waiter polls the copy of its workgroup index.
constexpr int kPubCopies = 16;
constexpr int kPubStride = 64;                                   // words: 256 bytes between copies
constexpr int kPubReady = 0;                                     // [input][copy]: word (input * kPubCopies + copy) * kPubStride
constexpr int kPubDone = BL_MAX_BATCH * kPubCopies * kPubStride; // waiting workgroups that have got past their wait
constexpr int kPubStatus = kPubDone + kPubStride;                // set to 1 by a workgroup whose wait gave up; sticky
constexpr int kPubBytes = (kPubStatus + kPubStride) * 4;
static_assert(kPubBytes <= BL_WORKSPACE_BYTES / 4, "the counters live in the workspace's tail");

// Which problem of the launch a workgroup belongs to.  The first workgroup of problems 1..7 (INT32_MAX beyond the
// launch's count) LEADS the argument list of the decode and quantization kernels as seven scalars, because their files are
// compiled with kernel-argument preload (-amdgpu-kernarg-preload-count=7): a kernel's first scalar arguments
// arrive in registers with the wave, so a workgroup knows its problem without a round trip to memory and the
// scalar loads of that problem's fields go out at once -- one dependent round before the first weight tile can be
// requested instead of two (0.4 us per launch on MI355X).  Without the compiler option, or on firmware that does
// not preload, the same code reads them from the argument segment as before.
#define BL_FIRST_WG_PARAMS \
    const int fw1, const int fw2, const int fw3, const int fw4, const int fw5, const int fw6, const int fw7
#define BL_FIRST_WG_ARGS(f) (f).v[1], (f).v[2], (f).v[3], (f).v[4], (f).v[5], (f).v[6], (f).v[7]
#define BL_PROBLEM_OF(blk) \
    (((blk) >= fw1) + ((blk) >= fw2) + ((blk) >= fw3) + ((blk) >= fw4) + ((blk) >= fw5) + ((blk) >= fw6) + ((blk) >= fw7))
static_assert(BL_MAX_BATCH == 8, "seven leading arguments");

// One activation matrix of a quantization launch.
struct QuantProblem {
    const void* x;
    int8_t*     q;
    float*      a_scale;
    int32_t*    q_sum;        // may be null
    int64_t     ldx;
    int32_t     M, K, Kp;
    int32_t     flags;        // bit 0: bf16, bit 1: 128-bit vector loads allowed
    int32_t     first_row;    // first workgroup of this matrix in the grid
};

struct QuantBatch {
    QuantProblem p[BL_MAX_BATCH];
    int32_t      count;
};

constexpr int kMaxDecodeLds = 128 * 1024;   // dynamic LDS ceiling of the decode kernels

// Raises one kernel's dynamic-LDS ceiling to kMaxDecodeLds, once per device (the setting belongs to the device the
// call is made on): a host-side attribute, no allocation.  One object per kernel; a repeated call from another
// thread is harmless.
struct LdsCeiling {
    uint64_t done = 0;   // one bit per device ordinal below 64; other devices set the attribute on every launch
    hipError_t ensure(const void* kernel) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
        if (dev >= 0 && ((done >> dev) & 1)) return hipSuccess;
        const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDecodeLds);
        if (e == hipSuccess && dev >= 0) done |= 1ull << dev;
        return e;
    }
};

// Launchers (each returns the hipError_t of its launch).
hipError_t launch_pack(const int8_t* w, const int8_t* w_up /* null: plain; else gate/up interleaved by 32 */, int64_t N,
                       int64_t K, int64_t Np, int64_t Kp, uint32_t* packed, int32_t* bad_count, hipStream_t s);
hipError_t launch_unpack(const uint32_t* packed, int64_t N, int64_t K, int64_t Np, int64_t Kp, int8_t* w,
                         hipStream_t s);
hipError_t launch_quant(const QuantBatch& b, hipStream_t s);
size_t decode_lds_bytes(int M, int64_t max_Kp, bool fused);
hipError_t launch_decode(const DecodeBatch& b, int M, bool fused, hipStream_t s);
int compute_unit_count();   // of the current device; 0 if unknown
int decode_split_grid(const DecodeBatch& b, bool fused);   // workgroups of the balanced form for this batch; 0: not chosen
bool plan_decode_split(DecodeBatch& b, bool fused, int& tiles_per_wave);   // false: the balanced form does not apply
hipError_t launch_decode_split(const DecodeBatch& b, int tiles_per_wave, bool fused, hipStream_t s);
hipError_t launch_gemm(const GemmProblem& p, int64_t M, hipStream_t s);
constexpr int kMaxGemmBatch = BL_MAX_GEMM_BATCH;
hipError_t launch_gemm_batch(const GemmProblem* ps, int count, int64_t M, hipStream_t s);   // 1 <= count <= kMaxGemmBatch
hipError_t launch_tl2_pack(const int8_t* w, int64_t N, int64_t K, int64_t Np, int64_t Kp, uint32_t* packed,
                           int32_t* bad_count, hipStream_t s);
hipError_t launch_tl2_unpack(const uint32_t* packed, int64_t N, int64_t K, int64_t Np, int64_t Kp, int8_t* w,
                             hipStream_t s);


// The decoder block around the products (bl_decoder.hip); arguments already validated.
hipError_t launch_norm_quant(const ::bl_norm_quant_args& a, hipStream_t s);
hipError_t launch_rope_table(float* table, int head_dim, int max_pos, double theta, hipStream_t s);
int attn_chunks(int max_pos);
hipError_t launch_attn_decode(const ::bl_attn_args& a, hipStream_t s);
hipError_t launch_pos_advance(int32_t* pos, hipStream_t s);
hipError_t launch_attn_prefill(const ::bl_attn_prefill_args& a, hipStream_t s);

// The calling thread's most recent product launch: kernel template instance and grid, for tools that label what they
// time (bl_last_kernel).  Only the pieces are stored at launch time; the text is formatted on request.
struct KernelNote {
    const char* fmt = nullptr;   // format over v[]: %d a number, %b true / false
    int v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int grid = 0;
};
extern thread_local KernelNote t_kernel_note;
inline void note_kernel(const char* fmt, int grid, int a = 0, int b = 0, int c = 0, int d = 0, int e = 0, int f = 0, int g = 0,
                        int h = 0) {
    t_kernel_note.fmt = fmt;
    t_kernel_note.grid = grid;
    const int v[8] = {a, b, c, d, e, f, g, h};
    for (int i = 0; i < 8; ++i) t_kernel_note.v[i] = v[i];
}

// Launch-shape overrides for experiments (0 = choose automatically).
void set_gemv_waves(int waves);
void set_attn_groups(int groups);   // bl_attn_decode's workgroups per head; 0 automatic
void set_gemm_mb(int mb);         // 0 automatic, else 1000*W + 100*(WK-1) + 10*MB + H (see bl_gemm.hip)
bool gemm_form_exists(int code);  // whether that code names a tile form the library has
void set_decode_stage(int v);     // 1: the matrix-core decode kernel never stages activations in LDS
void set_decode_split(int v);     // -1 never split row blocks over workgroups, 0 automatic, n: n workgroups per compute unit
void set_decode_path(int path);   // 0 automatic, 1 dot-product kernel, 2 matrix-core kernel
void set_decode_publish(int v);   // fused launches of 2..8 tokens quantize each input once and publish it: 0 when possible, -1 never
void set_decode_wait_limit(int v);   // polls before a waiting workgroup gives up (0: the default)
void set_decode_stream(int v);    // weight tiles by streaming loads: 0 automatic (by the launch's packed bytes), 1 always, -1 never
int64_t split_launches();         // work-balanced decode launches so far (host-side count)

}  // namespace bl
