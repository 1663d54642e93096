/*
 * bitlinear.h -- C ABI of the MI355X (gfx950) BitLinear library.
 *
 * The library computes the BitNet b1.58 BitLinear product that the ternary
 * kernels of arXiv 2410.16144 (Section 2) accelerate:
 *
 *     out[m,n] = ( sum_k q[m,k] * W[n,k] ) * w_scale * a_scale[m]
 *
 * with W in {-1,0,+1}^{N x K} stored as 2-bit codes (Table 1: -1->00, 0->01,
 * +1->10), q the per-token absmax int8 quantization of the activations, the
 * sum taken exactly in int32 and one fp32 dequantization multiply at the end.
 *
 * General rules for every entry point
 *   - Pointers named *_dev are DEVICE pointers owned by the caller (allocate
 *     them any way you like, e.g. hipMalloc or a torch tensor's data_ptr()).
 *     Pointers without that suffix are HOST pointers, read during the call.
 *   - The library never allocates or frees device memory, never synchronizes
 *     and owns no stream: all work is enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL = the default stream) and the call returns at
 *     once.  Results are valid once the stream reaches that point.
 *   - Every call returns a bl_status.  Arguments are validated on the host
 *     BEFORE any HIP call, so a bad call has no effect on the device.
 *     A failed launch is reported as BL_ERR_HIP.
 *   - Nothing here is thread-hostile; calls that touch the same buffers on
 *     different streams race like any other GPU work.
 */
#ifndef BITLINEAR_H
#define BITLINEAR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BL_OK = 0,
    BL_ERR_NULL = 1,        /* a required pointer is NULL                         */
    BL_ERR_SHAPE = 2,       /* N, K, M or a stride is out of range                */
    BL_ERR_M_RANGE = 3,     /* bl_gemv / bl_gemv_batch called with M outside 1..8 */
    BL_ERR_BUF_SMALL = 4,   /* descriptor's byte count does not match its shape   */
    BL_ERR_ALIGN = 5,       /* a pointer is not aligned as documented             */
    BL_ERR_DTYPE = 6,       /* unknown bl_dtype                                   */
    BL_ERR_LAYOUT = 7,      /* descriptor version is not BL_LAYOUT_VERSION        */
    BL_ERR_HIP = 8,         /* the HIP runtime refused the launch                 */
    BL_ERR_COUNT = 9,       /* a batch call's count is outside its range          */
    BL_ERR_WORKSPACE = 10   /* bl_gemv_batch_static: launch exceeds the static scratch */
} bl_status;

typedef enum { BL_F32 = 0, BL_BF16 = 1 } bl_dtype;

#define BL_LAYOUT_VERSION 1
#define BL_TILE_N 64        /* rows (output features) per packed tile            */
#define BL_TILE_K 64        /* K extent per packed tile                           */
#define BL_MAX_K 1048576    /* keeps every int32 partial sum far from overflow    */
#define BL_MAX_GEMV_M 8
#define BL_MAX_BATCH 8
#define BL_MAX_GEMM_M 4194304
#define BL_MAX_GEMM_BATCH 4
#define BL_MAX_SPLIT_WGS 2048   /* most workgroups of a work-balanced decode launch     */
#define BL_WORKSPACE_BYTES (BL_MAX_SPLIT_WGS * 64 * 8)   /* 1 MiB, see bl_gemv_batch   */
#define BL_STATIC_WS_WGS 1024   /* workgroups the static scratch of bl_gemv_batch_static serves */
#define BL_STATIC_WS_BYTES (BL_STATIC_WS_WGS * 64 * 8)   /* 512 KiB per GPU              */

/*
 * Host-side description of one packed ternary matrix.  Plain data; copy it,
 * store it next to the blob.  The packed blob itself is position independent.
 *
 * Packed layout (version 1), chosen for 64-lane wavefronts: the matrix is
 * padded to Np x Kp (multiples of 64; padding weights are 0) and cut into
 * tiles of 64 rows x 64 k.  Tile (rb, kc) is the 1 KiB block at byte offset
 * ((rb * (Kp/64)) + kc) * 1024.  Inside a tile, the 16 bytes at offset 16*r
 * belong to row 64*rb + r (one 128-bit load per lane, 1 KiB per wavefront);
 * they are four little-endian 32-bit words s = 0..3, word s covering
 * k = 64*kc + 16*s + t, t = 0..15, with the code (w+1) of k-offset t = 4j + b
 * stored at bits [8b + 2j, 8b + 2j + 1].  Hence (word >> 2j) & 0x03030303 is
 * four byte-wide codes for four consecutive k, aligned with one 32-bit word
 * of int8 activations.
 */
typedef struct {
    int32_t  version;   /* BL_LAYOUT_VERSION                                   */
    int32_t  reserved;  /* 0                                                   */
    int64_t  N;         /* output features (rows of W)                         */
    int64_t  K;         /* input features (columns of W)                       */
    int64_t  Np;        /* N rounded up to BL_TILE_N                           */
    int64_t  Kp;        /* K rounded up to BL_TILE_K; also the row stride of q */
    uint64_t bytes;     /* size of the packed blob = Np * Kp / 4               */
    float    w_scale;   /* per-matrix (absmean) scale, used in the dequant     */
    float    reserved2; /* 0                                                   */
} bl_packed_desc;

/* K rounded up to the layout's K tile: the row stride (in bytes) of quantized
 * activations.  Returns -1 if K is outside 1..BL_MAX_K. */
int64_t bl_padded_k(int64_t K);

/* N rounded up to the layout's row tile.  Returns -1 if N < 1. */
int64_t bl_padded_n(int64_t N);

/* Fill *d for an N x K ternary matrix with dequantization scale w_scale.
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE (N < 1, K outside 1..BL_MAX_K). */
bl_status bl_packed_desc_init(int64_t N, int64_t K, float w_scale, bl_packed_desc *d);

/*
 * Offline weight transformation (Section 2, I2_S: every weight becomes a
 * 2-bit value, Table 1) into the tiled layout described above.
 *   w_dev         [N,K] int8, row-major, values in {-1,0,+1}
 *   d             host descriptor from bl_packed_desc_init
 *   packed_dev    d->bytes bytes, 16-byte aligned; fully overwritten
 *   bad_count_dev optional int32 counter (caller zeroes it): incremented once
 *                 per input that is not ternary; such inputs are packed as 0
 * Errors: BL_ERR_NULL, BL_ERR_LAYOUT, BL_ERR_SHAPE, BL_ERR_BUF_SMALL,
 *         BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_pack_ternary(const int8_t *w_dev, const bl_packed_desc *d, void *packed_dev,
                          int32_t *bad_count_dev, void *stream);

/* Inverse of bl_pack_ternary ("the 2-bit weights are unpacked to the original
 * values", Table 1): writes w_dev [N,K] int8.  The unused code 11 decodes to 0.
 * For tests and round trips; not on the hot path. */
bl_status bl_unpack_ternary(const void *packed_dev, const bl_packed_desc *d, int8_t *w_dev,
                            void *stream);

/*
 * Per-token absmax quantization of activations to int8 (the BitNet b1.58
 * quantizer the paper builds on).  For each row m, in fp32 with every
 * operation rounded to nearest-even on its own:
 *     amax = max_k |x[m,k]|;  inv = 127 / amax;
 *     q[m,k] = clip(round_half_even(x[m,k] * inv), -128, 127);
 *     a_scale[m] = amax / 127;   q_sum[m] = sum_k q[m,k].
 * A row whose inv is not finite (amax = 0 or below ~3.7e-37) gives q = 0,
 * a_scale = 0, q_sum = 0.  NaN/Inf inputs are undefined behaviour.
 *   x_dev       [M, ldx] fp32 or bf16 (dt), ldx >= K in elements; aligned to
 *               its element size (16-byte alignment enables vector loads)
 *   q_dev       [M, Kp] int8, Kp = bl_padded_k(K), 16-byte aligned; columns
 *               K..Kp-1 are written as 0
 *   a_scale_dev [M] fp32
 *   q_sum_dev   [M] int32, may be NULL (bl_gemv and bl_gemm need it)
 * Errors: BL_ERR_NULL, BL_ERR_DTYPE, BL_ERR_SHAPE (M < 1, K out of range,
 *         ldx < K), BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_quant_act(const void *x_dev, bl_dtype dt, int64_t M, int64_t K, int64_t ldx,
                       int8_t *q_dev, float *a_scale_dev, int32_t *q_sum_dev, void *stream);

/* One activation matrix of a grouped quantization launch: the arguments of bl_quant_act. */
typedef struct {
    const void *x_dev;
    bl_dtype    dt;
    int64_t     M, K, ldx;
    int8_t     *q_dev;
    float      *a_scale_dev;
    int32_t    *q_sum_dev;    /* may be NULL */
} bl_quant_item;

/*
 * `count` independent bl_quant_act problems (1..BL_MAX_BATCH; shapes and
 * dtypes may differ) in ONE kernel launch: e.g. the four inputs of a decoder
 * layer ahead of a grouped bl_gemv_batch, the sequence to prefer over the
 * fused launch from about 4 tokens up.  Each item is validated like a
 * bl_quant_act call; results are identical.  `items` is a host array, read
 * during the call.  Extra error: BL_ERR_COUNT.
 */
bl_status bl_quant_act_batch(const bl_quant_item *items, int32_t count, void *stream);

/*
 * Decode product, 1 <= M <= 8 tokens (Section 2, I2_S: codes are turned back
 * into weights in registers and a plain multiply-add GEMV follows):
 *     acc[m,n] = sum_k q[m,k] * W[n,k]   (int32, exact)
 *     out[m,n] = (float)acc[m,n] * (w_scale * a_scale[m])
 * Streams the packed weights exactly once, whatever M is.
 *   packed_dev  blob written by bl_pack_ternary for descriptor d
 *   q_dev, a_scale_dev, q_sum_dev   as written by bl_quant_act ([M,Kp], [M], [M])
 *   out_dev     [M,N] fp32 row-major
 *   acc_dev     optional [M,N] int32 row-major: the exact accumulators
 * Errors: BL_ERR_NULL, BL_ERR_LAYOUT, BL_ERR_SHAPE, BL_ERR_BUF_SMALL,
 *         BL_ERR_M_RANGE, BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_gemv(const void *packed_dev, const bl_packed_desc *d, const int8_t *q_dev,
                  const float *a_scale_dev, const int32_t *q_sum_dev, int64_t M,
                  float *out_dev, int32_t *acc_dev, void *stream);

/* One problem of a grouped decode launch: the arguments of bl_gemv. */
typedef struct {
    const void           *packed_dev;
    const bl_packed_desc *desc;        /* host pointer */
    const int8_t         *q_dev;
    const float          *a_scale_dev;
    const int32_t        *q_sum_dev;
    float                *out_dev;
    int32_t              *acc_dev;     /* may be NULL */
} bl_gemv_item;

/*
 * `count` independent bl_gemv problems (1..BL_MAX_BATCH, all with the same M)
 * in ONE kernel launch: e.g. the Q/K/V projections or gate/up of a decoder
 * layer (Appendix A shapes), which share their input.  Each item is
 * validated like a bl_gemv call; results are identical to `count` separate
 * calls.  `items` is a host array, read during the call.
 *
 * `workspace_dev` (may be NULL): BL_WORKSPACE_BYTES of device memory, 256-byte
 * aligned, owned by the caller, ALL ZERO before its first use.  With it, a
 * one-token launch of medium size is work-balanced: every workgroup streams
 * the same number of weight tiles, and a 64-row block whose tiles fall to two
 * or more workgroups is finished through the workspace (exact integer partial
 * sums, so results do not change by a bit).  Every launch leaves the workspace
 * all zero again, so one buffer serves any number of successive launches on a
 * stream; launches that may run at the same time (different streams) must not
 * share one, and a buffer whose launch was aborted must be zeroed again.
 * Without it, or when balancing would not pay (M > 1, tiny or very large
 * launches), whole row blocks are dealt to workgroups and nothing is shared.
 * Extra errors: BL_ERR_COUNT; BL_ERR_ALIGN for a misaligned workspace.
 */
bl_status bl_gemv_batch(const bl_gemv_item *items, int32_t count, int64_t M, void *workspace_dev,
                        void *stream);

/*
 * bl_gemv_batch for callers that cannot hand over a workspace and must not
 * allocate one: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, validation and results as
 * bl_gemv_batch(items, count, M, workspace, stream) with a workspace; the
 * workspace is a static device array inside the library, BL_STATIC_WS_BYTES
 * (512 KiB) on every GPU the library is used on, held until the process ends.
 * The call allocates and frees nothing and synchronizes nothing.
 *   - Limit: a work-balanced launch uses 64 words of scratch per workgroup; a
 *     launch planned with more than BL_STATIC_WS_WGS workgroups (possible only
 *     through bl_set_tuning("decode_split", n) on a large device) is refused
 *     with BL_ERR_WORKSPACE and nothing is launched.
 *   - The first call on a device looks up that device's copy of the array and
 *     clears it with a small kernel on `stream`; make that first call outside
 *     graph capture.  Every launch leaves the array all zero again.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in
 *     time on one GPU (different streams) race; use bl_gemv_batch with
 *     separate workspaces for those.  After an aborted launch the array may
 *     be dirty for the rest of the process.
 * Errors: those of bl_gemv_batch, and BL_ERR_WORKSPACE.
 */
bl_status bl_gemv_batch_static(const bl_gemv_item *items, int32_t count, int64_t M, void *stream);

/* One problem of the fused decode launch. */
typedef struct {
    const void           *x_dev;        /* [M, ldx] activations, fp32 or bf16                  */
    bl_dtype              dt;
    int64_t               ldx;          /* row stride of x in elements, >= K                   */
    const void           *packed_dev;
    const bl_packed_desc *desc;         /* host pointer                                        */
    float                *out_dev;      /* [M,N] fp32                                          */
    int32_t              *acc_dev;      /* optional [M,N] int32                                */
    int8_t               *q_dev;        /* optional [M,Kp]: receives the quantized activations */
    float                *a_scale_dev;  /* optional [M]                                        */
    int32_t              *q_sum_dev;    /* optional [M]                                        */
} bl_decode_item;

/*
 * Fused decode: bl_quant_act followed by bl_gemv for `count` problems
 * (1..BL_MAX_BATCH, same M in 1..8) in ONE kernel launch.  Every workgroup
 * quantizes its token rows into on-chip memory while its first weight tiles
 * are already in flight, so the int8 activations never travel through HBM
 * and the separate quantization launch disappears.  Results (q, a_scale,
 * q_sum, acc, out) are bit-identical to the two-call sequence.
 * All items of one launch must have the same activation dtype (else
 * BL_ERR_DTYPE).  `workspace_dev`: as for bl_gemv_batch (may be NULL).
 * Limit: M * Kp (+ 5 KiB per token) must fit the kernel's 128 KiB of
 * on-chip memory, else BL_ERR_SHAPE; use the two-call sequence then.
 * From two tokens up there are two forms.  With a workspace AND q_dev, a_scale_dev,
 * q_sum_dev given for every item (vector-loadable rows: K and ldx multiples of 8,
 * x_dev 16-byte aligned), every DISTINCT input -- items that name the same x_dev,
 * ldx, K and the same three buffers -- is quantized once, by the launch's leading
 * workgroups, one token row each, and published through those buffers; the other
 * workgroups request their first weight tiles and then wait, a bounded number of
 * polls, for their input's rows.  A workgroup whose polls run out goes on with
 * whatever the buffers hold, so that every kernel ends, and sets the 32-bit word
 * 256 bytes before the workspace's end to 1: results of such a launch are
 * garbage and the workspace must be zeroed again (it never happened in testing
 * other than forced through bl_set_tuning("decode_wait_limit", 1)).  Otherwise
 * every workgroup quantizes all M rows for itself, which is bound by the vector
 * ALU.  Measured on MI355X (7B-shape layer, 7 products on 4 inputs): M = 4 / 8:
 * publishing 17.5 / 18.2 us, every workgroup for itself 17.7 / 27.6 us,
 * bl_quant_act_batch + bl_gemv_batch 16.8 / 16.7 us -- the hand-over between
 * workgroups (device-scope stores, their acknowledgement, the counter, the poll,
 * the re-read) costs about what a kernel boundary costs, so the two-call sequence
 * stays the one to prefer from about 4 tokens up.
 * Pointer alignment as for bl_quant_act / bl_gemv.
 * Errors: BL_ERR_NULL, BL_ERR_COUNT, BL_ERR_M_RANGE, BL_ERR_DTYPE,
 *         BL_ERR_LAYOUT, BL_ERR_SHAPE, BL_ERR_BUF_SMALL, BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_decode_batch(const bl_decode_item *items, int32_t count, int64_t M, void *workspace_dev,
                          void *stream);

/*
 * Prefill product, 1 <= M <= BL_MAX_GEMM_M: the same mathematics as bl_gemv,
 * computed as a dense contraction on the int8 matrix cores.  Arguments as
 * for bl_gemv (M outside the range: BL_ERR_SHAPE).
 */
bl_status bl_gemm(const void *packed_dev, const bl_packed_desc *d, const int8_t *q_dev,
                  const float *a_scale_dev, const int32_t *q_sum_dev, int64_t M,
                  float *out_dev, int32_t *acc_dev, void *stream);

/*
 * `count` independent bl_gemm problems (1..BL_MAX_GEMM_BATCH, all over the same
 * M) in ONE kernel launch: e.g. the Q/K/V projections or gate/up of a decoder
 * layer over a prompt of a few hundred tokens, where one product alone gives
 * every compute unit a single workgroup.  Items are validated like bl_gemm
 * calls; results are identical to `count` separate
 * calls.  `items` is a host array, read during the call.
 * Errors: those of bl_gemm, and BL_ERR_COUNT.
 */
bl_status bl_gemm_batch(const bl_gemv_item *items, int32_t count, int64_t M, void *stream);

/* ---- A 1.78-bit layout on the paper's TL2 code --------------------------
 *
 * Section 2 and Table 3: three ternary weights become one sign bit and a
 * 4-bit index (index = |9 w0 + 3 w1 + w2|, sign = 1 iff that sum is negative),
 * five bits for three weights.  Layout version 2 stores six such codes in a
 * 32-bit word (18 weights, two bits unused: 1.78 bits per weight), in tiles of
 * 64 rows x 72 k = 1 KiB: tile (rb, kc) at byte ((rb * Kp/72) + kc) * 1024; the
 * 16 bytes at offset 16 r of a tile are row 64 rb + r; word s of those four
 * holds the weights k = 72 kc + 18 s + 3 i + {0,1,2} as code i = sign << 4 |
 * index at bits [5 i, 5 i + 4].  Padding weights are 0.  The decode product
 * reads 11 % fewer bytes than with the 2-bit layout and spends about twice the
 * vector instructions per weight (measured: a tie on 100B-shape layers, slower
 * on smaller ones); one token only, no fused quantization.
 */
#define BL_TL2_TILE_K 72
#define BL_TL2_LAYOUT_VERSION 2

/* K rounded up to BL_TL2_TILE_K; -1 if K is outside 1..BL_MAX_K. */
int64_t bl_tl2_padded_k(int64_t K);

/* Descriptor of a version-2 blob: version = BL_TL2_LAYOUT_VERSION, Kp =
 * bl_tl2_padded_k(K), bytes = Np * Kp / 72 * 16.  Errors as bl_packed_desc_init. */
bl_status bl_tl2_desc_init(int64_t N, int64_t K, float w_scale, bl_packed_desc *d);

/* Offline transformation into the version-2 layout and its inverse; arguments
 * and errors as for bl_pack_ternary / bl_unpack_ternary (BL_ERR_LAYOUT if the
 * descriptor is not version 2).  Codes that Table 3 does not use decode to 0. */
bl_status bl_tl2_pack(const int8_t *w_dev, const bl_packed_desc *d, void *packed_dev,
                      int32_t *bad_count_dev, void *stream);
bl_status bl_tl2_unpack(const void *packed_dev, const bl_packed_desc *d, int8_t *w_dev,
                        void *stream);

/*
 * Decode product for ONE token over a version-2 blob:
 *   out[n] = (sum_k q[k] * W[n,k]) * w_scale * a_scale[0]
 *   q_dev       the token's int8 activations as bl_quant_act writes them, in a
 *               buffer of at least bl_tl2_padded_k(K) bytes, 16-byte aligned:
 *               the bytes from K on are read and meet zero weights, so their
 *               values do not matter
 *   a_scale_dev [1] fp32
 *   out_dev     [N] fp32;  acc_dev optional [N] int32 (the exact sums)
 * Results are identical to bl_gemv on the same weights.
 * Errors: BL_ERR_NULL, BL_ERR_LAYOUT, BL_ERR_SHAPE, BL_ERR_BUF_SMALL,
 *         BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_tl2_gemv(const void *packed_dev, const bl_packed_desc *d, const int8_t *q_dev,
                      const float *a_scale_dev, float *out_dev, int32_t *acc_dev, void *stream);

/*
 * `count` bl_tl2_gemv problems (1..BL_MAX_BATCH) in ONE kernel launch, e.g. the
 * seven projections of a decoder layer.  Items are bl_gemv_item with version-2
 * descriptors; q_sum_dev is not used and may be NULL (the table yields signed
 * weights).  `workspace_dev`: as for bl_gemv_batch (may be NULL): with it,
 * launches are work-balanced across workgroups.  Each item is
 * validated like a bl_tl2_gemv call; results are identical.
 * Errors: BL_ERR_NULL, BL_ERR_COUNT, BL_ERR_LAYOUT, BL_ERR_SHAPE,
 *         BL_ERR_BUF_SMALL, BL_ERR_ALIGN, BL_ERR_HIP.
 */
bl_status bl_tl2_gemv_batch(const bl_gemv_item *items, int32_t count, void *workspace_dev,
                            void *stream);

/*
 * Launch-shape override for experiments and sweeps; process-wide, not thread-safe; the integer
 * and fp32 results of the products never change.  Keys: "gemv_waves" = waves of the decode kernel that share one
 * 64-row block (1, 2, 4, 8, 16; 0 = automatic); "decode_split" = work-balanced one-token launches: -1 never,
 * 0 automatic (by launch size; never for the gated launch of bl_decode_norm_batch), n = 1..8 always with n workgroups per
 * compute unit when a workspace is given and the launch has at least 8 tiles per workgroup; "decode_path" = 0 automatic
 * (dot-product kernel for M = 1, matrix-core kernel for M >= 2), 1 = always the
 * dot-product kernel, 2 = always the matrix-core kernel; "decode_stage" = 1 keeps the matrix-core kernel
 * from staging the quantized activations in on-chip memory (0 = stage when they fit); "gemm_mb" = tile form of the prefill kernel as
 * 100*(WK-1) + 10*MB + H: wave tile (32*MB) tokens x (32*H) weight rows, WK of the workgroup's four waves along K and the rest
 * along N.  Forms: 12, 14, 22, 23, 24, 122, 124 (0 = automatic);
 * "decode_publish" = fused launches of 2..8 tokens: 0 = quantize every distinct input once and publish it when the call allows it (see
 * bl_decode_batch), -1 = never; "decode_wait_limit" = polls before a waiting workgroup of that form gives up (0 = the default, 262144);
 * "decode_stream" = how the decode kernels load weight tiles: 0 automatic (streaming, i.e. nontemporal, loads for launches of
 * 4 MiB of packed weights and more; ordinary loads below, so that a small model may stay in the memory-side cache), 1 always streaming, -1 never;
 * "attn_groups" = workgroups per head of bl_attn_decode (0 = automatic, else 1..65535, capped at the cache's chunks) -- the one
 * key that moves results, within that call's tolerance: it decides which chunks are folded together before the merge.
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE (unknown key/value).
 */
bl_status bl_set_tuning(const char *key, int32_t value);

/* Host-side counters for tests and tools.  Keys: "split_launches" = decode launches so far
 * that took the work-balanced form.  Unknown key or NULL: -1. */
int64_t bl_get_stat(const char *key);

/* Static, never-NULL description of a status code. */
const char *bl_status_str(bl_status s);

/* Text of the HIP error behind the calling thread's most recent BL_ERR_HIP ("no error" if
 * the thread's last launch succeeded).  Static string owned by the HIP runtime. */
const char *bl_last_hip_error(void);

/* Which kernel the calling thread's most recent decode or prefill product call launched: the
 * template instance and the grid, e.g. "decode_kernel<1, 1, 1, 1, 0, 0> grid=2112" (the name rocprofv3 shows
 * for it).  "" before the first such call.  Points into thread-local storage, valid until the
 * thread's next call of this function.  For tools that label what they time. */
const char *bl_last_kernel(void);

/* Library version string (static). */
const char *bl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BITLINEAR_H */
