/*
 * bitlinear_decoder.h -- the decoder block around the BitLinear products, one token at a time.
 *
 * arXiv 2410.16144 reports its speed in tokens per second of WHOLE models (Section 3, the
 * inference-speed tables) on dummy models of which Appendix A gives the shapes: hidden size,
 * intermediate size, layers and attention heads.  The seven ternary projections of a layer are
 * bitlinear.h's products; this header declares what stands between them so that a token can pass
 * through a layer without leaving the GPU.  The paper does not describe these operations; they are
 * the LLaMA-like block of BitNet b1.58 (RMSNorm, rotary position embedding, multi-head attention
 * over a key/value cache, SiLU-gated feed-forward, residuals, no biases), with one RMSNorm in front
 * of every activation quantizer:
 *
 *   y  = rmsnorm(h, g_in)           -> q, k, v = BitLinear(y)
 *   a  = attention(rope(q), cache + {rope(k), v})
 *   h += BitLinear_o(rmsnorm(a, g_attn))
 *   y  = rmsnorm(h, g_post)         -> gate, up = BitLinear(y)
 *   h += BitLinear_down(rmsnorm(silu(gate) * up, g_ffn))
 *
 * Conventions as in bitlinear.h: device pointers end in _dev, no entry point allocates, frees or
 * synchronizes, `stream` is a hipStream_t (NULL = default stream), errors are bl_status codes and
 * nothing is launched when one is returned.  All floating-point data here is fp32 except the
 * key/value cache (bf16 bit patterns).
 */
#ifndef BITLINEAR_DECODER_H
#define BITLINEAR_DECODER_H

#include "bitlinear.h"

#ifdef __cplusplus
extern "C" {
#endif

#define BL_NORM_MAX_K 49152     /* longest row bl_norm_quant takes (the paper's largest
                                   intermediate size, Appendix A "100B", is 45568)        */
#define BL_NORM_SCRATCH_BYTES 256 /* per token row, for bl_norm_quant_args.scratch_dev            */
#define BL_ATTN_MAX_HEAD_DIM 256
#define BL_ATTN_CHUNK 64        /* cache positions per workgroup of the attention kernel  */
#define BL_ATTN_BLOCK_MAX_HEAD_DIM 128 /* bl_attn_prefill: head sizes up to this go through the matrix cores */

typedef enum bl_norm_mode {
    BL_NORM_PLAIN = 0,      /* x = a                                                  */
    BL_NORM_RESIDUAL = 1,   /* x = h + a (a may be NULL: x = h); h is overwritten by x */
    BL_NORM_GATED = 2,      /* x = silu(a) * b, silu(t) = t / (1 + exp(-t))            */
    BL_NORM_PREMULTIPLIED = 3 /* a = x * gamma already, with `pieces` pairs (sum(x^2), max|a|) in
                                 scratch_dev (what a gated bl_decode_norm_batch launch leaves)
                                 FOLLOWED BY one 8-byte word that is zero before the first call
                                 (every call leaves it zero; the slices' sum(q) meet in it):
                                 y = a * r.  One token (M = 1), any K, one launch; gamma_dev unused */
} bl_norm_mode;

/*
 * One launch: for each of M token rows, form x (see bl_norm_mode), normalise
 *   y[k] = (x[k] * gamma[k]) * r,   r = 1 / sqrt(mean_k(x^2) + eps)     (two fp32 products, in this order)
 * and quantize y exactly as bl_quant_act does (per-token absmax int8):
 *   q [M, Kp] int8, a_scale [M], q_sum [M] -- ready for bl_gemv / bl_gemv_batch / bl_gemm.
 * Fusing the three keeps the row in registers: x is read once and only q leaves the chip.
 *   a_dev, b_dev, h_dev  [M, K] fp32, rows contiguous (stride K)
 *   gamma_dev            [K] fp32
 *   q_dev                [M, Kp] int8, Kp >= K a multiple of 4 (normally bl_padded_k(K) or
 *                        bl_tl2_padded_k(K)); bytes K..Kp-1 of each row are written as zero.
 *                        q_dev, a_scale_dev and q_sum_dev may ALL be NULL: then nothing is
 *                        quantized (the final norm of a model).
 *   q_sum_dev            optional
 *   y_dev                optional [M, K] fp32: the normalised values before quantization
 *   scratch_dev          optional, M * BL_NORM_SCRATCH_BYTES bytes, 8-byte aligned, contents free: with
 *                        it, rows of 16384 elements or more are cut into slices of 2048, one workgroup
 *                        each, in TWO launches (a single workgroup is bound by its compute unit on
 *                        such rows); q_sum then accumulates by integer atomics.  Same results up to
 *                        the order of the fp32 sum of squares.
 * K <= BL_NORM_MAX_K.  The sum of squares is an fp32 tree sum; y and the quantizer's decisions are
 * single IEEE operations on it, so q equals bl_quant_act of y_dev bit for bit.
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE (M < 1, K outside 1..BL_NORM_MAX_K, Kp < K or not a multiple
 *         of 4, unknown mode), BL_ERR_ALIGN (fp32 pointers 4 bytes, q_dev 4 bytes), BL_ERR_HIP.
 */
typedef struct bl_norm_quant_args {
    int32_t      mode;          /* bl_norm_mode */
    int32_t      M;
    int64_t      K;
    int64_t      Kp;
    const float *a_dev;
    const float *b_dev;         /* BL_NORM_GATED only */
    float       *h_dev;         /* BL_NORM_RESIDUAL only */
    const float *gamma_dev;
    float        eps;
    int8_t      *q_dev;
    float       *a_scale_dev;
    int32_t     *q_sum_dev;
    float       *y_dev;
    void        *scratch_dev;
    int32_t      pieces;        /* BL_NORM_PREMULTIPLIED: pairs (sum, max) at the head of scratch_dev */
} bl_norm_quant_args;

bl_status bl_norm_quant(const bl_norm_quant_args *args, void *stream);

/*
 * RMSNorm + quantizer + product in ONE launch, for one token and up to BL_MAX_BATCH matrices (e.g. Q, K, V
 * on the same normalised row): bl_decode_batch with the norm folded into its in-kernel quantizer.
 *
 *   x'  = x + delta                      (delta optional)
 *   out = BitLinear(rmsnorm(x', gamma))  = (sum_k q[k] W[n,k]) * w_scale * a_scale
 *
 * The norm's scalar r = 1 / sqrt(mean(x'^2) + eps) is positive and common to the row, so it passes through
 * the absmax quantizer: the codes are those of z = x' * gamma (q = bl_quant_act(z), bit for bit) and
 * a_scale = a_scale(z) * r.  Against quantizing y = r * z element by element, a code can differ only where
 * y sits within fp32 rounding of a tie.
 *   x_dev, delta_dev, gamma_dev   [K] fp32, 16-byte aligned; K a multiple of 8, K <= BL_DECODE_NORM_MAX_K
 *   h_out_dev   optional [K] fp32: receives x' (the updated residual stream).  Must not overlap
 *               x_dev or delta_dev: other workgroups still read those.  Give it to one item of
 *               a launch whose items share x_dev.
 *   packed_dev, desc, out_dev [N], acc_dev (optional), q_dev [Kp] / a_scale_dev [1] / q_sum_dev [1]
 *               (optional copies of the quantizer's results): as in bl_decode_item with M = 1
 *   workspace_dev: as for bl_gemv_batch (may be NULL)
 *
 * Two further forms, for the feed-forward half of the block (all items of a launch take the same forms):
 *
 *   Gated epilogue (glu_gamma_dev != NULL).  The packed matrix holds the GATE and UP projections interleaved by
 *   32 rows: rows 64 b .. 64 b + 31 are gate rows 32 b .. 32 b + 31, rows 64 b + 32 .. 64 b + 63 the up rows of
 *   the same 32 outputs (N = 2 F, F a multiple of 32; desc->w_scale is the gate matrix's scale, w_scale_up the up
 *   matrix's).  Instead of the 2 F products the launch writes
 *       out[n]    = silu(gate[n]) * up[n] * glu_gamma[n],   n < F      (out_dev: F floats)
 *       ss_out[b] = (sum over n in [32 b, 32 b + 32) of (silu(gate[n]) * up[n])^2, max over them of |out[n]|)
 *                                                             (ss_out_dev: F / 32 pairs of floats, 8-byte aligned)
 *   i.e. the feed-forward product already multiplied by the weight of the norm that follows it, and that norm's
 *   sum of squares (and the row's absmax) in pieces.  acc_dev, if given, still receives the 2 F raw sums.
 *
 *   Pre-multiplied row (gamma_dev == NULL, ss_in_dev != NULL): x_dev is such an `out`, ss_in_dev [ss_count] such
 *   pairs: the row is quantized as it is and r = 1 / sqrt(sum of the pieces' sums / K + eps) multiplies the
 *   scale.  delta_dev and h_out_dev must be NULL.  (A row too long for this entry point takes the same pieces
 *   through bl_norm_quant, mode BL_NORM_PREMULTIPLIED, and bl_gemv_batch.)
 *
 * Errors: BL_ERR_NULL, BL_ERR_COUNT, BL_ERR_LAYOUT, BL_ERR_SHAPE (also K not a multiple of 8 or beyond
 *         BL_DECODE_NORM_MAX_K, h_out_dev equal to x_dev or delta_dev, items of different forms, N not a multiple
 *         of 64 with the gated epilogue, ss_count < 1), BL_ERR_BUF_SMALL, BL_ERR_ALIGN, BL_ERR_HIP.
 */
#define BL_DECODE_NORM_MAX_K 16384

typedef struct bl_decode_norm_item {
    const float          *x_dev;
    const float          *delta_dev;
    float                *h_out_dev;
    const float          *gamma_dev;
    float                 eps;
    const void           *packed_dev;
    const bl_packed_desc *desc;
    float                *out_dev;
    int32_t              *acc_dev;
    int8_t               *q_dev;
    float                *a_scale_dev;
    int32_t              *q_sum_dev;
    const float          *ss_in_dev;       /* pre-multiplied row */
    int32_t               ss_count;
    float                 w_scale_up;      /* gated epilogue */
    const float          *glu_gamma_dev;
    float                *ss_out_dev;
} bl_decode_norm_item;

bl_status bl_decode_norm_batch(const bl_decode_norm_item *items, int32_t count, void *workspace_dev,
                               void *stream);

/*
 * The operand of the gated epilogue from its two matrices: gate and up ([F, K] int8 ternary each, row-major, F a
 * multiple of 32) go into ONE packed matrix of N = 2 F rows, interleaved by 32 -- packed row block b holds gate rows
 * 32 b .. 32 b + 31 in its rows 0-31 and up rows 32 b .. 32 b + 31 in its rows 32-63 (Section 2's offline weight
 * transformation, Table 1's codes, in the tiled layout of bl_pack_ternary).
 *   d           descriptor from bl_packed_desc_init(2 F, K, w_scale of the GATE matrix); the up matrix's scale is
 *               passed to the launch (bl_decode_norm_item.w_scale_up)
 *   packed_dev, bad_count_dev, stream   as for bl_pack_ternary
 * Errors: those of bl_pack_ternary; BL_ERR_SHAPE if d->N is not a multiple of 64.
 */
bl_status bl_pack_gate_up(const int8_t *gate_dev, const int8_t *up_dev, const bl_packed_desc *d, void *packed_dev,
                          int32_t *bad_count_dev, void *stream);

/*
 * Rotary table for bl_attn_decode, computed on the GPU in fp64 and rounded to fp32:
 *   table[(p * head_dim/2 + i) * 2 + {0, 1}] = {cos, sin}(p * theta^(-2 i / head_dim)),
 *   p = 0 .. max_pos-1, i = 0 .. head_dim/2 - 1.   table_dev: max_pos * head_dim floats.
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE (head_dim odd or outside 2..BL_ATTN_MAX_HEAD_DIM, max_pos < 1,
 *         theta <= 0), BL_ERR_ALIGN (8 bytes), BL_ERR_HIP.
 */
bl_status bl_rope_table(float *table_dev, int32_t head_dim, int32_t max_pos, double theta, void *stream);

/*
 * Attention for the ONE token at position p = *pos_dev (read on the device, so a captured graph can
 * be replayed as the position advances; 0 <= p < max_pos is the caller's responsibility -- a value
 * outside that range makes the launch do nothing).
 *   1. rotate the token's query and key (pairs (i, i + head_dim/2) within a head, angle from the
 *      table's row p), round key and value to bf16 and store them as row p of the caches;
 *   2. per head: weights softmax_j(q . k_j / sqrt(head_dim)) over cache rows j = 0 .. p, output
 *      sum_j weight_j * v_j.
 *   q_lin_dev, k_lin_dev, v_lin_dev   [n_heads * head_dim] fp32: the token's Q, K, V projections
 *   k_cache_dev, v_cache_dev          [max_pos, n_heads * head_dim] bf16 bit patterns, 16-byte aligned
 *   out_dev                           [n_heads * head_dim] fp32
 *   scratch_dev                       bl_attn_scratch_bytes(...) bytes, 16-byte aligned, ZERO-FILLED before
 *                                     the first call; every call leaves it usable for the next (it holds
 *                                     the partial results of the workgroups that share a head and one
 *                                     ticket counter per head, which the call puts back to zero).  Calls
 *                                     that may overlap in time must not share it.
 * One launch: n_heads x G workgroups, G = min(ceil(max_pos / BL_ATTN_CHUNK), ceil(1024 / n_heads), 32); a head's
 * workgroup y walks the chunks y, y + G, ... of BL_ATTN_CHUNK cache rows up to row p (one chunk each while
 * p < 64 G; workgroups with nothing to walk exit at once) and keeps one running maximum, sum and weighted
 * values; the workgroup of a head that finishes last merges the head's partial results -- it is told so by
 * the ticket it draws; no workgroup waits for another.
 * head_dim must be a multiple of 4 (4 .. BL_ATTN_MAX_HEAD_DIM).
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE, BL_ERR_ALIGN, BL_ERR_HIP.
 */
typedef struct bl_attn_args {
    const float   *q_lin_dev;
    const float   *k_lin_dev;
    const float   *v_lin_dev;
    const int32_t *pos_dev;
    const float   *rope_table_dev;
    uint16_t      *k_cache_dev;
    uint16_t      *v_cache_dev;
    float         *out_dev;
    void          *scratch_dev;
    int32_t        n_heads;
    int32_t        head_dim;
    int32_t        max_pos;
} bl_attn_args;

/* Bytes of bl_attn_args.scratch_dev; 0 if a shape is out of range. */
uint64_t bl_attn_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t max_pos);

bl_status bl_attn_decode(const bl_attn_args *args, void *stream);

/*
 * Attention for M consecutive tokens at positions pos0 .. pos0 + M - 1 (a prompt, or a piece of one): token m attends
 * to cache rows 0 .. pos0 + m.  Two launches: the M keys (rotated) and values go into the cache, rounded to bf16 as
 * bl_attn_decode rounds them (the same bits); then the attention.  Head sizes up to BL_ATTN_BLOCK_MAX_HEAD_DIM take one
 * workgroup per (head, 64 tokens) that forms scores and weighted values on the matrix cores, with the fp32 queries
 * entered as the sum of three bf16 numbers (all 24 bits) and the softmax weights, which lie in [0, 1], as the sum of
 * two (relative error below 2^-17), fp32 accumulation: the outputs agree with M bl_attn_decode calls to about 1e-5 of the output's scale, not bit for bit.
 * Larger head sizes take one bl_attn_decode-style workgroup per (head, 64 cache rows, token), and there the results
 * are those of M bl_attn_decode calls in order.
 *   q_lin_dev, k_lin_dev, v_lin_dev   [M, n_heads * head_dim] fp32, rows contiguous; k_lin_dev and v_lin_dev 8-byte aligned
 *   out_dev                           [M, n_heads * head_dim] fp32
 *   pos0, M                           host values; 0 <= pos0, pos0 + M <= max_pos, 1 <= M <= 65535
 *   scratch_dev                       bl_attn_prefill_scratch_bytes(...) bytes, 16-byte aligned, zero-filled before
 *                                     the first call (every call leaves its counters zero); 16 bytes that are not
 *                                     touched for head sizes up to BL_ATTN_BLOCK_MAX_HEAD_DIM
 *   rope_table_dev, k_cache_dev, v_cache_dev, n_heads, head_dim, max_pos: as in bl_attn_args
 * Errors: BL_ERR_NULL, BL_ERR_SHAPE, BL_ERR_ALIGN, BL_ERR_HIP.
 */
typedef struct bl_attn_prefill_args {
    const float *q_lin_dev;
    const float *k_lin_dev;
    const float *v_lin_dev;
    const float *rope_table_dev;
    uint16_t    *k_cache_dev;
    uint16_t    *v_cache_dev;
    float       *out_dev;
    void        *scratch_dev;
    int32_t      n_heads;
    int32_t      head_dim;
    int32_t      max_pos;
    int32_t      pos0;
    int32_t      M;
} bl_attn_prefill_args;

/* Bytes of bl_attn_prefill_args.scratch_dev for tokens pos0 .. pos0 + M - 1; 0 if a shape is out of range. */
uint64_t bl_attn_prefill_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t pos0, int32_t M);

bl_status bl_attn_prefill(const bl_attn_prefill_args *args, void *stream);

/* *pos_dev += 1 on the device (one thread), so that the token loop's position lives in the
 * graph's own memory.  Errors: BL_ERR_NULL, BL_ERR_ALIGN, BL_ERR_HIP. */
bl_status bl_pos_advance(int32_t *pos_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BITLINEAR_DECODER_H */
