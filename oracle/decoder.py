"""Plain CPU definition of the decoder layer around the BitLinear products (numpy, fp64).

TEST INFRASTRUCTURE, like the rest of this package: used by the test-suite only; it never imports
the GPU package and the GPU package never imports it.

What it covers.  arXiv 2410.16144 reports whole-model token rates (Section 3) on dummy models whose
shapes Appendix A lists (hidden size, intermediate size, layers, attention heads) and says nothing
else about the block around the ternary products.  The functions below write out the block BitNet
b1.58 describes as LLaMA-like -- RMSNorm, rotary position embedding, multi-head attention over a
key/value cache, a SiLU-gated feed-forward network, residual connections, no biases -- with one
normalisation in front of every activation quantizer (input, attention output, post-attention,
feed-forward product).  Each function is the textbook formula in fp64; the readings that the paper
leaves open (epsilon, rotary base and pairing, cache precision) are arguments or are stated where
they are taken.

Every function here is pinned by tests/test_decoder_oracle_pins.py against closed forms, invariants
and torch's own library routines.
"""
import numpy as np

from . import dequant, matmul_i32, quant_act


def rmsnorm(x, gamma, eps):
    """y[k] = x[k] / sqrt(mean_k(x^2) + eps) * gamma[k], over the last axis."""
    x = np.asarray(x, np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, np.float64)


def silu(x):
    """x * sigmoid(x)."""
    x = np.asarray(x, np.float64)
    return x / (1.0 + np.exp(-x))


def gated_ffn_input(gate, up):
    """The feed-forward product that the down projection consumes: silu(gate) * up."""
    return silu(gate) * np.asarray(up, np.float64)


def rope_angles(head_dim, n_pos, theta=10000.0):
    """angle[p, i] = p * theta^(-2 i / head_dim), i = 0 .. head_dim/2 - 1."""
    assert head_dim % 2 == 0
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    return np.arange(n_pos, dtype=np.float64)[:, None] * inv_freq[None, :]


def rope(v, pos, n_heads, theta=10000.0):
    """Rotary embedding of one token's vector [n_heads * head_dim] at position pos.

    Pairing (a reading: the split-half convention): within a head, element i pairs with element
    i + head_dim/2; the pair (a, b) becomes (a cos - b sin, a sin + b cos) with angle[pos, i]."""
    v = np.asarray(v, np.float64)
    d = v.shape[-1] // n_heads
    ang = rope_angles(d, pos + 1, theta)[pos]
    c, s = np.cos(ang), np.sin(ang)
    heads = v.reshape(n_heads, 2, d // 2)
    a, b = heads[:, 0, :], heads[:, 1, :]
    out = np.stack([a * c - b * s, a * s + b * c], axis=1)
    return out.reshape(-1)


def attention_decode(q, k_cache, v_cache, n_heads):
    """One query token against n_ctx cached tokens, per head:
    out_h = softmax_j(q_h . k_{j,h} / sqrt(head_dim)) @ v_{.,h}.
    q [hidden]; k_cache, v_cache [n_ctx, hidden]."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k_cache, np.float64)
    v = np.asarray(v_cache, np.float64)
    n_ctx, hidden = k.shape
    d = hidden // n_heads
    out = np.empty(hidden, np.float64)
    for h in range(n_heads):
        sl = slice(h * d, (h + 1) * d)
        s = k[:, sl] @ q[sl] / np.sqrt(float(d))
        p = np.exp(s - s.max())
        p /= p.sum()
        out[sl] = p @ v[:, sl]
    return out


def round_to_bf16(x):
    """Nearest bf16 (ties to even) of each value, returned as float64.  Finite inputs."""
    f = np.asarray(x, np.float64).astype(np.float32)     # fp64 -> fp32 nearest-even
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def bitlinear_f32(y, w, w_scale):
    """The BitLinear product of the fp32 rounding of y: quantize (per-token absmax int8), exact
    integer product, dequantize.  y [K] -> out [N] (fp32 values)."""
    q, a_scale, _ = quant_act(np.asarray(y, np.float64).astype(np.float32)[None, :])
    acc = matmul_i32(q, w)
    return dequant(acc, np.float32(w_scale), a_scale)[0]


def decoder_layer_step(h, pos, layer, k_cache, v_cache, n_heads, eps=1e-5, theta=10000.0):
    """One token through one decoder layer.

    h [hidden] fp64: the residual stream; pos: the token's position (the caches hold positions
    0 .. pos-1 in rows 0 .. pos-1 and receive row pos); layer: dict with ternary matrices
    'q','k','v','o','gate','up','down' (int8 [N,K]), their scales 's_q' ..., and the four norm weights
    'g_in', 'g_attn', 'g_post', 'g_ffn'.  Keys and values are stored in bf16 (a reading; llama.cpp
    keeps a 16-bit cache).  Returns the new residual stream; k_cache/v_cache rows pos are written."""
    y = rmsnorm(h, layer["g_in"], eps)
    ql = bitlinear_f32(y, layer["q"], layer["s_q"])
    kl = bitlinear_f32(y, layer["k"], layer["s_k"])
    vl = bitlinear_f32(y, layer["v"], layer["s_v"])
    qr = rope(ql, pos, n_heads, theta)
    k_cache[pos] = round_to_bf16(rope(kl, pos, n_heads, theta))
    v_cache[pos] = round_to_bf16(vl)
    a = attention_decode(qr, k_cache[:pos + 1], v_cache[:pos + 1], n_heads)
    h = h + bitlinear_f32(rmsnorm(a, layer["g_attn"], eps), layer["o"], layer["s_o"])
    y = rmsnorm(h, layer["g_post"], eps)
    gate = bitlinear_f32(y, layer["gate"], layer["s_gate"])
    up = bitlinear_f32(y, layer["up"], layer["s_up"])
    f = rmsnorm(gated_ffn_input(gate, up), layer["g_ffn"], eps)
    return h + bitlinear_f32(f, layer["down"], layer["s_down"])
