"""One token through decoder layers without leaving the GPU: argument marshalling for
include/bitlinear_decoder.h plus the launch sequence of a layer.

Every arithmetic step runs in the library's kernels; this module owns buffers (torch tensors) and
the order of the launches:

    decode_norm_batch(q, k, v)    h' = h + delta of the previous layer; the three products of rmsnorm(h', g_in)
    attn_decode                   rotary embedding, cache append, attention
    decode_norm_batch(o)          the product of rmsnorm(attention output, g_attn)
    decode_norm_batch(gate_up)    h'' = h' + o; gate and up (interleaved in one matrix) of rmsnorm(h'', g_post); the
                                  epilogue leaves z = silu(gate) * up * g_ffn and the pieces of sum((silu(gate) * up)^2)
    decode_norm_batch(down)       the product of z quantized as it is, the norm's scalar from the pieces
                                  -> delta for the next layer

(5 launches.  A feed-forward row over 16384 elements is quantized by bl_norm_quant from the same pieces, in front of a
plain bl_gemv_batch: 6.  Layers whose gate and up matrices are packed separately run bl_norm_quant on silu(gate) * up
instead: 6; hidden sizes that the folded form does not take go through bl_norm_quant + bl_gemv_batch throughout: 9.)

Shapes follow Appendix A of arXiv 2410.16144 (hidden size, intermediate size, layers, heads); the block
itself is the LLaMA-like one of BitNet b1.58, which the paper does not spell out.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional

import torch

from . import binding as B
from . import ops

EPS = 1e-5
ROPE_THETA = 10000.0


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def norm_quant(mode: int, gamma: Optional[torch.Tensor], eps: float = EPS, a: Optional[torch.Tensor] = None,
               b: Optional[torch.Tensor] = None, h: Optional[torch.Tensor] = None, out: Optional[ops.QuantAct] = None,
               y: Optional[torch.Tensor] = None, quantize: bool = True, scratch: Optional[torch.Tensor] = None,
               pieces: int = 0):
    """bl_norm_quant on [M,K] fp32 tensors.  Returns the QuantAct (None if quantize is False).  scratch: a uint8
    tensor of M * BL_NORM_SCRATCH_BYTES bytes lets long rows spread over several workgroups."""
    ref = h if mode == B.BL_NORM_RESIDUAL else a
    M, K = ref.shape
    for t in (a, b, h, y):
        assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.shape == (M, K) and t.is_contiguous())
    if mode == B.BL_NORM_PREMULTIPLIED:   # scratch: `pieces` pairs from a gated launch and the 8-byte word behind them
        assert gamma is None and scratch.numel() * scratch.element_size() >= 8 * pieces + 8
    else:
        assert gamma.dtype == torch.float32 and gamma.shape == (K,) and gamma.is_contiguous()
        assert scratch is None or scratch.numel() * scratch.element_size() >= M * B.BL_NORM_SCRATCH_BYTES
    if quantize and out is None:
        out = ops.alloc_quant(M, K, ref.device)
    ptr = lambda t: t.data_ptr() if t is not None else 0
    args = B.make_norm_quant_args(
        mode, M, K, ptr(gamma), eps, a_dev=ptr(a), b_dev=ptr(b), h_dev=ptr(h),
        q_dev=out.q.data_ptr() if quantize else 0, a_scale_dev=out.a_scale.data_ptr() if quantize else 0,
        q_sum_dev=out.q_sum.data_ptr() if quantize else 0, Kp=int(out.q.shape[1]) if quantize else 0, y_dev=ptr(y),
        scratch_dev=ptr(scratch), pieces=pieces)
    B.bl_norm_quant(args, _stream())
    return out if quantize else None


def rope_table(head_dim: int, max_pos: int, device, theta: float = ROPE_THETA) -> torch.Tensor:
    """[max_pos, head_dim/2, 2] fp32 (cos, sin) table (bl_rope_table)."""
    t = torch.empty((max_pos, head_dim // 2, 2), dtype=torch.float32, device=device)
    B.bl_rope_table(t.data_ptr(), head_dim, max_pos, theta, _stream())
    return t


class Attention:
    """Key/value cache of one layer plus a prepared bl_attn_decode call."""

    def __init__(self, n_heads: int, head_dim: int, max_pos: int, q_lin, k_lin, v_lin, pos: torch.Tensor,
                 table: torch.Tensor, out: Optional[torch.Tensor] = None):
        dev = q_lin.device
        hidden = n_heads * head_dim
        self.n_heads, self.head_dim, self.max_pos = n_heads, head_dim, max_pos
        self.k_cache = torch.zeros((max_pos, hidden), dtype=torch.bfloat16, device=dev)
        self.v_cache = torch.zeros((max_pos, hidden), dtype=torch.bfloat16, device=dev)
        self.scratch = torch.zeros(B.bl_attn_scratch_bytes(n_heads, head_dim, max_pos), dtype=torch.uint8, device=dev)
        self.out = out if out is not None else torch.empty((1, hidden), dtype=torch.float32, device=dev)
        for t in (q_lin, k_lin, v_lin, self.out):
            assert t.dtype == torch.float32 and t.numel() == hidden and t.is_contiguous()
        assert pos.dtype == torch.int32 and pos.numel() == 1 and table.shape == (max_pos, head_dim // 2, 2)
        self._keep = (q_lin, k_lin, v_lin, pos, table)
        self.args = B.make_attn_args(q_lin.data_ptr(), k_lin.data_ptr(), v_lin.data_ptr(), pos.data_ptr(), table.data_ptr(),
                                     self.k_cache.data_ptr(), self.v_cache.data_ptr(), self.out.data_ptr(),
                                     self.scratch.data_ptr(), n_heads, head_dim, max_pos)

    def launch(self):
        B.bl_attn_decode(self.args, _stream())
        return self.out


class NormDecodeGroup:
    """A prepared bl_decode_norm_batch launch: RMSNorm (with an optional residual add) folded into the quantizer of
    the products that consume the normalised row.  weights share x / delta / gamma; h_out receives x + delta.

    pieces (with gamma None): x is already multiplied by its norm weight and `pieces` holds sum(x^2) in parts (what a
    gated launch leaves behind: its .pieces tensor).  glu=(w_scale_up, glu_gamma): the one weight is gate and up
    interleaved (pack_gate_up); the launch writes silu(gate) * up * glu_gamma to outs[0] ([1, F]) and per 32 outputs
    the pair (sum((silu(gate) * up)^2), max|out|) to self.pieces ([F / 32 + 1, 2]; the last row stays zero)."""

    def __init__(self, weights, x: torch.Tensor, gamma: Optional[torch.Tensor], eps: float = EPS,
                 delta: Optional[torch.Tensor] = None, h_out: Optional[torch.Tensor] = None, want_acc: bool = False,
                 want_quant: bool = False, use_workspace=True, pieces: Optional[torch.Tensor] = None, glu=None):
        assert 1 <= len(weights) <= B.BL_MAX_BATCH
        dev = x.device
        K = weights[0].K
        for t in (x, delta, h_out, gamma):
            assert t is None or (t.dtype == torch.float32 and t.numel() == K and t.is_contiguous())
        assert all(w.K == K for w in weights) and (gamma is None) != (pieces is None)
        self.workspace_ptr = ops._workspace_ptr(use_workspace, dev)
        if glu is not None:
            assert len(weights) == 1 and weights[0].N % 64 == 0
            w_scale_up, glu_gamma = glu
            F = weights[0].N // 2
            assert glu_gamma.dtype == torch.float32 and glu_gamma.numel() == F and glu_gamma.is_contiguous()
            self.outs = [torch.empty((1, F), dtype=torch.float32, device=dev)]
            # F / 32 pairs (sum of squares, absmax), then the zero word a long row's quantizer wants behind them
            self.pieces = torch.zeros((F // 32 + 1, 2), dtype=torch.float32, device=dev)
        else:
            self.outs = [torch.empty((1, w.N), dtype=torch.float32, device=dev) for w in weights]
            self.pieces = None
        self.accs = [torch.empty((1, w.N), dtype=torch.int32, device=dev) for w in weights] if want_acc else None
        self.quants = [ops.alloc_quant(1, K, dev) for _ in weights] if want_quant else None
        self._keep = (weights, x, gamma, delta, h_out, pieces, glu)
        ptr = lambda t: t.data_ptr() if t is not None else 0
        items = []
        for i, w in enumerate(weights):
            it = dict(x=x.data_ptr(), delta=ptr(delta), h_out=ptr(h_out) if i == 0 else 0, gamma=ptr(gamma), eps=eps,
                      packed=w.blob.data_ptr(), desc=w.desc, out=self.outs[i].data_ptr(),
                      acc=self.accs[i].data_ptr() if want_acc else 0)
            if want_quant:
                it.update(q=self.quants[i].q.data_ptr(), a_scale=self.quants[i].a_scale.data_ptr(),
                          q_sum=self.quants[i].q_sum.data_ptr())
            if pieces is not None:
                it.update(ss_in=pieces.data_ptr(), ss_count=int(pieces.shape[0]) - 1)
            if glu is not None:
                it.update(w_scale_up=float(glu[0]), glu_gamma=glu[1].data_ptr(), ss_out=self.pieces.data_ptr())
            items.append(it)
        self.items = B.make_decode_norm_items(items)

    def launch(self):
        B.bl_decode_norm_batch(self.items, self.workspace_ptr, _stream())
        return self.outs


def pack_gate_up(w_gate: torch.Tensor, w_up: torch.Tensor, s_gate: float) -> ops.PackedWeight:
    """Gate and up projections ([F, K] int8 ternary each, F a multiple of 32) as ONE packed matrix of 2 F rows, interleaved
    by 32: row block b holds gate rows 32 b .. 32 b + 31, then the up rows of the same outputs -- the operand of a gated
    launch (NormDecodeGroup(glu=...)).  The descriptor carries the gate matrix's scale; the up matrix's goes with glu."""
    F, K = w_gate.shape
    assert w_up.shape == (F, K) and F % 32 == 0 and w_gate.is_contiguous() and w_up.is_contiguous()
    assert w_gate.dtype == torch.int8 and w_up.dtype == torch.int8 and w_gate.is_cuda and w_up.is_cuda
    desc = B.bl_packed_desc_init(2 * F, K, s_gate)
    blob = torch.empty(int(desc.bytes), dtype=torch.uint8, device=w_gate.device)
    B.bl_pack_gate_up(w_gate.data_ptr(), w_up.data_ptr(), desc, blob.data_ptr(), 0, _stream())
    return ops.PackedWeight(blob, desc)


def can_fold_norm(K: int) -> bool:
    return K % 8 == 0 and K <= B.BL_DECODE_NORM_MAX_K


@dataclass
class LayerWeights:
    proj: Dict[str, ops.PackedWeight]     # 'q','k','v','o','gate','up','down'; optionally 'gate_up' (pack_gate_up)
    g_in: torch.Tensor
    g_attn: torch.Tensor
    g_post: torch.Tensor
    g_ffn: torch.Tensor
    s_up: float = 0.0                     # the up matrix's scale, for 'gate_up'


class DecoderLayer:
    """Buffers and prepared launches of one layer for one token (M = 1).

    The residual stream alternates between two buffers: a launch that folds "h += delta" into its quantizer reads
    h and delta in every workgroup while one workgroup writes the sum, so the sum goes to the other buffer.
    h_in: where this layer finds the stream (delta_in, if given, still to be added); h_out: where it leaves it
    (delta_out still to be added by whoever comes next)."""

    def __init__(self, w: LayerWeights, n_heads: int, max_pos: int, h_in: torch.Tensor, h_alt: torch.Tensor,
                 delta_in: Optional[torch.Tensor], pos: torch.Tensor, table: torch.Tensor, eps: float = EPS,
                 use_workspace=True, fold_norm: Optional[bool] = None):
        dev = h_in.device
        hidden = int(h_in.shape[1])
        ffn = w.proj["down"].K
        assert h_in.shape == (1, hidden) and h_alt.shape == (1, hidden) and hidden % n_heads == 0
        self.w, self.eps, self.delta_in = w, eps, delta_in
        self.fold = can_fold_norm(hidden) if fold_norm is None else fold_norm
        self.q4 = ops.alloc_quant(1, ffn, dev)
        self.norm_scratch = torch.empty(B.BL_NORM_SCRATCH_BYTES, dtype=torch.uint8, device=dev)
        if self.fold:
            h_mid = h_alt if delta_in is not None else h_in          # the stream after "h += delta_in"
            self.h_out = h_in if h_mid is h_alt else h_alt           # ... and after "h += o"
            self.qkv = NormDecodeGroup([w.proj[n] for n in "qkv"], h_in, w.g_in, eps, delta=delta_in,
                                       h_out=h_mid if delta_in is not None else None, use_workspace=use_workspace)
            self.attn = Attention(n_heads, hidden // n_heads, max_pos, *self.qkv.outs, pos, table)
            self.o = NormDecodeGroup([w.proj["o"]], self.attn.out, w.g_attn, eps, use_workspace=use_workspace)
            # the gated form: gate and up interleaved in one matrix, silu(gate) * up * g_ffn out of the launch's epilogue,
            # and the down projection quantizes that row as it is (rows short enough to live in registers)
            self.gated = "gate_up" in w.proj
            if self.gated:
                self.gate_up = NormDecodeGroup([w.proj["gate_up"]], h_mid, w.g_post, eps, delta=self.o.outs[0],
                                               h_out=self.h_out, use_workspace=use_workspace, glu=(w.s_up, w.g_ffn))
                self.down_folded = can_fold_norm(ffn)
                if self.down_folded:
                    self.down = NormDecodeGroup([w.proj["down"]], self.gate_up.outs[0], None, eps,
                                                pieces=self.gate_up.pieces, use_workspace=use_workspace)
                else:   # a row too long for the product's quantizer: one launch of its own, from the same pieces
                    self.down = ops.GemvGroup([w.proj["down"]], [self.q4], use_workspace=use_workspace)
            else:
                self.gate_up = NormDecodeGroup([w.proj["gate"], w.proj["up"]], h_mid, w.g_post, eps, delta=self.o.outs[0],
                                               h_out=self.h_out, use_workspace=use_workspace)
        else:
            assert "gate" in w.proj, "the layer holds gate and up interleaved only: that form needs the folded norm"
            self.gated = False
            self.h, self.h_out = h_in, h_in                           # separate norm launches update the stream in place
            self.q1, self.q2, self.q3 = (ops.alloc_quant(1, hidden, dev) for _ in range(3))
            self.qkv = ops.GemvGroup([w.proj[n] for n in "qkv"], [self.q1] * 3, use_workspace=use_workspace)
            self.attn = Attention(n_heads, hidden // n_heads, max_pos, *self.qkv.outs, pos, table)
            self.o = ops.GemvGroup([w.proj["o"]], [self.q2], use_workspace=use_workspace)
            self.gate_up = ops.GemvGroup([w.proj["gate"], w.proj["up"]], [self.q3] * 2, use_workspace=use_workspace)
        if not (self.fold and self.gated):
            self.down = ops.GemvGroup([w.proj["down"]], [self.q4], use_workspace=use_workspace)
        self.delta_out = self.down.outs[0]

    def launch(self):
        w = self.w
        if self.fold:      # 5 launches with the gated form, else 6 (the gated norm on its own)
            self.qkv.launch()
            self.attn.launch()
            self.o.launch()
            self.gate_up.launch()
        else:              # 9 launches
            norm_quant(B.BL_NORM_RESIDUAL, w.g_in, self.eps, a=self.delta_in, h=self.h, out=self.q1)
            self.qkv.launch()
            self.attn.launch()
            norm_quant(B.BL_NORM_PLAIN, w.g_attn, self.eps, a=self.attn.out, out=self.q2)
            self.o.launch()
            norm_quant(B.BL_NORM_RESIDUAL, w.g_post, self.eps, a=self.o.outs[0], h=self.h, out=self.q3)
            self.gate_up.launch()
        if not self.gated:
            norm_quant(B.BL_NORM_GATED, w.g_ffn, self.eps, a=self.gate_up.outs[0], b=self.gate_up.outs[1], out=self.q4,
                       scratch=self.norm_scratch)
        elif not self.down_folded:
            norm_quant(B.BL_NORM_PREMULTIPLIED, None, self.eps, a=self.gate_up.outs[0], out=self.q4,
                       scratch=self.gate_up.pieces, pieces=int(self.gate_up.pieces.shape[0]) - 1)
        self.down.launch()
        return self.delta_out


class DecoderStack:
    """n layers, one token per step: h (the residual stream, [1, hidden] fp32) goes in, the final-normalised
    hidden state comes out; the position lives on the device and advances by one per step."""

    def __init__(self, layers: List[LayerWeights], g_final: torch.Tensor, n_heads: int, max_pos: int, device,
                 eps: float = EPS, theta: float = ROPE_THETA, use_workspace=True, fold_norm: Optional[bool] = None):
        hidden = layers[0].proj["q"].K
        self.hidden, self.n_heads, self.max_pos, self.eps = hidden, n_heads, max_pos, eps
        self.h = torch.zeros((1, hidden), dtype=torch.float32, device=device)       # the caller writes the token's input here
        self.h_alt = torch.zeros((1, hidden), dtype=torch.float32, device=device)
        self.y = torch.empty((1, hidden), dtype=torch.float32, device=device)
        self.pos = torch.zeros((1,), dtype=torch.int32, device=device)
        self.table = rope_table(hidden // n_heads, max_pos, device, theta)
        self.g_final = g_final
        self.layers: List[DecoderLayer] = []
        delta, h_in = None, self.h
        for w in layers:
            h_alt = self.h_alt if h_in is self.h else self.h
            layer = DecoderLayer(w, n_heads, max_pos, h_in, h_alt, delta, self.pos, self.table, eps, use_workspace, fold_norm)
            self.layers.append(layer)
            delta, h_in = layer.delta_out, layer.h_out
        self.h_last = h_in
        self.graph = None
        self._next_pos = 0      # host-side mirror of self.pos, to refuse a token beyond the cache

    def set_position(self, pos: int):
        """Continue at position `pos` (the caches must hold rows 0 .. pos-1)."""
        assert 0 <= pos <= self.max_pos
        self.pos.fill_(pos)
        self._next_pos = pos

    def launch(self):
        """All launches of one token on the current stream: the layers, the last residual add with the final
        norm (-> self.y), the position's increment."""
        for layer in self.layers:
            layer.launch()
        norm_quant(B.BL_NORM_RESIDUAL, self.g_final, self.eps, a=self.layers[-1].delta_out, h=self.h_last, y=self.y,
                   quantize=False)
        B.bl_pos_advance(self.pos.data_ptr(), _stream())
        return self.y

    def capture(self):
        """Capture launch() into a HIP graph (no memset nodes: every launch here is a kernel).  One token is run
        eagerly first -- kernels set their launch attributes on first use, which a capture does not allow -- and
        the residual stream and the position are put back afterwards (the cache row it wrote is rewritten by the
        first real token at that position)."""
        h0, pos0 = self.h.clone(), self.pos.clone()
        self.launch()
        torch.cuda.synchronize()
        self.h.copy_(h0)
        self.pos.copy_(pos0)   # the warm-up token does not count: _next_pos is untouched
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(s):
            with torch.cuda.graph(self.graph, stream=s):
                self.launch()
        torch.cuda.current_stream().wait_stream(s)
        return self.graph

    def prefill(self, x: torch.Tensor) -> torch.Tensor:
        """A prompt (or a piece of one): x [M, hidden] fp32, the inputs of M consecutive tokens starting at the present
        position.  Every product runs as a bl_gemm over the M rows (q, k, v in one launch, gate and up in one), the
        norms as M-row bl_norm_quant launches, the attention as bl_attn_prefill; eager launches, buffers sized to M on
        the spot.  Fills the caches, advances the
        position by M and returns the final-normalised hidden states [M, hidden].  The layers must hold gate and up
        as separate matrices (the interleaved one serves the one-token launches only)."""
        M, hidden = x.shape
        assert hidden == self.hidden and x.dtype == torch.float32 and x.is_contiguous()
        pos0 = self._next_pos
        if pos0 + M > self.max_pos:
            raise RuntimeError("the key/value cache holds %d positions: no room for %d more" % (self.max_pos, M))
        dev, d = x.device, self.hidden // self.n_heads
        H = x.clone()
        new = lambda n: torch.empty((M, n), dtype=torch.float32, device=dev)
        A, Y = new(hidden), new(hidden)
        scratch = torch.zeros(B.bl_attn_prefill_scratch_bytes(self.n_heads, d, pos0, M), dtype=torch.uint8, device=dev)
        delta = None
        for layer in self.layers:
            w = layer.w
            assert "gate" in w.proj and "up" in w.proj, "prefill needs gate and up as separate matrices"
            ffn = w.proj["down"].K
            wide = torch.empty(M * B.BL_NORM_SCRATCH_BYTES, dtype=torch.uint8, device=dev)
            q1 = norm_quant(B.BL_NORM_RESIDUAL, w.g_in, self.eps, a=delta, h=H)
            ql, kl, vl = ops.gemm_batch([w.proj[n] for n in "qkv"], q1)
            B.bl_attn_prefill(ql.data_ptr(), kl.data_ptr(), vl.data_ptr(), self.table.data_ptr(), layer.attn.k_cache.data_ptr(),
                              layer.attn.v_cache.data_ptr(), A.data_ptr(), scratch.data_ptr(), self.n_heads, d, self.max_pos,
                              pos0, M, _stream())
            o = ops.gemm(w.proj["o"], norm_quant(B.BL_NORM_PLAIN, w.g_attn, self.eps, a=A))
            q3 = norm_quant(B.BL_NORM_RESIDUAL, w.g_post, self.eps, a=o, h=H)
            gate, up = ops.gemm_batch([w.proj["gate"], w.proj["up"]], q3)
            q4 = norm_quant(B.BL_NORM_GATED, w.g_ffn, self.eps, a=gate, b=up, out=ops.alloc_quant(M, ffn, dev), scratch=wide)
            delta = ops.gemm(w.proj["down"], q4)
        norm_quant(B.BL_NORM_RESIDUAL, self.g_final, self.eps, a=delta, h=H, y=Y, quantize=False)
        self.set_position(pos0 + M)
        return Y

    def step(self):
        """One token: self.h holds its input; returns self.y.  Raises once the cache is full (the kernels themselves
        do nothing for a position outside the cache)."""
        if self._next_pos >= self.max_pos:
            raise RuntimeError("the key/value cache holds %d positions and is full" % self.max_pos)
        self._next_pos += 1
        if self.graph is not None:
            self.graph.replay()
        else:
            self.launch()
        return self.y


def make_stack(name: str, max_pos: int, device, config: int = 7, n_layers: Optional[int] = None,
               use_workspace=True, gated: bool = True) -> DecoderStack:
    """A dummy model of Appendix A's shape `name` (as in the paper: random ternary weights, drawn on the device from
    the seed rule of synth.seed_for), norm weights uniform in [0.5, 1.5]."""
    from . import synth
    hidden, ffn, layers = synth.PAPER_MODELS[name]
    n_layers = layers if n_layers is None else n_layers
    ws = []
    g = torch.Generator(device=device)
    for i in range(n_layers):
        proj = {}
        for j, p in enumerate(synth.layer_projections(hidden, ffn)):
            seed = synth.seed_for(config, i, j)
            wd = synth.ternary_weights_device(seed, p.N, p.K, device)
            proj[p.name] = ops.pack_ternary(wd, float(synth.draw_w_scale(synth.rng_for(seed))))
            del wd
        g.manual_seed(synth.seed_for(config, i, 8))
        gam = [torch.rand(k, device=device, generator=g) + 0.5 for k in (hidden, hidden, hidden, ffn)]
        s_up = 0.0
        if gated and can_fold_norm(hidden) and ffn % 32 == 0:
            # the interleaved matrix replaces the two separate ones (same weights, drawn again from their seeds)
            pj = {p.name: p for p in synth.layer_projections(hidden, ffn)}
            wg = synth.ternary_weights_device(synth.seed_for(config, i, 4), pj["gate"].N, pj["gate"].K, device)
            wu = synth.ternary_weights_device(synth.seed_for(config, i, 5), pj["up"].N, pj["up"].K, device)
            proj["gate_up"] = pack_gate_up(wg, wu, proj["gate"].desc.w_scale)
            s_up = float(proj["up"].desc.w_scale)
            del wg, wu, proj["gate"], proj["up"]
        ws.append(LayerWeights(proj, *gam, s_up=s_up))
    g.manual_seed(synth.seed_for(config, n_layers, 8))
    return DecoderStack(ws, torch.rand(hidden, device=device, generator=g) + 0.5, synth.PAPER_HEADS[name], max_pos, device,
                        use_workspace=use_workspace)
