"""Device-resident synthetic decoder layers for benchmarks and full-size parity tests.

A layer is the 7 BitLinear projections of Appendix A's model structure (Q, K, V, O, gate, up,
down) with their four distinct inputs: the attention input (shared by Q/K/V), the O input, the
MLP input (shared by gate/up) and the down input.  Everything here is buffer management and
calls into the C ABI; no arithmetic.
"""
from typing import List, Optional

import numpy as np
import torch

from . import binding as B
from . import ops, synth

# which of the four inputs each projection reads
INPUT_OF = {"q": 0, "k": 0, "v": 0, "o": 1, "gate": 2, "up": 2, "down": 3}


class DecodeLayer:
    """One layer's packed weights plus preallocated activations, quantized activations and outputs."""

    def __init__(self, hidden: int, ffn: int, M: int, device, weights: List[ops.PackedWeight],
                 xs: List[torch.Tensor]):
        self.hidden, self.ffn, self.M, self.device = hidden, ffn, M, device
        self.projs = synth.layer_projections(hidden, ffn)
        self.weights = weights
        self.xs = xs                                    # 4 inputs: [M,hidden] x3, [M,ffn]
        self.qas = [ops.alloc_quant(M, int(x.shape[1]), device) for x in xs]
        self.outs = [torch.empty((M, p.N), dtype=torch.float32, device=device) for p in self.projs]
        acts = [self.qas[INPUT_OF[p.name]] for p in self.projs]
        self.group_all = ops.GemvGroup(self.weights, acts, self.outs)
        # dependency-ordered grouping of a real decoder layer: [q,k,v] [o] [gate,up] [down]
        self.groups_dep = [ops.GemvGroup(self.weights[a:b], acts[a:b], self.outs[a:b])
                           for a, b in ((0, 3), (3, 4), (4, 6), (6, 7))]
        # fused quantize+multiply launches: everything at once, and in dependency order
        in_x = [self.xs[INPUT_OF[p.name]] for p in self.projs]
        self.fused_all = ops.DecodeGroup(self.weights, in_x, self.outs)
        self.fused_dep = [ops.DecodeGroup(self.weights[a:b], in_x[a:b], self.outs[a:b])
                          for a, b in ((0, 3), (3, 4), (4, 6), (6, 7))]
        self.quant_all = ops.QuantGroup(self.xs, self.qas)
        self.packed_bytes = sum(p.packed_bytes for p in self.projs)

    # -- the hot path ------------------------------------------------------------------
    def quantize(self):
        for x, qa in zip(self.xs, self.qas):
            ops.quant_act(x, qa)

    def step_fused(self):
        """One launch: every workgroup quantizes its input row on chip, then multiplies."""
        self.fused_all.launch()

    def step_fused_dependency_ordered(self):
        """Four fused launches in the order a real layer's data dependencies allow."""
        for g in self.fused_dep:
            g.launch()

    def step_two_launches(self):
        """All 4 inputs quantized in one grouped launch, then all 7 products in one grouped launch:
        the form to prefer from about 4 tokens up, where the fused launch re-quantizes too much."""
        self.quant_all.launch()
        self.group_all.launch()

    def step_single_launch(self):
        """4 activation quantizations, then all 7 products in one grouped launch."""
        self.quantize()
        self.group_all.launch()

    def step_dependency_ordered(self):
        """Quantize-then-multiply in the order a real layer's data dependencies allow."""
        for i, g in enumerate(self.groups_dep):
            ops.quant_act(self.xs[i], self.qas[i])
            g.launch()

    def step_separate(self):
        """One launch per projection (7 bl_gemv calls) after the 4 quantizations."""
        self.quantize()
        st = int(torch.cuda.current_stream().cuda_stream)
        for w, p, o in zip(self.weights, self.projs, self.outs):
            qa = self.qas[INPUT_OF[p.name]]
            B.bl_gemv(w.blob.data_ptr(), w.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), qa.q_sum.data_ptr(),
                      self.M, o.data_ptr(), 0, st)


def make_inputs(seed: int, hidden: int, ffn: int, M: int, device, outlier_frac: float, host: bool = False):
    """Four bf16 inputs.  Returns (device tensors, host bf16 bit arrays or None)."""
    widths = (hidden, hidden, hidden, ffn)
    if host:
        rng = synth.rng_for(seed)
        bits = [synth.to_bf16_bits(synth.activations(rng, M, k, outlier_frac=outlier_frac)) for k in widths]
        xs = [torch.from_numpy(b.view(np.int16)).to(device).view(torch.bfloat16) for b in bits]
        return xs, bits
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    xs = []
    for k in widths:
        x = torch.randn((M, k), device=device, dtype=torch.float32, generator=g)
        if outlier_frac > 0:
            mask = torch.rand((M, k), device=device, generator=g) < outlier_frac
            x = torch.where(mask, x * 20.0, x)
        xs.append(x.to(torch.bfloat16))
    return xs, None


def make_layer(config: int, layer: int, hidden: int, ffn: int, M: int, device, p_zero: Optional[float],
               outlier_frac: float, host: bool = False, keep_rows=None):
    """Build one synthetic layer.  host=True draws everything with numpy on the host (and also
    returns the host copies, for the oracle); host=False draws on the device.  keep_rows (device
    draw only): per projection an index array; those rows of the DRAWN int8 matrix are copied to the
    host before the matrix is freed and returned as {"w_rows": [...], "w_scale": [...]}, so that a
    parity test can feed the oracle the weights as drawn rather than as unpacked."""
    projs = synth.layer_projections(hidden, ffn)
    weights, host_w, scales, kept = [], [], [], []
    for i, p in enumerate(projs):
        seed = synth.seed_for(config, layer, i)
        rng = synth.rng_for(seed)
        scale = float(synth.draw_w_scale(rng))
        if host:
            w = synth.ternary_weights(rng, p.N, p.K, p_zero=p_zero)
            host_w.append(w)
            wd = torch.from_numpy(w).to(device)
        else:
            wd = synth.ternary_weights_device(seed, p.N, p.K, device, p_zero=p_zero)
            if keep_rows is not None:
                kept.append(wd[torch.as_tensor(np.asarray(keep_rows[i]), device=device)].cpu().numpy())
        weights.append(ops.pack_ternary(wd, scale))
        scales.append(np.float32(scale))
        del wd
    xs, bits = make_inputs(synth.seed_for(config, layer, 9), hidden, ffn, M, device, outlier_frac, host=host)
    lay = DecodeLayer(hidden, ffn, M, device, weights, xs)
    if host:
        return lay, {"w": host_w, "w_scale": scales, "x_bits": bits}
    if keep_rows is not None:
        return lay, {"w_rows": kept, "w_scale": scales}
    return lay, None
