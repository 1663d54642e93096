"""Torch-tensor conveniences over the C ABI: allocate outputs, pass data_ptr() and the current
stream.  No arithmetic happens here; every step runs in the library's HIP kernels."""
from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as B


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


@dataclass
class PackedWeight:
    blob: torch.Tensor          # uint8 [desc.bytes], device
    desc: B.PackedDesc

    @property
    def N(self):
        return int(self.desc.N)

    @property
    def K(self):
        return int(self.desc.K)

    @property
    def packed_bytes(self) -> int:
        """Unpadded 2-bit size N*K/4: the algorithmic bytes of one decode product."""
        return self.N * self.K // 4


def pack_ternary(w: torch.Tensor, w_scale: float, bad_count: Optional[torch.Tensor] = None) -> PackedWeight:
    """w: [N,K] int8 device tensor in {-1,0,+1} -> PackedWeight (bl_pack_ternary)."""
    assert w.is_cuda and w.dtype == torch.int8 and w.dim() == 2 and w.is_contiguous()
    N, K = w.shape
    desc = B.bl_packed_desc_init(N, K, w_scale)
    blob = torch.empty(int(desc.bytes), dtype=torch.uint8, device=w.device)
    B.bl_pack_ternary(w.data_ptr(), desc, blob.data_ptr(), bad_count.data_ptr() if bad_count is not None else 0,
                      _stream())
    return PackedWeight(blob, desc)


def unpack_ternary(pw: PackedWeight) -> torch.Tensor:
    w = torch.empty((pw.N, pw.K), dtype=torch.int8, device=pw.blob.device)
    B.bl_unpack_ternary(pw.blob.data_ptr(), pw.desc, w.data_ptr(), _stream())
    return w


def tl2_pack(w: torch.Tensor, w_scale: float, bad_count: Optional[torch.Tensor] = None) -> PackedWeight:
    """w: [N,K] int8 device tensor in {-1,0,+1} -> PackedWeight in the 1.78-bit layout (bl_tl2_pack)."""
    assert w.is_cuda and w.dtype == torch.int8 and w.dim() == 2 and w.is_contiguous()
    N, K = w.shape
    desc = B.bl_tl2_desc_init(N, K, w_scale)
    blob = torch.empty(int(desc.bytes), dtype=torch.uint8, device=w.device)
    B.bl_tl2_pack(w.data_ptr(), desc, blob.data_ptr(), bad_count.data_ptr() if bad_count is not None else 0, _stream())
    return PackedWeight(blob, desc)


def tl2_unpack(pw: PackedWeight) -> torch.Tensor:
    w = torch.empty((pw.N, pw.K), dtype=torch.int8, device=pw.blob.device)
    B.bl_tl2_unpack(pw.blob.data_ptr(), pw.desc, w.data_ptr(), _stream())
    return w


def tl2_quant_buffer(K: int, device) -> "QuantAct":
    """Quantization outputs for ONE token whose q row is long enough for bl_tl2_gemv (bl_tl2_padded_k(K) bytes,
    zero beyond what bl_quant_act writes)."""
    n = max(B.bl_tl2_padded_k(K), B.bl_padded_k(K))
    return QuantAct(torch.zeros((1, n), dtype=torch.int8, device=device),
                    torch.empty((1,), dtype=torch.float32, device=device),
                    torch.empty((1,), dtype=torch.int32, device=device), K)


def tl2_gemv(pw: PackedWeight, qa: "QuantAct", out: Optional[torch.Tensor] = None, want_acc: bool = False):
    """One-token decode product over a 1.78-bit blob (bl_tl2_gemv).  qa: from quant_act(x, tl2_quant_buffer(K, dev))."""
    assert qa.q.shape[0] == 1 and qa.q.shape[1] >= B.bl_tl2_padded_k(pw.K)
    dev = pw.blob.device
    if out is None:
        out = torch.empty((1, pw.N), dtype=torch.float32, device=dev)
    acc = torch.empty((1, pw.N), dtype=torch.int32, device=dev) if want_acc else None
    B.bl_tl2_gemv(pw.blob.data_ptr(), pw.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), out.data_ptr(),
                  acc.data_ptr() if acc is not None else 0, _stream())
    return (out, acc) if want_acc else out


@dataclass
class QuantAct:
    q: torch.Tensor         # int8 [M, Kp]
    a_scale: torch.Tensor   # fp32 [M]
    q_sum: torch.Tensor     # int32 [M]
    K: int

    @property
    def M(self):
        return int(self.q.shape[0])


def alloc_quant(M: int, K: int, device) -> QuantAct:
    Kp = B.bl_padded_k(K)
    return QuantAct(torch.empty((M, Kp), dtype=torch.int8, device=device),
                    torch.empty((M,), dtype=torch.float32, device=device),
                    torch.empty((M,), dtype=torch.int32, device=device), K)


def quant_act(x: torch.Tensor, out: Optional[QuantAct] = None) -> QuantAct:
    """x: [M,K] fp32 or bf16 device tensor (last dim contiguous) -> QuantAct (bl_quant_act)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    if x.dtype == torch.float32:
        dt = B.BL_F32
    elif x.dtype == torch.bfloat16:
        dt = B.BL_BF16
    else:
        raise TypeError("activations must be float32 or bfloat16")
    M, K = x.shape
    if out is None:
        out = alloc_quant(M, K, x.device)
    B.bl_quant_act(x.data_ptr(), dt, M, K, x.stride(0), out.q.data_ptr(), out.a_scale.data_ptr(),
                   out.q_sum.data_ptr(), _stream())
    return out


class QuantGroup:
    """A prepared grouped quantization launch (bl_quant_act_batch): up to 8 inputs, one kernel."""

    def __init__(self, xs, outs=None):
        assert 1 <= len(xs) <= B.BL_MAX_BATCH
        self.xs = list(xs)
        for x in self.xs:
            assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
        self.outs = list(outs) if outs is not None else [
            alloc_quant(int(x.shape[0]), int(x.shape[1]), x.device) for x in self.xs]
        self.items = B.make_quant_items(
            (x.data_ptr(), _dtype_code(x), int(x.shape[0]), int(x.shape[1]), x.stride(0), o.q.data_ptr(),
             o.a_scale.data_ptr(), o.q_sum.data_ptr()) for x, o in zip(self.xs, self.outs))

    def launch(self):
        B.bl_quant_act_batch(self.items, _stream())
        return self.outs


def _product(fn, pw: PackedWeight, qa: QuantAct, out, want_acc):
    M = qa.M
    assert qa.K == pw.K
    if out is None:
        out = torch.empty((M, pw.N), dtype=torch.float32, device=pw.blob.device)
    acc = torch.empty((M, pw.N), dtype=torch.int32, device=pw.blob.device) if want_acc else None
    fn(pw.blob.data_ptr(), pw.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), qa.q_sum.data_ptr(), M,
       out.data_ptr(), acc.data_ptr() if acc is not None else 0, _stream())
    return (out, acc) if want_acc else out


def gemv(pw: PackedWeight, qa: QuantAct, out: Optional[torch.Tensor] = None, want_acc: bool = False):
    """Decode product, M <= 8 (bl_gemv).  Returns out [M,N] fp32 (and acc int32 if want_acc)."""
    return _product(B.bl_gemv, pw, qa, out, want_acc)


def gemm(pw: PackedWeight, qa: QuantAct, out: Optional[torch.Tensor] = None, want_acc: bool = False):
    """Prefill product (bl_gemm)."""
    return _product(B.bl_gemm, pw, qa, out, want_acc)


def gemm_batch(pws, qa: QuantAct):
    """Several prefill products over the same quantized activations in ONE launch (bl_gemm_batch): a list of fp32
    outputs [M, N_i], each identical to gemm(pw_i, qa)."""
    M, dev = qa.M, qa.q.device
    assert 1 <= len(pws) <= B.BL_MAX_GEMM_BATCH and all(pw.K == qa.K for pw in pws)
    outs = [torch.empty((M, pw.N), dtype=torch.float32, device=dev) for pw in pws]
    B.bl_gemm_batch([(pw.blob.data_ptr(), pw.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), qa.q_sum.data_ptr(), o.data_ptr(), 0)
                     for pw, o in zip(pws, outs)], M, _stream())
    return outs


_workspaces = {}


def workspace(device) -> torch.Tensor:
    """The zero-filled workspace of the work-balanced decode launches, one per device.  Launches that
    may overlap in time (different streams) must not share one: give those groups a tensor of their own."""
    key = torch.device(device).index or 0
    ws = _workspaces.get(key)
    if ws is None:
        ws = _workspaces[key] = torch.zeros(B.BL_WORKSPACE_BYTES, dtype=torch.uint8, device=device)
    return ws


def _workspace_ptr(use_workspace, device) -> int:
    """use_workspace: True = the device's shared workspace, False = none, or a zero-filled uint8 tensor."""
    if use_workspace is True:
        return workspace(device).data_ptr()
    if use_workspace is False or use_workspace is None:
        return 0
    assert use_workspace.is_cuda and use_workspace.numel() * use_workspace.element_size() >= B.BL_WORKSPACE_BYTES
    return use_workspace.data_ptr()


class GemvGroup:
    """A prepared grouped decode launch (bl_gemv_batch): fixed weights, activations and outputs."""

    def __init__(self, weights, acts, outs=None, want_acc=False, use_workspace=True):
        assert 1 <= len(weights) <= B.BL_MAX_BATCH and len(weights) == len(acts)
        self.use_workspace = use_workspace
        self.workspace_ptr = _workspace_ptr(use_workspace, weights[0].blob.device)
        self.M = acts[0].M
        dev = weights[0].blob.device
        self.weights, self.acts = list(weights), list(acts)
        self.outs = list(outs) if outs is not None else [
            torch.empty((self.M, w.N), dtype=torch.float32, device=dev) for w in weights]
        self.accs = [torch.empty((self.M, w.N), dtype=torch.int32, device=dev) for w in weights] if want_acc else None
        self.items = B.make_gemv_items(
            (w.blob.data_ptr(), w.desc, a.q.data_ptr(), a.a_scale.data_ptr(), a.q_sum.data_ptr(), o.data_ptr(),
             self.accs[i].data_ptr() if want_acc else 0)
            for i, (w, a, o) in enumerate(zip(self.weights, self.acts, self.outs)))

    def launch(self):
        B.bl_gemv_batch(self.items, self.M, self.workspace_ptr, _stream())
        return self.outs


class Tl2GemvGroup:
    """A prepared grouped one-token launch over 1.78-bit blobs (bl_tl2_gemv_batch).  acts[i]: from
    quant_act(x, tl2_quant_buffer(K, dev))."""

    def __init__(self, weights, acts, outs=None, want_acc=False, use_workspace=True):
        assert 1 <= len(weights) <= B.BL_MAX_BATCH and len(weights) == len(acts)
        dev = weights[0].blob.device
        self.workspace_ptr = _workspace_ptr(use_workspace, dev)
        for w, a in zip(weights, acts):
            assert a.q.shape[0] == 1 and a.q.shape[1] >= B.bl_tl2_padded_k(w.K)
        self.weights, self.acts = list(weights), list(acts)
        self.outs = list(outs) if outs is not None else [
            torch.empty((1, w.N), dtype=torch.float32, device=dev) for w in weights]
        self.accs = [torch.empty((1, w.N), dtype=torch.int32, device=dev) for w in weights] if want_acc else None
        self.items = B.make_gemv_items(
            (w.blob.data_ptr(), w.desc, a.q.data_ptr(), a.a_scale.data_ptr(), 0, o.data_ptr(),
             self.accs[i].data_ptr() if want_acc else 0)
            for i, (w, a, o) in enumerate(zip(self.weights, self.acts, self.outs)))

    def launch(self):
        B.bl_tl2_gemv_batch(self.items, self.workspace_ptr, _stream())
        return self.outs


def _dtype_code(x: torch.Tensor) -> int:
    if x.dtype == torch.float32:
        return B.BL_F32
    if x.dtype == torch.bfloat16:
        return B.BL_BF16
    raise TypeError("activations must be float32 or bfloat16")


class DecodeGroup:
    """A prepared fused decode launch (bl_decode_batch): quantization + product of up to 8
    BitLinears in one kernel.  `xs[i]` is the [M,K_i] input of `weights[i]` (inputs may repeat)."""

    def __init__(self, weights, xs, outs=None, want_acc=False, want_quant=False, use_workspace=True):
        assert 1 <= len(weights) <= B.BL_MAX_BATCH and len(weights) == len(xs)
        self.use_workspace = use_workspace
        self.workspace_ptr = _workspace_ptr(use_workspace, weights[0].blob.device)
        self.M = int(xs[0].shape[0])
        dev = weights[0].blob.device
        self.weights, self.xs = list(weights), list(xs)
        for w, x in zip(self.weights, self.xs):
            assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.shape == (self.M, w.K)
        self.outs = list(outs) if outs is not None else [
            torch.empty((self.M, w.N), dtype=torch.float32, device=dev) for w in weights]
        self.accs = [torch.empty((self.M, w.N), dtype=torch.int32, device=dev) for w in weights] if want_acc else None
        self.quants = [alloc_quant(self.M, w.K, dev) for w in weights] if want_quant else None
        # From two tokens up the library quantizes every distinct input ONCE per launch and publishes the rows through
        # the items' quantization buffers (see bl_decode_batch): give it such buffers, one set per distinct input.
        pub = self.quants
        if pub is None and self.M >= 2 and self.workspace_ptr:
            shared = {}
            for w, x in zip(self.weights, self.xs):
                key = (x.data_ptr(), x.stride(0), w.K)
                if key not in shared:
                    shared[key] = alloc_quant(self.M, w.K, dev)
            pub = [shared[(x.data_ptr(), x.stride(0), w.K)] for w, x in zip(self.weights, self.xs)]
        self.published = pub
        self.items = B.make_decode_items(
            (x.data_ptr(), _dtype_code(x), x.stride(0), w.blob.data_ptr(), w.desc, o.data_ptr(),
             self.accs[i].data_ptr() if want_acc else 0,
             pub[i].q.data_ptr() if pub else 0,
             pub[i].a_scale.data_ptr() if pub else 0,
             pub[i].q_sum.data_ptr() if pub else 0)
            for i, (w, x, o) in enumerate(zip(self.weights, self.xs, self.outs)))

    def launch(self):
        B.bl_decode_batch(self.items, self.M, self.workspace_ptr, _stream())
        return self.outs
