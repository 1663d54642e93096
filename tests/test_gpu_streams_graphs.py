"""The library launches on the stream it is given, never synchronizes, and its launches can be
captured into a HIP graph (the benchmark's timed region is one); every replay must reproduce the
eager results bit for bit, including the work-balanced launches that pass partial sums through the
workspace."""
import numpy as np
import pytest

import oracle
from paper_2410_16144_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def ops():
    from paper_2410_16144_amd import binding
    from paper_2410_16144_amd import ops as _ops
    binding.lib()
    return _ops


def _layers(ops, dev, count, hidden, ffn, M):
    from paper_2410_16144_amd.decode_layer import make_layer
    return [make_layer(2, 50 + i, hidden, ffn, M, dev, 0.4, 0.01)[0] for i in range(count)]


def _snapshot(layers):
    return [[o.clone() for o in l.outs] for l in layers]


def _same(a, b):
    return all(torch.equal(x, y) for la, lb in zip(a, b) for x, y in zip(la, lb))


@pytest.mark.parametrize("M", [1, 4])
def test_graph_replays_equal_eager(dev, ops, M):
    layers = _layers(ops, dev, 3, 3200, 8640, M)     # M = 1 takes the work-balanced kernel (workspace)
    for l in layers:
        l.step_fused()
    torch.cuda.synchronize()
    ref_fused = _snapshot(layers)
    for l in layers:
        l.step_single_launch()
    torch.cuda.synchronize()
    assert _same(ref_fused, _snapshot(layers))
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for l in layers:
                l.step_fused()
            for l in layers:
                l.step_single_launch()
    torch.cuda.synchronize()
    for replay in range(4):
        for l in layers:
            for o in l.outs:
                o.fill_(float(replay))          # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert _same(ref_fused, _snapshot(layers)), "replay %d" % replay
    assert not ops.workspace(dev).any()


def test_launches_follow_the_given_stream(dev, ops):
    """A long kernel is queued on a side stream first; the products queued behind it on the same stream
    must see its result, which they only do if they really run on that stream."""
    rng = synth.rng_for(4242)
    K, N, M = 2048, 512, 2
    w = synth.ternary_weights(rng, N, K)
    bits = synth.to_bf16_bits(synth.activations(rng, M, K))
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), 0.02)
    x_final = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    x = torch.zeros_like(x_final)
    big = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(8):
            big.fill_(1)                       # a few hundred microseconds of work ahead in the queue
        x.copy_(x_final)                       # the product's input only becomes valid after it
        qa = ops.quant_act(x)
        out, acc = ops.gemv(pw, qa, want_acc=True)
        out2, acc2 = ops.gemm(pw, qa, want_acc=True)
        grp = ops.DecodeGroup([pw], [x], want_acc=True)
        grp.launch()
    side.synchronize()
    q_ref, a_ref, _ = oracle.quant_act(bits)
    acc_ref = oracle.matmul_i32(q_ref, w)
    for got in (acc, acc2, grp.accs[0]):
        assert np.array_equal(got.cpu().numpy(), acc_ref)
    assert torch.equal(out, out2) and torch.equal(out, grp.outs[0])
