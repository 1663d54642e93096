"""Parity at the full sizes of the benchmark configurations, in the launch configurations that
bench.py times.  Whole outputs are compared where the oracle finishes in seconds; the prefill
products are compared on sampled output columns and rows (the oracle computes those one by one)
plus the property that the prefill kernel reproduces the decode kernel bit for bit.
"""
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


def _bf16_dev(bits, dev):
    return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)


def _check_out(got, acc_ref, w_scale, a_ref):
    ref = oracle.dequant(acc_ref, w_scale, a_ref)
    assert np.all(np.abs(got - ref) <= 1e-6 * np.abs(ref))
    assert np.array_equal(got == 0, ref == 0)


def _check_layer(ops, dev, config, hidden, ffn, Ms, p_zero, outl):
    """One whole layer (7 projections, 4 inputs) for each M in Ms: fused launch and the
    quantize-then-grouped-GEMV sequence, both against the oracle on every output element."""
    from paper_2410_16144_amd.decode_layer import INPUT_OF, make_layer
    for M in Ms:
        layer, host = make_layer(config, 0, hidden, ffn, M, dev, p_zero, outl, host=True)
        refs_q = [oracle.quant_act(b) for b in host["x_bits"]]
        accs = []
        for i, p in enumerate(layer.projs):
            accs.append(oracle.matmul_i32(refs_q[INPUT_OF[p.name]][0], host["w"][i]))
        # (a) fused launch, with the quantizer's results copied out
        in_x = [layer.xs[INPUT_OF[p.name]] for p in layer.projs]
        grp = ops.DecodeGroup(layer.weights, in_x, want_acc=True, want_quant=True)
        outs = grp.launch()
        torch.cuda.synchronize()
        for i, p in enumerate(layer.projs):
            q, a, s = refs_q[INPUT_OF[p.name]]
            assert np.array_equal(grp.quants[i].q.cpu().numpy()[:, :p.K], q)
            assert np.array_equal(grp.quants[i].a_scale.cpu().numpy().view(np.uint32), a.view(np.uint32))
            assert np.array_equal(grp.quants[i].q_sum.cpu().numpy(), s)
            assert np.array_equal(grp.accs[i].cpu().numpy(), accs[i])
            _check_out(outs[i].cpu().numpy(), accs[i], host["w_scale"][i], a)
        # (b) bl_quant_act x4 + one grouped bl_gemv_batch launch
        for o in layer.outs:
            o.zero_()
        layer.step_single_launch()
        torch.cuda.synchronize()
        for j in range(4):
            assert np.array_equal(layer.qas[j].q.cpu().numpy()[:, :refs_q[j][0].shape[1]], refs_q[j][0])
        for i, p in enumerate(layer.projs):
            _check_out(layer.outs[i].cpu().numpy(), accs[i], host["w_scale"][i], refs_q[INPUT_OF[p.name]][1])
        del layer, grp
        torch.cuda.empty_cache()


def test_config2_3b_layer_decode_m1(dev, ops):
    _check_layer(ops, dev, 2, 3200, 8640, (1,), 0.4, 0.01)


def test_config3_7b_layer_batched_decode(dev, ops):
    _check_layer(ops, dev, 3, 4096, 11008, (1, 4, 8), None, 0.0)


@pytest.mark.parametrize("K,N", [(4096, 11008), (11008, 4096)])
def test_config4_prefill_sampled(dev, ops, K, N):
    rng = synth.rng_for(synth.seed_for(4, 0, 0 if K == 4096 else 1))
    w = synth.ternary_weights(rng, N, K)
    w_scale = synth.draw_w_scale(rng)
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(w_scale))
    for M in (512, 2048):
        bits = synth.to_bf16_bits(synth.activations(rng, M, K))
        qa = ops.quant_act(_bf16_dev(bits, dev))
        out, acc = ops.gemm(pw, qa, want_acc=True)
        torch.cuda.synchronize()
        q_ref, a_ref, s_ref = oracle.quant_act(bits)
        assert np.array_equal(qa.q.cpu().numpy()[:, :K], q_ref)
        assert np.array_equal(qa.a_scale.cpu().numpy().view(np.uint32), a_ref.view(np.uint32))
        acc_h, out_h = acc.cpu().numpy(), out.cpu().numpy()
        # sampled columns (every token): includes the first/last column of tiles and the last column
        cols = np.unique(np.concatenate([rng.integers(0, N, 56), [0, 63, 64, 255, 256, N - 257, N - 64, N - 1]]))
        acc_cols = oracle.matmul_i32_cols(q_ref, w, cols)
        assert np.array_equal(acc_h[:, cols], acc_cols)
        _check_out(out_h[:, cols], acc_cols, w_scale, a_ref)
        # sampled token rows (every column), including tile edges
        rows = np.unique(np.concatenate([rng.integers(0, M, 3), [0, 31, 32, 63, 64, M - 1]]))
        acc_rows = oracle.matmul_i32(np.ascontiguousarray(q_ref[rows]), w)
        assert np.array_equal(acc_h[rows], acc_rows)
        _check_out(out_h[rows], acc_rows, w_scale, a_ref[rows])
        # property at full size: the first 8 tokens through the decode kernel give the same bits
        qa8 = ops.QuantAct(qa.q[:8].contiguous(), qa.a_scale[:8].contiguous(), qa.q_sum[:8].contiguous(), K)
        out8, acc8 = ops.gemv(pw, qa8, want_acc=True)
        assert torch.equal(acc8, acc[:8]) and torch.equal(out8, out[:8])


@pytest.mark.parametrize("K,N,idx", [(12288, 12288, 0), (12288, 33792, 4), (33792, 12288, 6)])
def test_config5_100b_shapes_decode_m1(dev, ops, K, N, idx):
    rng = synth.rng_for(synth.seed_for(5, 0, idx))
    w = synth.ternary_weights(rng, N, K)
    w_scale = synth.draw_w_scale(rng)
    bits = synth.to_bf16_bits(synth.activations(rng, 1, K))
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(w_scale))
    x = _bf16_dev(bits, dev)
    q_ref, a_ref, s_ref = oracle.quant_act(bits)
    acc_ref = oracle.matmul_i32(q_ref, w)
    grp = ops.DecodeGroup([pw], [x], want_acc=True, want_quant=True)
    out = grp.launch()[0]
    qa = ops.quant_act(x)
    out2, acc2 = ops.gemv(pw, qa, want_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(grp.quants[0].q.cpu().numpy()[:, :K], q_ref)
    assert np.array_equal(grp.accs[0].cpu().numpy(), acc_ref)
    assert np.array_equal(acc2.cpu().numpy(), acc_ref)
    _check_out(out.cpu().numpy(), acc_ref, w_scale, a_ref)
    _check_out(out2.cpu().numpy(), acc_ref, w_scale, a_ref)


def test_config5_100b_whole_layer_fused_launch(dev, ops):
    """Layer 0 of the 100B-shape model, all 7 matrices in the launches bench.py times (fused and
    grouped), every output element against the oracle."""
    _check_layer(ops, dev, 5, 12288, 33792, (1,), None, 0.0)


@pytest.mark.parametrize("layer_index", [1, 79])
def test_config5_100b_device_drawn_layers_sampled_rows(dev, ops, layer_index):
    """Layers drawn on the device (as the 37 GB benchmark model is): 64 seeded rows per matrix plus the
    first and last row of the DRAWN int8 matrix are copied to the host before the matrix is packed and
    freed; the oracle computes those outputs one by one from them.  Second assertion: the same rows
    come back unchanged through bl_unpack_ternary."""
    from paper_2410_16144_amd.decode_layer import INPUT_OF, make_layer
    rng = synth.rng_for(synth.seed_for(5, layer_index, 8))
    projs = synth.layer_projections(12288, 33792)
    rows_of = [np.unique(np.concatenate([rng.integers(0, p.N, 64), [0, p.N - 1]])) for p in projs]
    layer, drawn = make_layer(5, layer_index, 12288, 33792, 1, dev, None, 0.0, keep_rows=rows_of)
    layer.step_fused()
    torch.cuda.synchronize()
    fused = [o.cpu().numpy().copy() for o in layer.outs]
    for o in layer.outs:
        o.zero_()
    layer.step_single_launch()
    torch.cuda.synchronize()
    x_bits = [x.view(torch.int16).cpu().numpy().view(np.uint16) for x in layer.xs]
    refs_q = [oracle.quant_act(b) for b in x_bits]
    for i, p in enumerate(layer.projs):
        q, a, s = refs_q[INPUT_OF[p.name]]
        rows, w_rows = rows_of[i], drawn["w_rows"][i]
        assert w_rows.shape == (rows.size, p.K) and set(np.unique(w_rows)) <= {-1, 0, 1}
        acc_ref = oracle.matmul_i32(q, np.ascontiguousarray(w_rows))
        w_scale = drawn["w_scale"][i]
        assert w_scale == np.float32(layer.weights[i].desc.w_scale)
        for got in (fused[i], layer.outs[i].cpu().numpy()):
            _check_out(got[:, rows], acc_ref, w_scale, a)
        back = ops.unpack_ternary(layer.weights[i])[torch.from_numpy(rows).to(dev)].cpu().numpy()
        assert np.array_equal(back, w_rows)
    del layer
    torch.cuda.empty_cache()
