"""bl_gemv_batch_static: the grouped decode launch whose workspace is the library's static device array.

Through the C ABI, two calls in a row (the second on a smaller input), each compared with bl_gemv_batch on a
caller-owned workspace (bit for bit) and with the oracle (int32 sums exact, fp32 within 1e-6).  The shapes are chosen
so that the work-balanced kernel, the one that uses the scratch, is what runs.
"""
import numpy as np
import pytest

import oracle
from paper_2410_16144_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

REL_TOL = 1e-6


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def _problem(ops, dev, seed, shapes):
    """Matrices of `shapes` (N, K) sharing nothing; returns device and host sides."""
    rng = synth.rng_for(seed)
    ws, pws, qas, refs = [], [], [], []
    for N, K in shapes:
        w = synth.ternary_weights(rng, N, K, p_zero=0.4)
        scale = synth.draw_w_scale(rng)
        bits = synth.to_bf16_bits(synth.activations(rng, 1, K, outlier_frac=0.01))
        x = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        pws.append(ops.pack_ternary(torch.from_numpy(w).to(dev), float(scale)))
        qas.append(ops.quant_act(x))
        q, a, _ = oracle.quant_act(bits)
        acc = oracle.matmul_i32(q, w)
        refs.append((acc, oracle.dequant(acc, scale, a)))
        ws.append(w)
    return pws, qas, refs


def _run_both(ops, binding, dev, pws, qas):
    outs_s = [torch.full((1, p.N), float("nan"), dtype=torch.float32, device=dev) for p in pws]
    accs_s = [torch.full((1, p.N), -7, dtype=torch.int32, device=dev) for p in pws]
    items = binding.make_gemv_items(
        (p.blob.data_ptr(), p.desc, a.q.data_ptr(), a.a_scale.data_ptr(), a.q_sum.data_ptr(), o.data_ptr(), c.data_ptr())
        for p, a, o, c in zip(pws, qas, outs_s, accs_s))
    st = int(torch.cuda.current_stream().cuda_stream)
    before = binding.bl_get_stat("split_launches")
    binding.bl_gemv_batch_static(items, 1, st)
    split = binding.bl_get_stat("split_launches") - before
    grp = ops.GemvGroup(pws, qas, want_acc=True, use_workspace=torch.zeros(binding.BL_WORKSPACE_BYTES, dtype=torch.uint8, device=dev))
    outs_w = grp.launch()
    torch.cuda.synchronize()
    return outs_s, accs_s, outs_w, grp.accs, split


def test_static_workspace_entry_point_two_calls(dev):
    from paper_2410_16144_amd import binding, ops
    binding.lib()
    # first a 3B-shape group (Q, K, V, O-sized and one gate-sized matrix), then a smaller, ragged one
    for seed, shapes in ((9101, [(3200, 3200)] * 3 + [(8640, 3200)]), (9102, [(3000, 3136), (3100, 3200)])):
        pws, qas, refs = _problem(ops, dev, seed, shapes)
        outs_s, accs_s, outs_w, accs_w, split = _run_both(ops, binding, dev, pws, qas)
        assert split == 1, "the shapes are meant to take the work-balanced kernel, which uses the scratch"
        for i, (acc_ref, out_ref) in enumerate(refs):
            assert torch.equal(accs_s[i], accs_w[i]) and torch.equal(outs_s[i], outs_w[i])
            assert np.array_equal(accs_s[i].cpu().numpy(), acc_ref)
            got = outs_s[i].cpu().numpy()
            assert np.all(np.abs(got - out_ref) <= REL_TOL * np.abs(out_ref))
            assert np.array_equal(got == 0, out_ref == 0)


def test_static_workspace_rejects_a_plan_beyond_its_size(dev):
    from paper_2410_16144_amd import binding, ops
    binding.lib()
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    if cus * 8 <= binding.BL_STATIC_WS_WGS:
        pytest.skip("this device cannot plan more workgroups than the static scratch serves")
    pws, qas, _ = _problem(ops, dev, 9103, [(8640, 3200)] * 4)
    out = [torch.zeros((1, p.N), dtype=torch.float32, device=dev) for p in pws]
    items = binding.make_gemv_items(
        (p.blob.data_ptr(), p.desc, a.q.data_ptr(), a.a_scale.data_ptr(), a.q_sum.data_ptr(), o.data_ptr(), 0)
        for p, a, o in zip(pws, qas, out))
    binding.bl_set_tuning("decode_split", 8)
    try:
        with pytest.raises(binding.BitLinearError) as err:
            binding.bl_gemv_batch_static(items, 1, int(torch.cuda.current_stream().cuda_stream))
        assert err.value.status == binding.BL_ERR_WORKSPACE
    finally:
        binding.bl_set_tuning("decode_split", 0)
    torch.cuda.synchronize()
    assert not any(bool(o.any()) for o in out)       # nothing was launched
    # and the array still serves the next ordinary call
    binding.bl_gemv_batch_static(items, 1, int(torch.cuda.current_stream().cuda_stream))
    ref = ops.GemvGroup(pws, qas).launch()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(out, ref))
