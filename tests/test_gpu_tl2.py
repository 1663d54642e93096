"""GPU parity of the 1.78-bit layout built on the paper's TL2 code (Table 3): pack / unpack against the
oracle's codes read through the documented layout, and the one-token decode product against the oracle's
exact accumulators and against the 2-bit kernel on the same weights."""
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


@pytest.fixture(scope="module")
def ops():
    from paper_2410_16144_amd import binding, ops as _ops
    binding.lib()
    return _ops


def codes_of_blob(blob, N, K):
    """Independent reading of the documented version-2 layout (include/bitlinear.h): -> [Np, Kp/3] codes."""
    Np, KC = (N + 63) // 64 * 64, (K + 71) // 72
    words = np.frombuffer(blob.tobytes(), dtype="<u4").reshape(Np // 64, KC, 64, 4)   # rb, kc, r, s
    assert not (words >> np.uint32(30)).any()
    codes = np.zeros((Np // 64, 64, KC, 4, 6), np.uint8)                              # rb, r, kc, s, i
    for i in range(6):
        codes[..., i] = ((words >> np.uint32(5 * i)) & np.uint32(31)).transpose(0, 2, 1, 3)
    return codes.reshape(Np, KC * 24)


@pytest.mark.parametrize("N,K", [(64, 72), (1, 1), (70, 100), (130, 1000), (257, 3200), (64, 73), (200, 8640)])
def test_tl2_pack_matches_table3_codes_and_round_trips(dev, ops, N, K):
    rng = synth.rng_for(7000 + N + K)
    w = synth.ternary_weights(rng, N, K, p_zero=0.4)
    pw = ops.tl2_pack(torch.from_numpy(w).to(dev), 0.02)
    assert pw.desc.version == 2 and pw.blob.numel() == pw.desc.bytes
    got = codes_of_blob(pw.blob.cpu().numpy(), N, K)
    ref, bad = oracle.tl2_encode_rows(w)
    assert bad == 0
    groups = (K + 2) // 3
    assert np.array_equal(got[:N, :groups], ref)
    assert not got[N:].any() and not got[:, groups:].any()        # padding rows and groups are zero weights
    assert torch.equal(ops.tl2_unpack(pw).cpu(), torch.from_numpy(w))


def test_tl2_pack_counts_non_ternary(dev, ops):
    w = np.zeros((3, 10), np.int8)
    w[0, 0], w[1, 4], w[2, 9] = 2, -2, 100
    w[0, 1] = -1
    bad = torch.zeros(1, dtype=torch.int32, device=dev)
    pw = ops.tl2_pack(torch.from_numpy(w).to(dev), 1.0, bad)
    assert int(bad.item()) == 3
    back = ops.tl2_unpack(pw).cpu().numpy()
    exp = w.copy()
    exp[0, 0] = exp[1, 4] = exp[2, 9] = 0
    assert np.array_equal(back, exp)


def _quantized(ops, dev, x_bits, K):
    x = torch.from_numpy(x_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    return x, ops.quant_act(x, ops.tl2_quant_buffer(K, dev))


@pytest.mark.parametrize("N,K", [(64, 72), (1, 1), (70, 100), (200, 1000), (257, 3200), (3200, 8640), (129, 72 * 37),
                                 (192, 33792), (1100, 72 * 8 * 16 + 5), (64, 65536 + 64)])
def test_tl2_gemv_parity(dev, ops, N, K):
    rng = synth.rng_for(7100 + 3 * N + K)
    w = synth.ternary_weights(rng, N, K, p_zero=0.4)
    w_scale = float(synth.draw_w_scale(rng))
    bits = synth.to_bf16_bits(synth.activations(rng, 1, K, outlier_frac=0.01))
    x, qa = _quantized(ops, dev, bits, K)
    qa.q[0, ops.B.bl_padded_k(K):] = 77           # beyond what the quantizer writes: must meet zero weights
    pw = ops.tl2_pack(torch.from_numpy(w).to(dev), w_scale)
    out, acc = ops.tl2_gemv(pw, qa, want_acc=True)
    torch.cuda.synchronize()
    ref = oracle.bitlinear(bits, w, np.float32(w_scale))
    assert np.array_equal(qa.q.cpu().numpy()[:, :K], ref["q"])
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    got = out.cpu().numpy()
    assert np.all(np.abs(got - ref["out"]) <= REL_TOL * np.abs(ref["out"])) and np.array_equal(got == 0, ref["out"] == 0)
    # and bit for bit what the 2-bit kernel gives on the same weights
    pw2 = ops.pack_ternary(torch.from_numpy(w).to(dev), w_scale)
    qa2 = ops.quant_act(x)
    out2, acc2 = ops.gemv(pw2, qa2, want_acc=True)
    assert torch.equal(acc, acc2) and torch.equal(out, out2)


def test_tl2_gemv_closed_forms(dev, ops):
    K, N = 72 * 5 + 7, 130
    rng = synth.rng_for(7200)
    bits = synth.to_bf16_bits(synth.activations(rng, 1, K))
    x, qa = _quantized(ops, dev, bits, K)
    q = qa.q.cpu().numpy()[0, :K].astype(np.int64)
    # all +1: every row is sum(q); all -1: its negative; one-hot rows pick single activations
    for val in (1, -1):
        pw = ops.tl2_pack(torch.full((N, K), val, dtype=torch.int8, device=dev), 1.0)
        _, acc = ops.tl2_gemv(pw, qa, want_acc=True)
        assert (acc.cpu().numpy() == val * q.sum()).all()
    w = np.zeros((N, K), np.int8)
    for n in range(N):
        w[n, (n * 3) % K] = 1 if n % 2 else -1
    pw = ops.tl2_pack(torch.from_numpy(w).to(dev), 1.0)
    _, acc = ops.tl2_gemv(pw, qa, want_acc=True)
    exp = np.array([(1 if n % 2 else -1) * q[(n * 3) % K] for n in range(N)])
    assert np.array_equal(acc.cpu().numpy()[0], exp)


def _layer_problems(shapes, seed):
    probs = []
    for i, (N, K) in enumerate(shapes):
        rng = synth.rng_for(seed + i)
        w = synth.ternary_weights(rng, N, K, p_zero=0.4)
        bits = synth.to_bf16_bits(synth.activations(rng, 1, K, outlier_frac=0.01))
        probs.append((w, float(synth.draw_w_scale(rng)), bits))
    return probs


def _assert_tl2_batch(ops, dev, probs, use_workspace, expect_split):
    from paper_2410_16144_amd import binding
    weights, acts = [], []
    for w, s, bits in probs:
        weights.append(ops.tl2_pack(torch.from_numpy(w).to(dev), s))
        acts.append(_quantized(ops, dev, bits, w.shape[1])[1])
    before = binding.bl_get_stat("split_launches")
    grp = ops.Tl2GemvGroup(weights, acts, want_acc=True, use_workspace=use_workspace)
    grp.launch()
    torch.cuda.synchronize()
    assert binding.bl_get_stat("split_launches") - before == (1 if expect_split else 0)
    if use_workspace:
        assert not ops.workspace(dev).any()          # the balanced form leaves its workspace zero
    for i, (w, s, bits) in enumerate(probs):
        ref = oracle.bitlinear(bits, w, np.float32(s))
        assert np.array_equal(grp.accs[i].cpu().numpy(), ref["acc"]), i
        got = grp.outs[i].cpu().numpy()
        assert np.all(np.abs(got - ref["out"]) <= REL_TOL * np.abs(ref["out"])), i
    first = [o.clone() for o in grp.outs]
    grp.launch()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(first, grp.outs))


def test_tl2_batch_of_seven_row_block_form(dev, ops):
    shapes = [(320, 640), (320, 640), (128, 640), (640, 320), (64, 72), (200, 1000), (1000, 200)]
    _assert_tl2_batch(ops, dev, _layer_problems(shapes, 7300), use_workspace=False, expect_split=False)


@pytest.mark.parametrize("n", [1, 2])
def test_tl2_batch_balanced_form(dev, ops, n):
    from paper_2410_16144_amd import binding
    binding.bl_set_tuning("decode_split", n)
    try:
        shapes = [(2000 * n, 4000), (1000 * n, 9000), (5000 * n, 3000), (700 * n, 6000), (64, 72), (2000 * n, 4000), (130, 12000)]
        _assert_tl2_batch(ops, dev, _layer_problems(shapes, 7400 + n), use_workspace=True, expect_split=True)
        # one matrix whose every row block is shared by several workgroups
        _assert_tl2_batch(ops, dev, _layer_problems([(4100, 8200)], 7450 + n), use_workspace=True, expect_split=True)
    finally:
        binding.bl_set_tuning("decode_split", 0)


def test_tl2_layer_shape_automatic_choice(dev, ops):
    projs = synth.layer_projections(3200, 8640)
    _assert_tl2_batch(ops, dev, _layer_problems([(p.N, p.K) for p in projs], 7500), use_workspace=True, expect_split=True)

