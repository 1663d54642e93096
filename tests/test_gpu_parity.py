"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on the same
seeded inputs.  int8 activations, scales and int32 accumulators must be bit-identical; fp32
outputs within 1e-6 relative (and exactly 0 where the accumulator is 0).
"""
import numpy as np
import pytest

import oracle
from paper_2410_16144_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

REL_TOL = 1e-6   # product of the two scales, three roundings at most


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def ops():
    from paper_2410_16144_amd import ops as _ops
    from paper_2410_16144_amd import binding
    binding.lib()   # fails loudly if the library is not built
    return _ops


def _to_dev_bf16(bits, dev):
    return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)


def _check_out(out_gpu, acc_ref, w_scale, a_scale_ref):
    ref = oracle.dequant(acc_ref, w_scale, a_scale_ref)
    got = out_gpu.cpu().numpy()
    assert got.shape == ref.shape
    denom = np.maximum(np.abs(ref), 1e-30)
    assert np.all(np.abs(got - ref) <= REL_TOL * denom), float(np.max(np.abs(got - ref) / denom))
    assert np.array_equal(got == 0, ref == 0)


def decode_blob_host(blob, N, K):
    """Independent reading of the documented version-1 layout (see include/bitlinear.h)."""
    Np, Kp = (N + 63) // 64 * 64, (K + 63) // 64 * 64
    words = np.frombuffer(blob.tobytes(), dtype="<u4").reshape(Np // 64, Kp // 64, 64, 4)  # rb, kc, r, s
    w = np.zeros((Np, Kp), np.int8)
    w5 = w.reshape(Np // 64, 64, Kp // 64, 4, 16)                                          # rb, r, kc, s, t
    for t in range(16):
        j, b = t // 4, t % 4
        codes = (words >> np.uint32(8 * b + 2 * j)) & np.uint32(3)
        assert codes.max() <= 2
        w5[:, :, :, :, t] = (codes.astype(np.int8) - 1).transpose(0, 2, 1, 3)
    return w[:N, :K], w


# ------------------------------------------------------------------ pack / unpack

@pytest.mark.parametrize("N,K", [(64, 64), (1, 1), (70, 100), (130, 1000), (257, 4097 - 64), (1536, 1536),
                                 (3200, 8640)])
def test_pack_unpack_roundtrip_and_documented_layout(dev, ops, N, K):
    rng = synth.rng_for(N * 7 + K)
    w = synth.ternary_weights(rng, N, K, p_zero=0.4)
    wd = torch.from_numpy(w).to(dev)
    pw = ops.pack_ternary(wd, 0.02)
    assert pw.blob.numel() == ((N + 63) // 64 * 64) * ((K + 63) // 64 * 64) // 4
    back = ops.unpack_ternary(pw)
    assert torch.equal(back, wd)
    got, padded = decode_blob_host(pw.blob.cpu().numpy(), N, K)
    assert np.array_equal(got, w)
    padded[:N, :K] = 0
    assert not padded.any()                       # padding is weight 0 (code 01)


def test_pack_counts_non_ternary(dev, ops):
    w = synth.ternary_weights(synth.rng_for(3), 100, 200)
    w[5, 7] = 2
    w[99, 199] = -128
    w[0, 0] = 127
    bad = torch.zeros(1, dtype=torch.int32, device=dev)
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), 1.0, bad_count=bad)
    assert int(bad.item()) == 3
    w[5, 7] = w[99, 199] = w[0, 0] = 0
    assert np.array_equal(ops.unpack_ternary(pw).cpu().numpy(), w)


# ------------------------------------------------------------------ activation quantizer

def _quant_both(ops, dev, x_np, bf16):
    if bf16:
        bits = synth.to_bf16_bits(x_np)
        ref = oracle.quant_act(bits)
        xd = _to_dev_bf16(bits, dev)
    else:
        ref = oracle.quant_act(x_np)
        xd = torch.from_numpy(x_np).to(dev)
    qa = ops.quant_act(xd)
    return qa, ref


def _assert_quant_equal(qa, ref, K):
    q_ref, a_ref, s_ref = ref
    q = qa.q.cpu().numpy()
    assert np.array_equal(q[:, :K], q_ref)
    assert not q[:, K:].any()
    assert np.array_equal(qa.a_scale.cpu().numpy().view(np.uint32), a_ref.view(np.uint32))
    assert np.array_equal(qa.q_sum.cpu().numpy(), s_ref)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("M,K,outl", [(1, 1536, 0.0), (1, 3200, 0.01), (3, 8640, 0.01), (8, 4096, 0.0),
                                      (5, 100, 0.0), (2, 1001, 0.05), (1, 7, 0.0), (64, 11008, 0.0),
                                      (1, 33792, 0.0)])
def test_quant_act_bit_exact(dev, ops, M, K, outl, bf16):
    rng = synth.rng_for(M * 100003 + K)
    x = synth.activations(rng, M, K, outlier_frac=outl)
    qa, ref = _quant_both(ops, dev, x, bf16)
    _assert_quant_equal(qa, ref, K)


def test_quant_act_edge_rows(dev, ops):
    K = 256
    x = np.zeros((8, K), np.float32)
    rng = synth.rng_for(77)
    x[1] = rng.standard_normal(K).astype(np.float32)
    x[2, :8] = [127.0, 62.5, -61.5, 0.5, 1.5, 2.5, -0.5, -2.5]        # exact ties (inv = 1)
    x[3] = 1e-38                                                      # absmax too small: zero token
    x[3, 5] = -2e-40
    x[4, :5] = [5e-37, -2.5e-37, 8e-39, -1e-45, 4e-39]                # denormal inputs, finite inv (2.54e38)
    x[5] = x[1] * np.float32(2.0 ** 40)
    x[6] = -x[1]
    x[7, 100] = -3.0                                                  # single non-zero
    qa, ref = _quant_both(ops, dev, x, False)
    _assert_quant_equal(qa, ref, K)
    q = qa.q.cpu().numpy()
    assert q[2, :8].tolist() == [127, 62, -62, 0, 2, 2, 0, -2]
    assert not q[0].any() and not q[3].any() and float(qa.a_scale[3]) == 0.0
    assert q[4, :5].tolist() == [127, -63, 2, 0, 1]                    # denormals are not flushed
    assert np.array_equal(q[5], q[1]) and np.array_equal(q[6], -q[1])
    assert q[7, 100] == -127 and int(qa.q_sum[7]) == -127


@pytest.mark.parametrize("bf16", [False, True])
def test_quant_act_strided_and_unaligned_input(dev, ops, bf16):
    # ldx > K, and a base pointer that is only element-aligned: takes the scalar path
    M, K, ldx = 4, 520, 777
    rng = synth.rng_for(123)
    full = synth.activations(rng, M, ldx + 1)
    if bf16:
        bits = synth.to_bf16_bits(full)
        big = _to_dev_bf16(bits, dev)
        view = big.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K]
        ref = oracle.quant_act(np.ascontiguousarray(bits.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K]))
    else:
        big = torch.from_numpy(full).to(dev)
        view = big.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K]
        ref = oracle.quant_act(np.ascontiguousarray(full.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K]))
    qa = ops.quant_act(view)
    _assert_quant_equal(qa, ref, K)


def test_quant_act_batch_mixed_shapes_and_dtypes(dev, ops):
    # one launch: different M, K, dtypes, a strided element-aligned view, a zero row
    rng = synth.rng_for(321)
    specs = [(1, 3200, True), (4, 8640, True), (3, 100, False), (8, 4096, True), (2, 520, False), (1, 64, True),
             (5, 1000, False), (1, 11008, True)]
    xs, refs = [], []
    for i, (M, K, bf16) in enumerate(specs):
        x = synth.activations(rng, M, K, outlier_frac=0.01)
        if i == 2:
            x[1] = 0.0
        if bf16:
            bits = synth.to_bf16_bits(x)
            refs.append(oracle.quant_act(bits))
            xs.append(_to_dev_bf16(bits, dev))
        elif i == 4:   # strided view with an odd offset: the scalar load path
            ldx = 777
            full = np.zeros(M * ldx + 1, np.float32)
            full[1:].reshape(M, ldx)[:, :K] = x
            big = torch.from_numpy(full).to(dev)
            xs.append(big[1:].reshape(M, ldx)[:, :K])
            refs.append(oracle.quant_act(x))
        else:
            refs.append(oracle.quant_act(x))
            xs.append(torch.from_numpy(x).to(dev))
    grp = ops.QuantGroup(xs)
    outs = grp.launch()
    torch.cuda.synchronize()
    for (M, K, _), qa, ref in zip(specs, outs, refs):
        _assert_quant_equal(qa, ref, K)


# ------------------------------------------------------------------ decode product

def _problem(seed, M, K, N, p_zero=None, outl=0.0, bf16=True):
    rng = synth.rng_for(seed)
    w = synth.ternary_weights(rng, N, K, p_zero=p_zero)
    w_scale = synth.draw_w_scale(rng)
    x = synth.activations(rng, M, K, outlier_frac=outl)
    return w, w_scale, (synth.to_bf16_bits(x) if bf16 else x)


def _run_product(ops, dev, kind, w, w_scale, x, waves=None):
    from paper_2410_16144_amd import binding
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(w_scale))
    xd = _to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev)
    qa = ops.quant_act(xd)
    if waves is not None:
        binding.bl_set_tuning("gemv_waves", waves)
    try:
        out, acc = (ops.gemv if kind == "gemv" else ops.gemm)(pw, qa, want_acc=True)
    finally:
        if waves is not None:
            binding.bl_set_tuning("gemv_waves", 0)
    torch.cuda.synchronize()
    return pw, qa, out, acc


def _assert_product(ops, dev, kind, w, w_scale, x, waves=None):
    q_ref, a_ref, s_ref = oracle.quant_act(x)
    acc_ref = oracle.matmul_i32(q_ref, w)
    pw, qa, out, acc = _run_product(ops, dev, kind, w, w_scale, x, waves)
    _assert_quant_equal(qa, (q_ref, a_ref, s_ref), w.shape[1])
    got = acc.cpu().numpy()
    if not np.array_equal(got, acc_ref):
        # say which side moved: the same launch again, the oracle again, the packed weights read back
        bad = np.argwhere(got != acc_ref)
        again = (ops.gemv if kind == "gemv" else ops.gemm)(pw, qa, want_acc=True)[1]
        torch.cuda.synchronize()
        pytest.fail("%s acc: %d of %d elements differ, first at %s (got %d, oracle %d); rows %s cols %s; "
                    "second launch equals first: %s, equals oracle: %s; oracle repeatable: %s; unpack == w: %s"
                    % (kind, len(bad), got.size, bad[0].tolist(), got[tuple(bad[0])], acc_ref[tuple(bad[0])],
                       np.unique(bad[:, 0])[:8].tolist(), np.unique(bad[:, 1])[:8].tolist(),
                       np.array_equal(again.cpu().numpy(), got), np.array_equal(again.cpu().numpy(), acc_ref),
                       np.array_equal(oracle.matmul_i32(q_ref, w), acc_ref),
                       np.array_equal(ops.unpack_ternary(pw).cpu().numpy(), w)))
    _check_out(out, acc_ref, w_scale, a_ref)
    return pw, qa, out, acc


@pytest.fixture
def decode_path():
    """Force the dot-product (1) or matrix-core (2) decode kernel for one test, then restore."""
    from paper_2410_16144_amd import binding

    def force(path):
        binding.bl_set_tuning("decode_path", path)
    yield force
    binding.bl_set_tuning("decode_path", 0)


@pytest.mark.parametrize("path", [0, 1, 2])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_gemv_parity_all_m(dev, ops, decode_path, M, path):
    decode_path(path)
    w, s, x = _problem(500 + M, M, 1536, 320)
    _assert_product(ops, dev, "gemv", w, s, x)


@pytest.mark.parametrize("N,K", [(64, 64), (1, 1), (70, 100), (200, 1000), (1536, 1536), (257, 3200),
                                 (3200, 8640), (129, 64 * 37)])
@pytest.mark.parametrize("M", [1, 4])
def test_gemv_parity_shapes(dev, ops, N, K, M):
    w, s, x = _problem(N * 31 + K + M, M, K, N, p_zero=0.4, outl=0.01)
    _assert_product(ops, dev, "gemv", w, s, x)


@pytest.mark.parametrize("waves", [1, 2, 4, 8, 16])
def test_gemv_parity_every_launch_shape(dev, ops, waves):
    w, s, x = _problem(900 + waves, 2, 64 * 37, 192)
    _assert_product(ops, dev, "gemv", w, s, x, waves=waves)
    w, s, x = _problem(901 + waves, 1, 64 * 3, 128)      # fewer K tiles than waves
    _assert_product(ops, dev, "gemv", w, s, x, waves=waves)


def test_gemv_fp32_activations_config1(dev, ops):
    # config 1: M=1, K=N=1536, uniform ternary, scale 0.02, fp32 N(0,1), seed 0
    rng = synth.rng_for(synth.seed_for(1))
    w = synth.ternary_weights(rng, 1536, 1536)
    x = synth.activations(rng, 1, 1536)
    _assert_product(ops, dev, "gemv", w, np.float32(0.02), x)


def test_gemv_invariants_and_determinism(dev, ops):
    w, s, x = _problem(42, 3, 1024, 256)
    pw, qa, out, acc = _run_product(ops, dev, "gemv", w, s, x)
    for _ in range(3):
        _, _, out2, acc2 = _run_product(ops, dev, "gemv", w, s, x)
        assert torch.equal(acc, acc2) and torch.equal(out, out2)
    _, _, outn, accn = _run_product(ops, dev, "gemv", -w, s, x)
    assert torch.equal(accn, -acc) and torch.equal(outn, -out)
    _, _, outz, accz = _run_product(ops, dev, "gemv", np.zeros_like(w), s, x)
    assert not accz.any() and not outz.any()
    xz = np.zeros_like(x)
    _, qz, outz, accz = _run_product(ops, dev, "gemv", w, s, xz)
    assert not qz.q.any() and not outz.any() and not accz.any()
    ones = np.ones_like(w)
    _, qa1, _, acc1 = _run_product(ops, dev, "gemv", ones, s, x)
    assert torch.equal(acc1, qa1.q_sum[:, None].expand(-1, w.shape[0]))


def test_gemv_batch_equals_separate_calls(dev, ops):
    shapes = [(320, 640), (320, 640), (128, 640), (640, 320), (64, 64), (200, 1000), (1000, 200)]
    M = 2
    weights, acts, refs = [], [], []
    for i, (N, K) in enumerate(shapes):
        w, s, x = _problem(700 + i, M, K, N)
        pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(s))
        qa = ops.quant_act(_to_dev_bf16(x, dev))
        weights.append(pw)
        acts.append(qa)
        refs.append(ops.gemv(pw, qa, want_acc=True))
    grp = ops.GemvGroup(weights, acts, want_acc=True)
    outs = grp.launch()
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        assert torch.equal(outs[i], refs[i][0]) and torch.equal(grp.accs[i], refs[i][1])
        q_ref = acts[i].q.cpu().numpy()[:, :shapes[i][1]]
        w_ref = ops.unpack_ternary(weights[i]).cpu().numpy()
        assert np.array_equal(grp.accs[i].cpu().numpy(), oracle.matmul_i32(np.ascontiguousarray(q_ref), w_ref))


def test_decode_at_the_largest_k(dev, ops):
    """K at the ABI's limit (2^20): one row block of 16384 tiles; the longest int32 sums the library allows.
    One token with a workspace (the row block is shared by every workgroup of the balanced launch), one token
    without, and two tokens on the matrix cores."""
    from paper_2410_16144_amd import binding
    K, N = binding.BL_MAX_K, 70
    rng = synth.rng_for(3300)
    w = synth.ternary_weights(rng, N, K)
    w[0] = 1            # |acc| as large as it gets: sum |q|
    w[1] = -1
    x = synth.activations(rng, 2, K)
    x[0] = np.abs(x[0]) + 1.0
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), 0.02)
    for M, use_ws in ((1, True), (1, False), (2, True)):
        xd = torch.from_numpy(np.ascontiguousarray(x[:M])).to(dev)
        qa = ops.quant_act(xd)
        grp = ops.GemvGroup([pw], [qa], want_acc=True, use_workspace=use_ws)
        grp.launch()
        torch.cuda.synchronize()
        q_ref, a_ref, s_ref = oracle.quant_act(np.ascontiguousarray(x[:M]))
        _assert_quant_equal(qa, (q_ref, a_ref, s_ref), K)
        acc_ref = oracle.matmul_i32(q_ref, w)
        assert np.array_equal(grp.accs[0].cpu().numpy(), acc_ref)
        assert abs(int(acc_ref[0, 0])) > 2 ** 24     # beyond exact fp32 integers: out still within tolerance
        _check_out(grp.outs[0], acc_ref, np.float32(0.02), a_ref)
    assert not ops.workspace(dev).any()


# ------------------------------------------------------------------ fused decode

def _assert_fused(ops, dev, problems, M):
    """problems: list of (w, w_scale, x) with x either fp32 or bf16 bits; all with the same M."""
    weights, xs = [], []
    for w, s, x in problems:
        weights.append(ops.pack_ternary(torch.from_numpy(w).to(dev), float(s)))
        xs.append(_to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev))
    grp = ops.DecodeGroup(weights, xs, want_acc=True, want_quant=True)
    outs = grp.launch()
    torch.cuda.synchronize()
    for i, (w, s, x) in enumerate(problems):
        q_ref, a_ref, s_ref = oracle.quant_act(x)
        _assert_quant_equal(grp.quants[i], (q_ref, a_ref, s_ref), w.shape[1])
        acc_ref = oracle.matmul_i32(q_ref, w)
        assert np.array_equal(grp.accs[i].cpu().numpy(), acc_ref)
        _check_out(outs[i], acc_ref, s, a_ref)
    return grp


@pytest.mark.parametrize("path", [0, 1, 2])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_fused_decode_parity_all_m(dev, ops, decode_path, M, path):
    decode_path(path)
    _assert_fused(ops, dev, [_problem(1500 + M, M, 1536, 320, outl=0.01)], M)


@pytest.mark.parametrize("stage", [0, 1])
@pytest.mark.parametrize("M", [2, 8])
@pytest.mark.parametrize("N,K", [(70, 100), (200, 1000), (4096, 11008), (129, 64 * 37)])
def test_matrix_core_decode_shapes(dev, ops, N, K, M, stage):
    # stage 0: activations copied into LDS when they fit (M*Kp <= 64 KiB), else fetched per tile;
    # stage 1: always fetched per tile
    from paper_2410_16144_amd import binding
    binding.bl_set_tuning("decode_stage", stage)
    try:
        prob = _problem(N * 19 + K + M, M, K, N, p_zero=0.4, outl=0.01)
        _assert_product(ops, dev, "gemv", *prob)
        if stage == 0:
            _assert_fused(ops, dev, [prob], M)
    finally:
        binding.bl_set_tuning("decode_stage", 0)


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("N,K", [(64, 64), (1, 1), (70, 100), (200, 1000), (257, 3200), (3200, 8640), (129, 64 * 37),
                                 (192, 33792)])
def test_fused_decode_parity_shapes(dev, ops, N, K, bf16):
    _assert_fused(ops, dev, [_problem(N * 17 + K, 1, K, N, p_zero=0.4, outl=0.01, bf16=bf16)], 1)


def test_fused_decode_batch_of_seven_mixed_shapes(dev, ops):
    shapes = [(320, 640), (320, 640), (128, 640), (640, 320), (64, 64), (200, 1000), (1000, 200)]
    for M in (1, 3):
        _assert_fused(ops, dev, [_problem(1700 + i + M, M, K, N, outl=0.01) for i, (N, K) in enumerate(shapes)], M)


def test_fused_decode_edge_rows_and_strided_input(dev, ops):
    K, N, M = 520, 130, 4
    rng = synth.rng_for(1800)
    w = synth.ternary_weights(rng, N, K)
    x = np.zeros((M, K), np.float32)
    x[1] = rng.standard_normal(K).astype(np.float32)
    x[2, :8] = [127.0, 62.5, -61.5, 0.5, 1.5, 2.5, -0.5, -2.5]
    x[3] = 1e-38
    _assert_fused(ops, dev, [(w, np.float32(0.03), x)], M)
    # strided, only element-aligned input: the scalar load path
    ldx = 777
    full = synth.activations(rng, M, ldx + 1)
    big = torch.from_numpy(full).to(dev)
    view = big.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K]
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), 0.03)
    grp = ops.DecodeGroup([pw], [view], want_acc=True, want_quant=True)
    grp.launch()
    torch.cuda.synchronize()
    xh = np.ascontiguousarray(full.reshape(-1)[1:1 + M * ldx].reshape(M, ldx)[:, :K])
    q_ref, a_ref, s_ref = oracle.quant_act(xh)
    _assert_quant_equal(grp.quants[0], (q_ref, a_ref, s_ref), K)
    assert np.array_equal(grp.accs[0].cpu().numpy(), oracle.matmul_i32(q_ref, w))


def test_fused_decode_equals_two_call_sequence(dev, ops):
    w, s, x = _problem(1900, 2, 2048, 512, outl=0.01)
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(s))
    xd = _to_dev_bf16(x, dev)
    qa = ops.quant_act(xd)
    out2, acc2 = ops.gemv(pw, qa, want_acc=True)
    grp = ops.DecodeGroup([pw], [xd], want_acc=True, want_quant=True)
    out1 = grp.launch()[0]
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(grp.accs[0], acc2)
    assert torch.equal(grp.quants[0].q, qa.q) and torch.equal(grp.quants[0].a_scale, qa.a_scale)
    assert torch.equal(grp.quants[0].q_sum, qa.q_sum)


@pytest.mark.parametrize("publish", [0, -1])
@pytest.mark.parametrize("M", [2, 3, 4, 5, 6, 7, 8])
def test_fused_decode_publishing_and_requantizing_forms(dev, ops, M, publish):
    """Fused launches of 2..8 tokens: with a workspace and quantization buffers every distinct input is quantized once
    by a leading workgroup and published (publish = 0); otherwise, or when forbidden (publish = -1), every workgroup
    quantizes for itself.  Both against the oracle, a batch of mixed shapes (one long-K problem that is fetched per
    tile at M = 8), and the workspace -- counters and status word included -- all zero afterwards."""
    from paper_2410_16144_amd import binding
    shapes = [(320, 640), (128, 640), (640, 320), (200, 1000), (1000, 200), (192, 64 * 131)]
    binding.bl_set_tuning("decode_publish", publish)
    try:
        _assert_fused(ops, dev, [_problem(6100 + i + M, M, K, N, outl=0.01) for i, (N, K) in enumerate(shapes)], M)
        name = binding.bl_last_kernel()
        assert name.startswith("decode_mfma_kernel<%d, " % M)
        assert (name.split(" grid=")[0].count(",") == 4) == (publish == 0), name     # the publishing form's name has a fifth argument
    finally:
        binding.bl_set_tuning("decode_publish", 0)
    assert not ops.workspace(dev).any()


def test_fused_decode_publishing_shared_inputs_like_a_layer(dev, ops):
    """Seven products on four inputs, as a decoder layer has them, M = 4 and 8: without quantization outputs the binding
    hands over one set of buffers per distinct input, so four inputs are quantized, not seven; results equal the
    quantize-then-multiply sequence bit for bit, launch after launch."""
    from paper_2410_16144_amd import binding
    from paper_2410_16144_amd.decode_layer import INPUT_OF, make_layer
    for M in (4, 8):
        layer, host = make_layer(3, 0, 1024, 2752, M, dev, None, 0.0, host=True)
        for rep in range(3):
            for o in layer.outs:
                o.zero_()
            layer.step_fused()
            name = binding.bl_last_kernel()
            torch.cuda.synchronize()
            assert name.split(" grid=")[0].count(",") == 4, name
            fused = [o.clone() for o in layer.outs]
            layer.step_two_launches()
            torch.cuda.synchronize()
            for a, b_ in zip(fused, layer.outs):
                assert torch.equal(a, b_)
        refs_q = [oracle.quant_act(b_) for b_ in host["x_bits"]]
        for i, p in enumerate(layer.projs):
            q, a, s = refs_q[INPUT_OF[p.name]]
            _check_out(fused[i], oracle.matmul_i32(q, host["w"][i]), host["w_scale"][i], a)
        assert len({id(q) for q in layer.fused_all.published}) == 4
    assert not ops.workspace(dev).any()


def test_fused_decode_publishing_wait_gives_up_and_every_kernel_exits(dev, ops):
    """The waiters' polls are bounded.  With the limit forced down to one poll from the host they give up long before the
    quantizers have published: the launch must still end (every wave reaches the exit), must say so in the status
    word, and the same buffers must serve a correct launch once the workspace has been zeroed again."""
    from paper_2410_16144_amd import binding
    M = 4
    probs = [_problem(6200 + i, M, K, N, outl=0.01) for i, (N, K) in enumerate([(2048, 4096), (1024, 4096), (4096, 2048)])]
    weights = [ops.pack_ternary(torch.from_numpy(w).to(dev), float(s)) for w, s, x in probs]
    xs = [_to_dev_bf16(x, dev) for w, s, x in probs]
    ws = torch.zeros(binding.BL_WORKSPACE_BYTES, dtype=torch.uint8, device=dev)
    grp = ops.DecodeGroup(weights, xs, want_acc=True, want_quant=True, use_workspace=ws)
    binding.bl_set_tuning("decode_wait_limit", 1)
    try:
        grp.launch()
        torch.cuda.synchronize()            # returns: nobody is left waiting
    finally:
        binding.bl_set_tuning("decode_wait_limit", 0)
    words = ws.view(torch.int32)
    assert int(words[-64]) == 1, "a waiter that gave up must leave the status word (the workspace's last 256 bytes) set"
    ws.zero_()
    grp.launch()
    torch.cuda.synchronize()
    for i, (w, s, x) in enumerate(probs):
        q_ref, a_ref, s_ref = oracle.quant_act(x)
        _assert_quant_equal(grp.quants[i], (q_ref, a_ref, s_ref), w.shape[1])
        assert np.array_equal(grp.accs[i].cpu().numpy(), oracle.matmul_i32(q_ref, w))
    assert not ws.any()


# ------------------------------------------------------------------ work-balanced decode (workspace)

@pytest.fixture
def decode_split():
    """Force the work-balanced one-token launch with n workgroups per compute unit, then restore."""
    from paper_2410_16144_amd import binding

    def force(n):
        binding.bl_set_tuning("decode_split", n)
    yield force
    binding.bl_set_tuning("decode_split", 0)


def _assert_split(ops, dev, problems, expect_split):
    """Plain and fused one-token launches with a workspace against the oracle; the workspace must be
    all zero again afterwards, and a second launch on the same workspace must give the same bits."""
    from paper_2410_16144_amd import binding
    ws = ops.workspace(dev)
    assert not ws.any()
    weights, xs, acts = [], [], []
    for w, s, x in problems:
        weights.append(ops.pack_ternary(torch.from_numpy(w).to(dev), float(s)))
        xs.append(_to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev))
        acts.append(ops.quant_act(xs[-1]))
    before = binding.bl_get_stat("split_launches")
    plain = ops.GemvGroup(weights, acts, want_acc=True)
    plain.launch()
    fused = ops.DecodeGroup(weights, xs, want_acc=True, want_quant=True)
    fused.launch()
    torch.cuda.synchronize()
    assert binding.bl_get_stat("split_launches") - before == (2 if expect_split else 0)
    assert not ws.any()
    for i, (w, s, x) in enumerate(problems):
        q_ref, a_ref, s_ref = oracle.quant_act(x)
        acc_ref = oracle.matmul_i32(q_ref, w)
        _assert_quant_equal(fused.quants[i], (q_ref, a_ref, s_ref), w.shape[1])
        for grp in (plain, fused):
            assert np.array_equal(grp.accs[i].cpu().numpy(), acc_ref)
            _check_out(grp.outs[i], acc_ref, s, a_ref)
    first = [o.clone() for o in fused.outs]
    for o in fused.outs:
        o.zero_()
    fused.launch()
    fused.launch()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(first, fused.outs)) and not ws.any()
    # without a workspace: the row-block kernels, same bits
    nows = ops.DecodeGroup(weights, xs, use_workspace=False)
    nows.launch()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(first, nows.outs))


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("n,N,K", [(1, 4100, 8200),     # every row block shared by about four workgroups
                                   (1, 33000, 1100),    # short rows: whole row blocks inside a chunk
                                   (2, 8200, 8200),
                                   (1, 321, 64 * 1800)])  # 6 row blocks, each spread over about 42 workgroups
def test_split_decode_single_matrix(dev, ops, decode_split, n, N, K, bf16):
    decode_split(n)
    _assert_split(ops, dev, [_problem(N + 3 * K + n, 1, K, N, p_zero=0.4, outl=0.01, bf16=bf16)], True)


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("N,K", [(8197, 1016), (8200, 1024), (8200, 1032),   # one wave holds the row / just not
                                 (4100, 2056), (1300, 8192 + 8),            # 3 and 9 holding waves
                                 (700, 16384),                              # all 16 waves hold it, both vectors full
                                 (700, 16384 + 8)])                         # one vector too long: the two-pass quantizer
def test_fused_decode_row_holder_boundaries(dev, ops, decode_split, N, K, bf16):
    # the fused one-token kernels keep the token row in the registers of as few leading waves as can hold it;
    # the cases sit on both sides of every change in that number, in the balanced and (inside _assert_split, without
    # a workspace) the row-block kernel
    decode_split(1)
    _assert_split(ops, dev, [_problem(3 * N + K, 1, K, N, p_zero=0.4, outl=0.01, bf16=bf16)], True)


@pytest.mark.parametrize("n", [1, 2])
def test_split_decode_batch_mixed_shapes(dev, ops, decode_split, n):
    decode_split(n)
    shapes = [(2000, 4000), (1000, 9000), (5000, 3000), (700, 6000), (64, 64), (2000, 4000), (130, 12000)]
    scale = 2 if n == 2 else 1
    _assert_split(ops, dev, [_problem(2100 + i, 1, K, N * scale, outl=0.01) for i, (N, K) in enumerate(shapes)], True)


def test_split_decode_falls_back_when_it_does_not_apply(dev, ops, decode_split):
    decode_split(1)
    # K = 64: a chunk would touch more row blocks than the kernel keeps partial sums for
    _assert_split(ops, dev, [_problem(2200, 1, 64, 64 * 9000)], False)
    # too small to be worth balancing
    _assert_split(ops, dev, [_problem(2201, 1, 1536, 1536)], False)
    decode_split(-1)
    _assert_split(ops, dev, [_problem(2202, 1, 8200, 4100)], False)


def test_split_decode_layer_shape_automatic(dev, ops):
    # a 3B-shape layer (Appendix A structure) is in the range where the automatic choice balances
    from paper_2410_16144_amd import binding
    projs = synth.layer_projections(3200, 8640)
    problems = [_problem(2300 + i, 1, p.K, p.N, p_zero=0.4, outl=0.01) for i, p in enumerate(projs)]
    _assert_split(ops, dev, problems, True)


@pytest.mark.parametrize("stream", [-1, 1])
def test_decode_streaming_and_ordinary_weight_loads_agree(dev, ops, stream):
    """The decode kernels exist in two forms that differ only in how weight tiles are loaded (streaming loads for large
    launches, ordinary loads for small ones): forcing either form on launches of both sizes must not change a bit --
    row-block kernel, matrix-core kernel, work-balanced kernel, fused and plain."""
    from paper_2410_16144_amd import binding
    problems = [_problem(2400 + i, M, K, N, p_zero=0.4, outl=0.01) for i, (M, K, N) in
                enumerate(((1, 1536, 704), (1, 4096, 2048), (4, 1000, 330), (8, 2048, 512), (1, 8640, 3200)))]
    ref = [_run_product(ops, dev, "gemv", w, s, x) for w, s, x in problems]
    binding.bl_set_tuning("decode_stream", stream)
    try:
        for (w, s, x), r in zip(problems, ref):
            got = _run_product(ops, dev, "gemv", w, s, x)
            assert torch.equal(got[2], r[2]) and torch.equal(got[3], r[3])
            name = binding.bl_last_kernel()
            assert ("true>" if stream > 0 else "false>") in name.split(" grid=")[0][-8:], name
            _assert_product(ops, dev, "gemv", w, s, x)
        w, s, x = problems[4]
        pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(s))
        xd = _to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev)
        grp = ops.DecodeGroup([pw, pw], [xd, xd], want_acc=True)
        grp.launch()
        torch.cuda.synchronize()
        assert torch.equal(grp.accs[0], ref[4][3]) and torch.equal(grp.outs[1], ref[4][2])
    finally:
        binding.bl_set_tuning("decode_stream", 0)


# ------------------------------------------------------------------ prefill product

@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (7, 70, 100), (33, 200, 1000), (128, 256, 512), (130, 320, 1536),
                                   (300, 1000, 832), (512, 192, 4096)])
def test_gemm_parity(dev, ops, M, N, K):
    w, s, x = _problem(M * 13 + N + K, M, K, N, p_zero=0.4, outl=0.01)
    _assert_product(ops, dev, "gemm", w, s, x)


@pytest.mark.parametrize("tile", [12, 14, 22, 23, 24, 122, 124])
def test_gemm_parity_every_wave_tile(dev, ops, tile):
    from paper_2410_16144_amd import binding
    binding.bl_set_tuning("gemm_mb", tile)
    try:
        for M, N, K in ((200, 1000, 832), (33, 200, 1000), (257, 704, 64 * 5), (70, 600, 64 * 31)):
            w, s, x = _problem(M * 11 + N + K + tile, M, K, N, p_zero=0.4, outl=0.01)
            _assert_product(ops, dev, "gemm", w, s, x)
    finally:
        binding.bl_set_tuning("gemm_mb", 0)


def test_gemm_long_k(dev, ops):
    M, N, K = 70, 130, 65536 + 64     # 1025 K steps (odd: the K-split form pads one group), ragged M and N
    w, s, x = _problem(3200, M, K, N, p_zero=0.4, outl=0.01)
    _assert_product(ops, dev, "gemm", w, s, x)


def test_gemm_many_token_tiles(dev, ops):
    # more token tiles than a 16-bit grid dimension could index, ragged in every direction
    M, N, K = 66000 + 7, 70, 100
    w, s, x = _problem(3100, M, K, N, p_zero=0.4)
    _assert_product(ops, dev, "gemm", w, s, x)


def test_gemm_equals_gemv_for_small_m(dev, ops):
    w, s, x = _problem(4242, 8, 1536, 448)
    _, _, out_v, acc_v = _run_product(ops, dev, "gemv", w, s, x)
    _, _, out_m, acc_m = _run_product(ops, dev, "gemm", w, s, x)
    assert torch.equal(acc_v, acc_m) and torch.equal(out_v, out_m)


def test_gemm_determinism(dev, ops):
    w, s, x = _problem(4243, 200, 1024, 320)
    _, _, out, acc = _run_product(ops, dev, "gemm", w, s, x)
    for _ in range(2):
        _, _, out2, acc2 = _run_product(ops, dev, "gemm", w, s, x)
        assert torch.equal(acc, acc2) and torch.equal(out, out2)


@pytest.mark.parametrize("tile", [0, 12, 14, 22, 23, 24, 122, 124])
def test_gemm_batch_parity(dev, ops, tile):
    """Several products over the same activations in one launch: int32 sums equal to the oracle's, outputs and sums
    bit for bit those of separate bl_gemm calls -- products of different N (ragged, one below a workgroup's rows), the
    batch's ends, every wave tile."""
    from paper_2410_16144_amd import binding
    M, K = 150, 832
    ns = [1000, 70, 704, 330]
    x = _problem(5100 + tile, M, K, 64)[2]
    qa = ops.quant_act(_to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev))
    q_ref, a_ref, _ = oracle.quant_act(x)
    ws = [_problem(5200 + tile + i, 1, K, n, p_zero=0.4, outl=0.01)[:2] for i, n in enumerate(ns)]
    pws = [ops.pack_ternary(torch.from_numpy(w).to(dev), float(s)) for w, s in ws]
    binding.bl_set_tuning("gemm_mb", tile)
    try:
        for count in (4, 2, 1):
            outs = [torch.empty((M, pw.N), device=dev) for pw in pws[:count]]
            accs = [torch.empty((M, pw.N), dtype=torch.int32, device=dev) for pw in pws[:count]]
            binding.bl_gemm_batch([(pw.blob.data_ptr(), pw.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), qa.q_sum.data_ptr(),
                                    o.data_ptr(), a.data_ptr()) for pw, o, a in zip(pws, outs, accs)], M,
                                  torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            for (w, s), pw, o, a in zip(ws, pws, outs, accs):
                acc_ref = oracle.matmul_i32(q_ref, w)
                assert np.array_equal(a.cpu().numpy(), acc_ref)
                _check_out(o, acc_ref, s, a_ref)
                o1, a1 = ops.gemm(pw, qa, want_acc=True)
                assert torch.equal(o, o1) and torch.equal(a, a1)
    finally:
        binding.bl_set_tuning("gemm_mb", 0)
    outs = ops.gemm_batch(pws[:3], qa)
    assert all(torch.equal(o, ops.gemm(pw, qa)) for o, pw in zip(outs, pws))


def _launch_gemm(ops, pw, qa, out, acc):
    from paper_2410_16144_amd import binding
    binding.bl_gemm(pw.blob.data_ptr(), pw.desc, qa.q.data_ptr(), qa.a_scale.data_ptr(), qa.q_sum.data_ptr(),
                    qa.q.shape[0], out.data_ptr(), acc.data_ptr(), torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("K", [192, 64 * 30])
@pytest.mark.parametrize("tile", [12, 14, 22, 23, 24, 122, 124])
def test_gemm_first_steps_under_load(dev, ops, tile, K):
    """Short K and enough workgroups to keep every compute unit's load queue busy, launched back to back: every launch
    must give the oracle's bits.  K = 192: the whole product is the kernel's first three steps (the waits of the
    activation ring's first stages, whose margin is the smallest when the memory system is busy).  K = 1920: 30 steps
    (15 with two K groups), i.e. three whole trips of the unrolled loop and a tail of six or seven steps, whose waits
    count requests only."""
    from paper_2410_16144_amd import binding
    M, N = 1024, 2048                  # 128 to 1024 workgroups depending on the tile
    w, s, x = _problem(5000 + tile + K, M, K, N, p_zero=0.4, outl=0.01)
    q_ref, a_ref, s_ref = oracle.quant_act(x)
    acc_ref = torch.from_numpy(oracle.matmul_i32(q_ref, w)).to(dev)
    pw = ops.pack_ternary(torch.from_numpy(w).to(dev), float(s))
    qa = ops.quant_act(_to_dev_bf16(x, dev) if x.dtype == np.uint16 else torch.from_numpy(x).to(dev))
    outs = [torch.empty((M, N), dtype=torch.float32, device=dev) for _ in range(8)]
    accs = [torch.empty((M, N), dtype=torch.int32, device=dev) for _ in range(8)]
    binding.bl_set_tuning("gemm_mb", tile)
    try:
        for rep in range(25 if K < 1000 else 8):
            for o, a in zip(outs, accs):
                _launch_gemm(ops, pw, qa, o, a)
            torch.cuda.synchronize()
            for i, a in enumerate(accs):
                assert torch.equal(a, acc_ref), "launch %d of round %d differs from the oracle" % (i, rep)
    finally:
        binding.bl_set_tuning("gemm_mb", 0)

