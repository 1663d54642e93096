"""Host-side logic of the C ABI: exported symbols, descriptor arithmetic and argument
validation.  No kernel is launched (validation runs before any HIP call), so this runs on a
machine without a GPU.
"""
import ctypes
import os
import re

import pytest

from paper_2410_16144_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bl_[a-z0-9_]+)\s*\(", body))
    assert declared == set(B.DECLARED_SYMBOLS)
    lib = B.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert "gfx950" in B.version()


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.PackedDesc) == 56
    assert B.PackedDesc.bytes.offset == 40 and B.PackedDesc.w_scale.offset == 48
    assert ctypes.sizeof(B.GemvItem) == 56
    assert ctypes.sizeof(B.QuantItem) == 64 and B.QuantItem.q_dev.offset == 40
    assert ctypes.sizeof(B.DecodeItem) == 80 and B.DecodeItem.packed_dev.offset == 24
    assert ctypes.sizeof(B.NormQuantArgs) == 112 and B.NormQuantArgs.eps.offset == 56 and B.NormQuantArgs.q_dev.offset == 64
    assert ctypes.sizeof(B.AttnArgs) == 88 and B.AttnArgs.n_heads.offset == 72
    assert ctypes.sizeof(B.DecodeNormItem) == 128 and B.DecodeNormItem.packed_dev.offset == 40 and B.DecodeNormItem.glu_gamma_dev.offset == 112


def test_padding_and_descriptor():
    assert B.bl_padded_k(1) == 64 and B.bl_padded_k(64) == 64 and B.bl_padded_k(65) == 128
    assert B.bl_padded_k(0) == -1 and B.bl_padded_k(B.BL_MAX_K + 1) == -1 and B.bl_padded_k(B.BL_MAX_K) == B.BL_MAX_K
    assert B.bl_padded_n(1) == 64 and B.bl_padded_n(8640) == 8640 and B.bl_padded_n(0) == -1
    d = B.bl_packed_desc_init(3200, 8640, 0.02)
    assert (d.version, d.N, d.K, d.Np, d.Kp, d.bytes) == (1, 3200, 8640, 3200, 8640, 3200 * 8640 // 4)
    d = B.bl_packed_desc_init(70, 100, 1.0)
    assert (d.Np, d.Kp, d.bytes) == (128, 128, 128 * 128 // 4)
    for n, k in ((0, 64), (64, 0), (-1, 5), (5, B.BL_MAX_K + 1)):
        with pytest.raises(B.BitLinearError) as e:
            B.bl_packed_desc_init(n, k, 1.0)
        assert e.value.status == B.BL_ERR_SHAPE


def _st(fn, *a):
    with pytest.raises(B.BitLinearError) as e:
        fn(*a)
    return e.value.status


def test_argument_validation_happens_before_any_launch():
    d = B.bl_packed_desc_init(128, 128, 0.5)
    P = 0x10000  # a fake, well-aligned "device pointer": never dereferenced because validation fails first
    # nulls
    assert _st(B.bl_pack_ternary, 0, d, P) == B.BL_ERR_NULL
    assert _st(B.bl_pack_ternary, P, d, 0) == B.BL_ERR_NULL
    assert _st(B.bl_unpack_ternary, 0, d, P) == B.BL_ERR_NULL
    assert _st(B.bl_quant_act, 0, B.BL_F32, 1, 128, 128, P, P, P) == B.BL_ERR_NULL
    assert _st(B.bl_gemv, P, d, P, P, 0, 1, P) == B.BL_ERR_NULL          # q_sum is required
    assert _st(B.bl_gemm, P, d, 0, P, P, 1, P) == B.BL_ERR_NULL
    # M range
    assert _st(B.bl_gemv, P, d, P, P, P, 9, P) == B.BL_ERR_M_RANGE
    assert _st(B.bl_gemv, P, d, P, P, P, 0, P) == B.BL_ERR_M_RANGE
    assert _st(B.bl_gemm, P, d, P, P, P, 0, P) == B.BL_ERR_SHAPE
    assert _st(B.bl_gemm, P, d, P, P, P, B.BL_MAX_GEMM_M + 1, P) == B.BL_ERR_SHAPE
    # alignment
    assert _st(B.bl_pack_ternary, P, d, P + 4) == B.BL_ERR_ALIGN
    assert _st(B.bl_gemv, P + 8, d, P, P, P, 1, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_gemv, P, d, P + 4, P, P, 1, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_gemv, P, d, P, P + 2, P, 1, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_quant_act, P + 2, B.BL_F32, 1, 128, 128, P, P, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_quant_act, P + 1, B.BL_BF16, 1, 128, 128, P, P, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_quant_act, P, B.BL_F32, 1, 128, 128, P + 8, P, P) == B.BL_ERR_ALIGN
    # dtype / shapes
    assert _st(B.bl_quant_act, P, 7, 1, 128, 128, P, P, P) == B.BL_ERR_DTYPE
    assert _st(B.bl_quant_act, P, B.BL_F32, 0, 128, 128, P, P, P) == B.BL_ERR_SHAPE
    assert _st(B.bl_quant_act, P, B.BL_F32, 1, 128, 100, P, P, P) == B.BL_ERR_SHAPE   # ldx < K
    assert _st(B.bl_quant_act, P, B.BL_F32, 1, 0, 0, P, P, P) == B.BL_ERR_SHAPE
    # descriptor tampering
    bad = B.bl_packed_desc_init(128, 128, 0.5)
    bad.version = 2
    assert _st(B.bl_gemv, P, bad, P, P, P, 1, P) == B.BL_ERR_LAYOUT
    bad = B.bl_packed_desc_init(128, 128, 0.5)
    bad.bytes -= 1
    assert _st(B.bl_pack_ternary, P, bad, P) == B.BL_ERR_BUF_SMALL
    bad = B.bl_packed_desc_init(128, 128, 0.5)
    bad.Kp = 192
    assert _st(B.bl_gemm, P, bad, P, P, P, 1, P) == B.BL_ERR_SHAPE
    # the gated form's packer: both matrices, 2 F rows with F a multiple of 32
    assert _st(B.bl_pack_gate_up, P, 0, d, P) == B.BL_ERR_NULL
    assert _st(B.bl_pack_gate_up, P, P, B.bl_packed_desc_init(96, 128, 0.5), P) == B.BL_ERR_SHAPE
    assert _st(B.bl_pack_gate_up, P, P, d, P + 8) == B.BL_ERR_ALIGN
    # the static-workspace variant validates like bl_gemv_batch, before it touches the device
    items = B.make_gemv_items([(P, d, P, P, P, P, 0)])
    assert B.lib().bl_gemv_batch_static(items, 0, 1, None) == B.BL_ERR_COUNT
    assert B.lib().bl_gemv_batch_static(items, 1, 9, None) == B.BL_ERR_M_RANGE
    assert B.lib().bl_gemv_batch_static(None, 1, 1, None) == B.BL_ERR_NULL
    assert B.lib().bl_gemv_batch_static(B.make_gemv_items([(P, d, P + 4, P, P, P, 0)]), 1, 1, None) == B.BL_ERR_ALIGN
    assert B.status_str(B.BL_ERR_WORKSPACE) != B.status_str(99)
    # batch count
    items = B.make_gemv_items([(P, d, P, P, P, P, 0)])
    assert B.lib().bl_gemv_batch(items, 0, 1, None, None) == B.BL_ERR_COUNT
    assert B.lib().bl_gemv_batch(items, 9, 1, None, None) == B.BL_ERR_COUNT
    assert B.lib().bl_gemv_batch(None, 1, 1, None, None) == B.BL_ERR_NULL
    assert B.lib().bl_gemm_batch(items, 0, 1, None) == B.BL_ERR_COUNT
    assert B.lib().bl_gemm_batch(items, B.BL_MAX_GEMM_BATCH + 1, 1, None) == B.BL_ERR_COUNT
    assert B.lib().bl_gemm_batch(None, 1, 1, None) == B.BL_ERR_NULL
    assert B.lib().bl_gemm_batch(items, 1, 0, None) == B.BL_ERR_SHAPE
    assert B.lib().bl_gemm_batch(items, 1, B.BL_MAX_GEMM_M + 1, None) == B.BL_ERR_SHAPE
    assert B.lib().bl_gemm_batch(B.make_gemv_items([(P, d, P, P, P, P, 0), (P, d, 0, P, P, P, 0)]), 2, 1, None) == B.BL_ERR_NULL
    assert B.lib().bl_gemm_batch(B.make_gemv_items([(P, d, P, P, P, P, 0), (P + 8, d, P, P, P, P, 0)]), 2, 1, None) == B.BL_ERR_ALIGN
    # fused decode
    ditems = B.make_decode_items([(P, B.BL_BF16, 128, P, d, P, 0, 0, 0, 0)])
    lib = B.lib()
    assert lib.bl_decode_batch(ditems, 1, 9, None, None) == B.BL_ERR_M_RANGE
    assert lib.bl_decode_batch(ditems, 0, 1, None, None) == B.BL_ERR_COUNT
    assert lib.bl_decode_batch(None, 1, 1, None, None) == B.BL_ERR_NULL
    assert lib.bl_decode_batch(B.make_decode_items([(0, B.BL_BF16, 128, P, d, P, 0, 0, 0, 0)]), 1, 1, None, None) == B.BL_ERR_NULL
    assert lib.bl_decode_batch(B.make_decode_items([(P, 5, 128, P, d, P, 0, 0, 0, 0)]), 1, 1, None, None) == B.BL_ERR_DTYPE
    assert lib.bl_decode_batch(B.make_decode_items([(P, B.BL_BF16, 64, P, d, P, 0, 0, 0, 0)]), 1, 1, None, None) == B.BL_ERR_SHAPE
    assert lib.bl_decode_batch(B.make_decode_items([(P + 1, B.BL_BF16, 128, P, d, P, 0, 0, 0, 0)]), 1, 1, None, None) == B.BL_ERR_ALIGN
    big = B.bl_packed_desc_init(64, 65536, 1.0)    # 8 tokens x 64 KiB of activations exceed on-chip memory
    assert lib.bl_decode_batch(B.make_decode_items([(P, B.BL_BF16, 65536, P, big, P, 0, 0, 0, 0)]), 1, 8, None, None) == B.BL_ERR_SHAPE
    # grouped quantization
    qitems = B.make_quant_items([(P, B.BL_BF16, 1, 128, 128, P, P, P)])
    assert lib.bl_quant_act_batch(qitems, 0, None) == B.BL_ERR_COUNT
    assert lib.bl_quant_act_batch(qitems, 9, None) == B.BL_ERR_COUNT
    assert lib.bl_quant_act_batch(None, 1, None) == B.BL_ERR_NULL
    assert lib.bl_quant_act_batch(B.make_quant_items([(P, B.BL_BF16, 1, 128, 64, P, P, P)]), 1, None) == B.BL_ERR_SHAPE
    assert lib.bl_quant_act_batch(B.make_quant_items([(P, 7, 1, 128, 128, P, P, P)]), 1, None) == B.BL_ERR_DTYPE
    assert lib.bl_quant_act_batch(B.make_quant_items([(P, B.BL_BF16, 1, 128, 128, P + 8, P, P)]), 1, None) == B.BL_ERR_ALIGN
    # workspace alignment
    assert B.lib().bl_gemv_batch(items, 1, 1, P + 64, None) == B.BL_ERR_ALIGN
    assert lib.bl_decode_batch(ditems, 1, 1, P + 16, None) == B.BL_ERR_ALIGN
    # tuning hook
    assert _st(B.bl_set_tuning, "decode_split", 9) == B.BL_ERR_SHAPE
    assert _st(B.bl_set_tuning, "decode_split", -2) == B.BL_ERR_SHAPE
    B.bl_set_tuning("decode_split", 0)
    assert _st(B.bl_set_tuning, "attn_groups", -1) == B.BL_ERR_SHAPE and _st(B.bl_set_tuning, "attn_groups", 65536) == B.BL_ERR_SHAPE
    B.bl_set_tuning("attn_groups", 7)
    B.bl_set_tuning("attn_groups", 0)
    assert B.bl_get_stat("nonsense") == -1 and B.bl_get_stat("split_launches") >= 0
    assert _st(B.bl_set_tuning, "nonsense", 1) == B.BL_ERR_SHAPE
    assert _st(B.bl_set_tuning, "gemv_waves", 3) == B.BL_ERR_SHAPE
    B.bl_set_tuning("gemv_waves", 0)
    assert _st(B.bl_set_tuning, "decode_path", 3) == B.BL_ERR_SHAPE
    assert _st(B.bl_set_tuning, "decode_stage", 2) == B.BL_ERR_SHAPE
    B.bl_set_tuning("decode_stage", 0)
    assert _st(B.bl_set_tuning, "gemm_mb", 7) == B.BL_ERR_SHAPE
    B.bl_set_tuning("gemm_mb", 0)
    B.bl_set_tuning("decode_path", 0)


def test_status_strings():
    seen = set()
    for s in range(0, 10):
        txt = B.status_str(s)
        assert txt and txt != "unknown status"
        seen.add(txt)
    assert len(seen) == 10
    assert B.status_str(99) == "unknown status"


def test_tl2_descriptor_and_validation():
    assert B.bl_tl2_padded_k(1) == 72 and B.bl_tl2_padded_k(72) == 72 and B.bl_tl2_padded_k(73) == 144
    assert B.bl_tl2_padded_k(0) == -1 and B.bl_tl2_padded_k(B.BL_MAX_K + 1) == -1
    d = B.bl_tl2_desc_init(3200, 8640, 0.02)            # 8640 = 120 tiles of 72
    assert (d.version, d.N, d.K, d.Np, d.Kp, d.bytes) == (2, 3200, 8640, 3200, 8640, 3200 * 120 * 16)
    assert d.bytes * 9 == B.bl_packed_desc_init(3200, 8640, 0.02).bytes * 8   # 16 bytes per 72 weights against 18
    d = B.bl_tl2_desc_init(70, 100, 1.0)
    assert (d.Np, d.Kp, d.bytes) == (128, 144, 128 * 2 * 16)
    assert _st(B.bl_tl2_desc_init, 0, 64, 1.0) == B.BL_ERR_SHAPE
    P = 0x10000
    v1 = B.bl_packed_desc_init(128, 144, 0.5)
    v2 = B.bl_tl2_desc_init(128, 144, 0.5)
    # the two layouts do not mix
    assert _st(B.bl_tl2_pack, P, v1, P) == B.BL_ERR_LAYOUT
    assert _st(B.bl_tl2_gemv, P, v1, P, P, P) == B.BL_ERR_LAYOUT
    assert _st(B.bl_gemv, P, v2, P, P, P, 1, P) == B.BL_ERR_LAYOUT
    assert _st(B.bl_pack_ternary, P, v2, P) == B.BL_ERR_LAYOUT
    # nulls, alignment, tampering
    assert _st(B.bl_tl2_pack, 0, v2, P) == B.BL_ERR_NULL
    assert _st(B.bl_tl2_unpack, P, v2, 0) == B.BL_ERR_NULL
    assert _st(B.bl_tl2_gemv, P, v2, 0, P, P) == B.BL_ERR_NULL
    assert _st(B.bl_tl2_gemv, P, v2, P, P, 0) == B.BL_ERR_NULL
    assert _st(B.bl_tl2_gemv, P + 8, v2, P, P, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_tl2_gemv, P, v2, P + 4, P, P) == B.BL_ERR_ALIGN
    assert _st(B.bl_tl2_pack, P, v2, P + 4) == B.BL_ERR_ALIGN
    items = B.make_gemv_items([(P, v2, P, P, 0, P, 0)])
    assert B.lib().bl_tl2_gemv_batch(items, 0, None, None) == B.BL_ERR_COUNT
    assert B.lib().bl_tl2_gemv_batch(items, 9, None, None) == B.BL_ERR_COUNT
    assert B.lib().bl_tl2_gemv_batch(None, 1, None, None) == B.BL_ERR_NULL
    assert B.lib().bl_tl2_gemv_batch(items, 1, P + 64, None) == B.BL_ERR_ALIGN
    assert B.lib().bl_tl2_gemv_batch(B.make_gemv_items([(P, v1, P, P, 0, P, 0)]), 1, None, None) == B.BL_ERR_LAYOUT
    bad = B.bl_tl2_desc_init(128, 144, 0.5)
    bad.bytes += 16
    assert _st(B.bl_tl2_gemv, P, bad, P, P, P) == B.BL_ERR_BUF_SMALL
    bad = B.bl_tl2_desc_init(128, 144, 0.5)
    bad.Kp = 192
    assert _st(B.bl_tl2_unpack, P, bad, P) == B.BL_ERR_SHAPE



def test_decoder_block_validation():
    P = 0x10000  # fake aligned device pointer, never dereferenced: validation fails first
    ok = dict(mode=B.BL_NORM_PLAIN, M=1, K=128, gamma_dev=P, eps=1e-5, a_dev=P, q_dev=P, a_scale_dev=P, q_sum_dev=P, Kp=128)
    def norm(**kw):
        return _st(B.bl_norm_quant, B.make_norm_quant_args(**dict(ok, **kw)))
    assert norm(gamma_dev=0) == B.BL_ERR_NULL
    assert norm(a_dev=0) == B.BL_ERR_NULL
    assert norm(mode=B.BL_NORM_RESIDUAL, h_dev=0) == B.BL_ERR_NULL
    assert norm(mode=B.BL_NORM_GATED, b_dev=0) == B.BL_ERR_NULL
    assert norm(a_scale_dev=0) == B.BL_ERR_NULL                      # q without its scale
    assert norm(q_dev=0, a_scale_dev=0) == B.BL_ERR_NULL             # q_sum without q
    assert norm(mode=4) == B.BL_ERR_SHAPE
    assert norm(M=0) == B.BL_ERR_SHAPE
    assert norm(K=0) == B.BL_ERR_SHAPE
    assert norm(K=B.BL_NORM_MAX_K + 1, Kp=B.BL_NORM_MAX_K + 4) == B.BL_ERR_SHAPE
    assert norm(Kp=124) == B.BL_ERR_SHAPE
    assert norm(Kp=130) == B.BL_ERR_SHAPE
    assert norm(a_dev=P + 2) == B.BL_ERR_ALIGN
    assert norm(q_dev=P + 1) == B.BL_ERR_ALIGN
    assert norm(scratch_dev=P + 4) == B.BL_ERR_ALIGN
    pre = dict(mode=B.BL_NORM_PREMULTIPLIED, gamma_dev=0, scratch_dev=P, pieces=8)
    assert norm(**dict(pre, scratch_dev=0)) == B.BL_ERR_NULL and norm(**dict(pre, pieces=0)) == B.BL_ERR_SHAPE
    assert norm(**dict(pre, M=2)) == B.BL_ERR_SHAPE and norm(**dict(pre, a_dev=0)) == B.BL_ERR_NULL
    assert _st(B.bl_rope_table, 0, 64, 16, 10000.0) == B.BL_ERR_NULL
    assert _st(B.bl_rope_table, P, 63, 16, 10000.0) == B.BL_ERR_SHAPE
    assert _st(B.bl_rope_table, P, 64, 0, 10000.0) == B.BL_ERR_SHAPE
    assert _st(B.bl_rope_table, P, 64, 16, 0.0) == B.BL_ERR_SHAPE
    assert _st(B.bl_rope_table, P + 4, 64, 16, 10000.0) == B.BL_ERR_ALIGN
    assert B.bl_attn_scratch_bytes(32, 102, 512) == 0                # head_dim not a multiple of 4
    assert B.bl_attn_scratch_bytes(32, 128, 513) == 32 * 9 * 130 * 4 + 32 * 4
    assert B.bl_attn_scratch_bytes(0, 128, 512) == 0 and B.bl_attn_scratch_bytes(1, 264, 512) == 0
    good = [P] * 9 + [4, 64, 100]
    def attn(i, v):
        a = list(good)
        a[i] = v
        return _st(B.bl_attn_decode, B.make_attn_args(*a))
    for i in range(9):
        assert attn(i, 0) == B.BL_ERR_NULL
    assert attn(9, 0) == B.BL_ERR_SHAPE and attn(10, 62) == B.BL_ERR_SHAPE and attn(11, 0) == B.BL_ERR_SHAPE
    assert attn(5, P + 8) == B.BL_ERR_ALIGN and attn(4, P + 4) == B.BL_ERR_ALIGN and attn(0, P + 1) == B.BL_ERR_ALIGN
    assert _st(B.bl_pos_advance, 0) == B.BL_ERR_NULL and _st(B.bl_pos_advance, P + 2) == B.BL_ERR_ALIGN


def test_decode_norm_batch_validation():
    P = 0x10000
    d = B.bl_packed_desc_init(128, 256, 0.5)
    ok = dict(x=P, delta=P, h_out=P + 0x1000, gamma=P, eps=1e-5, packed=P, desc=d, out=P)
    def call(count_items=1, ws=0, **kw):
        return _st(B.bl_decode_norm_batch, B.make_decode_norm_items([dict(ok, **kw)] * count_items), ws)
    for k in ("x", "packed", "out"):
        assert call(**{k: 0}) == B.BL_ERR_NULL
    assert call(gamma=0) == B.BL_ERR_NULL                                  # neither form of the norm
    assert call(h_out=P) == B.BL_ERR_SHAPE                                 # h_out on top of x (and of delta)
    assert call(desc=B.bl_packed_desc_init(128, 100, 0.5)) == B.BL_ERR_SHAPE            # K not a multiple of 8
    assert call(desc=B.bl_packed_desc_init(128, B.BL_DECODE_NORM_MAX_K + 8, 0.5)) == B.BL_ERR_SHAPE
    assert call(x=P + 8) == B.BL_ERR_ALIGN and call(gamma=P + 4) == B.BL_ERR_ALIGN and call(delta=P + 4) == B.BL_ERR_ALIGN
    assert call(count_items=9) == B.BL_ERR_COUNT
    assert call(ws=P + 16) == B.BL_ERR_ALIGN
    assert call(desc=B.bl_tl2_desc_init(128, 256, 0.5)) == B.BL_ERR_LAYOUT
    # the pre-multiplied row: no gamma, pieces instead; no residual add with it
    pre = dict(gamma=0, delta=0, h_out=0, ss_in=P, ss_count=4)
    assert call(**dict(pre, ss_count=0)) == B.BL_ERR_SHAPE
    assert call(**dict(pre, delta=P)) == B.BL_ERR_SHAPE
    assert call(ss_in=P, ss_count=4) == B.BL_ERR_SHAPE                     # both forms at once
    assert call(**dict(pre, ss_in=P + 4)) == B.BL_ERR_ALIGN
    # the gated epilogue: wants its pieces' destination and whole row blocks
    assert call(glu_gamma=P) == B.BL_ERR_NULL
    assert call(glu_gamma=P, ss_out=P, desc=B.bl_packed_desc_init(96, 256, 0.5)) == B.BL_ERR_SHAPE
    mixed = B.make_decode_norm_items([dict(ok), dict(ok, glu_gamma=P, ss_out=P)])
    assert _st(B.bl_decode_norm_batch, mixed, 0) == B.BL_ERR_SHAPE


def test_attn_prefill_validation():
    P = 0x10000
    ok = [P] * 8 + [4, 64, 100, 10, 20]
    def call(i, v):
        a = list(ok)
        a[i] = v
        return _st(B.bl_attn_prefill, *a)
    for i in range(8):
        assert call(i, 0) == B.BL_ERR_NULL
    assert call(8, 0) == B.BL_ERR_SHAPE and call(9, 62) == B.BL_ERR_SHAPE and call(12, 0) == B.BL_ERR_SHAPE
    assert call(11, -1) == B.BL_ERR_SHAPE and call(11, 90) == B.BL_ERR_SHAPE            # pos0 + M beyond the cache
    assert call(4, P + 8) == B.BL_ERR_ALIGN and call(7, P + 4) == B.BL_ERR_ALIGN
    assert call(1, P + 4) == B.BL_ERR_ALIGN and call(2, P + 4) == B.BL_ERR_ALIGN
    assert B.bl_attn_prefill_scratch_bytes(4, 160, 10, 20) == 20 * (4 * 1 * 162 + 4) * 4
    assert B.bl_attn_prefill_scratch_bytes(4, 160, 60, 10) == 10 * (4 * 2 * 162 + 4) * 4
    assert B.bl_attn_prefill_scratch_bytes(4, 64, 60, 10) == 16 == B.bl_attn_prefill_scratch_bytes(4, 128, 0, 1)
    assert B.bl_attn_prefill_scratch_bytes(4, 64, 0, 0) == 0 and B.bl_attn_prefill_scratch_bytes(4, 62, 0, 5) == 0
    assert ctypes.sizeof(B.AttnPrefillArgs) == 88


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus value ends with a message and a non-zero status before
    anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
