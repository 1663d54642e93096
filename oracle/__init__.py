"""numpy-facing wrapper over the C oracle (oracle/bitlinear_oracle.c).

TEST INFRASTRUCTURE: the plain CPU definition of the BitLinear product of
arXiv 2410.16144, used by the test-suite, the smoke check and the benchmark's
cpu_baseline leg only.  It never imports the GPU package and the GPU package
never imports it.  All arithmetic lives in the C file; this module only
marshals numpy arrays.

bf16 activations are passed as numpy uint16 arrays holding the bit patterns;
fp32 activations as float32 arrays.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = ctypes.CDLL(_build.build())

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_f32 = ctypes.c_float

_lib.orc_num_threads.restype = ctypes.c_int
_lib.orc_set_num_threads.argtypes = [ctypes.c_int]
_lib.orc_absmean_ternarize.argtypes = [_vp, _i64, _vp, _vp]
_lib.orc_i2s_encode.argtypes = [ctypes.c_int]
_lib.orc_i2s_encode.restype = ctypes.c_int
_lib.orc_i2s_decode.argtypes = [ctypes.c_int]
_lib.orc_i2s_decode.restype = ctypes.c_int
_lib.orc_i2s_pack.argtypes = [_vp, _i64, _i64, _vp]
_lib.orc_i2s_pack.restype = _i64
_lib.orc_i2s_unpack.argtypes = [_vp, _i64, _i64, _vp]
_lib.orc_i2s_unpack.restype = _i64
_lib.orc_tl1_index.argtypes = [ctypes.c_int, ctypes.c_int]
_lib.orc_tl1_index.restype = ctypes.c_int
_lib.orc_tl2_code.argtypes = [ctypes.c_int] * 3 + [_vp, _vp]
_lib.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
_lib.orc_bf16_to_f32.restype = _f32
_lib.orc_quant_act.argtypes = [_vp, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _vp, _vp]
_lib.orc_matmul_i32.argtypes = [_vp, _i64, _i64, _i64, _vp, _i64, _vp]
_lib.orc_matmul_i32_cols.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _i64, _vp]
_lib.orc_dequant.argtypes = [_vp, _i64, _i64, _f32, _vp, _vp]
_lib.orc_bitlinear.argtypes = [_vp, ctypes.c_int, _i64, _i64, _i64, _vp, _i64, _f32, _vp, _vp, _vp, _vp]
_lib.orc_tl1_gemv_i32.argtypes = [_vp, _i64, _vp, _i64, _vp]
_lib.orc_tl2_gemv_i32.argtypes = [_vp, _i64, _vp, _i64, _vp]
_lib.orc_tl2_encode_rows.argtypes = [_vp, _i64, _i64, _vp]
_lib.orc_tl2_encode_rows.restype = _i64
_lib.orc_tl2_decode_rows.argtypes = [_vp, _i64, _i64, _vp]
_lib.orc_tl2_decode_rows.restype = _i64


def _p(a):
    return a.ctypes.data_as(_vp)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError("expected %s, got %s" % (np.dtype(dtype), a.dtype))
    return a


def num_threads() -> int:
    return int(_lib.orc_num_threads())


def set_num_threads(n: int) -> None:
    _lib.orc_set_num_threads(int(n))


def absmean_ternarize(wf):
    """fp32 matrix -> (ternary int8 matrix, fp32 absmean scale)."""
    wf = _c(wf, np.float32)
    wt = np.empty(wf.shape, np.int8)
    s = ctypes.c_float(0.0)
    _lib.orc_absmean_ternarize(_p(wf), wf.size, _p(wt), ctypes.byref(s))
    return wt, np.float32(s.value)


def i2s_encode(w: int) -> int:
    return int(_lib.orc_i2s_encode(int(w)))


def i2s_decode(code: int) -> int:
    return int(_lib.orc_i2s_decode(int(code)))


def i2s_pack(w):
    """[N,K] int8 -> ([N, ceil(K/4)] uint8 canonical packing, bad count)."""
    w = _c(w, np.int8)
    n, k = w.shape
    out = np.empty((n, (k + 3) // 4), np.uint8)
    bad = _lib.orc_i2s_pack(_p(w), n, k, _p(out))
    return out, int(bad)


def i2s_unpack(packed, k: int):
    packed = _c(packed, np.uint8)
    n = packed.shape[0]
    assert packed.shape[1] == (k + 3) // 4
    w = np.empty((n, k), np.int8)
    bad = _lib.orc_i2s_unpack(_p(packed), n, k, _p(w))
    return w, int(bad)


def tl1_index(w0: int, w1: int) -> int:
    return int(_lib.orc_tl1_index(int(w0), int(w1)))


def tl2_code(w0: int, w1: int, w2: int):
    s = ctypes.c_int(0)
    i = ctypes.c_int(0)
    _lib.orc_tl2_code(int(w0), int(w1), int(w2), ctypes.byref(s), ctypes.byref(i))
    return s.value, i.value


def tl2_encode_rows(w):
    """[N,K] int8 -> ([N, ceil(K/3)] uint8 codes sign << 4 | index (Table 3), bad count)."""
    w = _c(w, np.int8)
    n, k = w.shape
    codes = np.empty((n, (k + 2) // 3), np.uint8)
    bad = _lib.orc_tl2_encode_rows(_p(w), n, k, _p(codes))
    return codes, int(bad)


def tl2_decode_rows(codes, k: int):
    codes = _c(codes, np.uint8)
    n = codes.shape[0]
    assert codes.shape[1] == (k + 2) // 3
    w = np.empty((n, k), np.int8)
    bad = _lib.orc_tl2_decode_rows(_p(codes), n, k, _p(w))
    return w, int(bad)


def bf16_to_f32(bits) -> np.ndarray:
    bits = np.asarray(bits, np.uint16)
    flat = bits.reshape(-1)
    out = np.array([_lib.orc_bf16_to_f32(int(h)) for h in flat], np.float32)
    return out.reshape(bits.shape)


def quant_act(x):
    """[M,K] float32 or uint16(bf16 bits) -> (q int8 [M,K], a_scale f32 [M], q_sum i32 [M])."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        is_bf16 = 0
    elif x.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("activations must be float32 or uint16 (bf16 bits)")
    m, k = x.shape
    q = np.empty((m, k), np.int8)
    a = np.empty((m,), np.float32)
    s = np.empty((m,), np.int32)
    _lib.orc_quant_act(_p(x), is_bf16, m, k, k, _p(q), k, _p(a), _p(s))
    return q, a, s


def matmul_i32(q, w):
    """q [M,K] int8, w [N,K] int8 ternary -> acc [M,N] int32 (exact)."""
    q = _c(q, np.int8)
    w = _c(w, np.int8)
    m, k = q.shape
    n, k2 = w.shape
    assert k == k2
    acc = np.empty((m, n), np.int32)
    _lib.orc_matmul_i32(_p(q), m, k, k, _p(w), n, _p(acc))
    return acc


def matmul_i32_cols(q, w, n_idx):
    """As matmul_i32 but only for the output columns listed in n_idx."""
    q = _c(q, np.int8)
    w = _c(w, np.int8)
    n_idx = np.ascontiguousarray(n_idx, np.int64)
    m, k = q.shape
    assert w.shape[1] == k
    assert n_idx.size == 0 or (n_idx.min() >= 0 and n_idx.max() < w.shape[0])
    acc = np.empty((m, n_idx.size), np.int32)
    _lib.orc_matmul_i32_cols(_p(q), m, k, k, _p(w), _p(n_idx), n_idx.size, _p(acc))
    return acc


def dequant(acc, w_scale, a_scale):
    acc = _c(acc, np.int32)
    a_scale = _c(a_scale, np.float32)
    m, n = acc.shape
    out = np.empty((m, n), np.float32)
    _lib.orc_dequant(_p(acc), m, n, float(np.float32(w_scale)), _p(a_scale), _p(out))
    return out


def bitlinear(x, w, w_scale):
    """Full forward.  Returns dict(q, a_scale, q_sum, acc, out)."""
    q, a, s = quant_act(x)
    acc = matmul_i32(q, w)
    out = dequant(acc, w_scale, a)
    return {"q": q, "a_scale": a, "q_sum": s, "acc": acc, "out": out}


def bitlinear_whole(x, w, w_scale):
    """The C oracle's one-call forward (orc_bitlinear): quantize, integer product, dequantize inside one C
    function.  Returns dict(q, a_scale, acc, out); must agree bit for bit with bitlinear()."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        is_bf16 = 0
    elif x.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("activations must be float32 or uint16 (bf16 bits)")
    w = _c(w, np.int8)
    m, k = x.shape
    n, k2 = w.shape
    assert k == k2
    q = np.empty((m, k), np.int8)
    a = np.empty((m,), np.float32)
    acc = np.empty((m, n), np.int32)
    out = np.empty((m, n), np.float32)
    _lib.orc_bitlinear(_p(x), is_bf16, m, k, k, _p(w), n, float(np.float32(w_scale)), _p(q), _p(a), _p(acc), _p(out))
    return {"q": q, "a_scale": a, "acc": acc, "out": out}


def tl1_gemv_i32(q_row, w):
    q_row = _c(q_row, np.int8).reshape(-1)
    w = _c(w, np.int8)
    n, k = w.shape
    assert q_row.size == k
    acc = np.empty((n,), np.int32)
    _lib.orc_tl1_gemv_i32(_p(q_row), k, _p(w), n, _p(acc))
    return acc


def tl2_gemv_i32(q_row, w):
    q_row = _c(q_row, np.int8).reshape(-1)
    w = _c(w, np.int8)
    n, k = w.shape
    assert q_row.size == k
    acc = np.empty((n,), np.int32)
    _lib.orc_tl2_gemv_i32(_p(q_row), k, _p(w), n, _p(acc))
    return acc
