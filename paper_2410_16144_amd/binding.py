"""ctypes binding of libbitlinear.so: the same names and arguments as include/bitlinear.h.

Argument marshalling only.  Device pointers are plain integers (e.g. tensor.data_ptr()),
the stream is a hipStream_t handle as an integer (0 = default stream).  Every wrapper raises
BitLinearError on a non-zero status.  There is no fallback of any kind: if the shared
library has not been built, loading raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbitlinear.so")

BL_OK = 0
BL_ERR_NULL, BL_ERR_SHAPE, BL_ERR_M_RANGE, BL_ERR_BUF_SMALL, BL_ERR_ALIGN = 1, 2, 3, 4, 5
BL_ERR_DTYPE, BL_ERR_LAYOUT, BL_ERR_HIP, BL_ERR_COUNT, BL_ERR_WORKSPACE = 6, 7, 8, 9, 10
BL_F32, BL_BF16 = 0, 1
BL_LAYOUT_VERSION = 1
BL_TILE_N = 64
BL_TILE_K = 64
BL_MAX_K = 1048576
BL_MAX_GEMV_M = 8
BL_MAX_BATCH = 8
BL_MAX_GEMM_BATCH = 4
BL_MAX_SPLIT_WGS = 2048
BL_WORKSPACE_BYTES = BL_MAX_SPLIT_WGS * 64 * 8
BL_STATIC_WS_WGS = 1024
BL_STATIC_WS_BYTES = BL_STATIC_WS_WGS * 64 * 8
BL_MAX_GEMM_M = 4194304
BL_TL2_TILE_K = 72
BL_TL2_LAYOUT_VERSION = 2

# every symbol include/bitlinear.h and include/bitlinear_decoder.h declare
DECLARED_SYMBOLS = (
    "bl_padded_k", "bl_padded_n", "bl_packed_desc_init", "bl_pack_ternary", "bl_unpack_ternary",
    "bl_quant_act", "bl_quant_act_batch", "bl_gemv", "bl_gemv_batch", "bl_gemv_batch_static", "bl_decode_batch", "bl_gemm", "bl_gemm_batch", "bl_set_tuning", "bl_get_stat", "bl_status_str", "bl_last_hip_error", "bl_last_kernel", "bl_version",
    "bl_tl2_padded_k", "bl_tl2_desc_init", "bl_tl2_pack", "bl_tl2_unpack", "bl_tl2_gemv", "bl_tl2_gemv_batch",
    "bl_norm_quant", "bl_rope_table", "bl_attn_scratch_bytes", "bl_attn_decode", "bl_pos_advance", "bl_decode_norm_batch", "bl_pack_gate_up", "bl_attn_prefill", "bl_attn_prefill_scratch_bytes",
)

BL_NORM_MAX_K = 49152
BL_NORM_SCRATCH_BYTES = 256
BL_ATTN_MAX_HEAD_DIM = 256
BL_ATTN_CHUNK = 64
BL_ATTN_BLOCK_MAX_HEAD_DIM = 128
BL_NORM_PLAIN, BL_NORM_RESIDUAL, BL_NORM_GATED, BL_NORM_PREMULTIPLIED = 0, 1, 2, 3
BL_DECODE_NORM_MAX_K = 16384


class BitLinearError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        detail = ""
        if self.status == BL_ERR_HIP:
            detail = ": " + lib().bl_last_hip_error().decode()
        super().__init__("%s failed: status %d (%s%s)" % (where, self.status, status_str(self.status), detail))


class PackedDesc(ctypes.Structure):
    """Mirror of bl_packed_desc."""
    _fields_ = [("version", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("Np", ctypes.c_int64), ("Kp", ctypes.c_int64),
                ("bytes", ctypes.c_uint64), ("w_scale", ctypes.c_float), ("reserved2", ctypes.c_float)]


class GemvItem(ctypes.Structure):
    """Mirror of bl_gemv_item."""
    _fields_ = [("packed_dev", ctypes.c_void_p), ("desc", ctypes.POINTER(PackedDesc)),
                ("q_dev", ctypes.c_void_p), ("a_scale_dev", ctypes.c_void_p), ("q_sum_dev", ctypes.c_void_p),
                ("out_dev", ctypes.c_void_p), ("acc_dev", ctypes.c_void_p)]


class QuantItem(ctypes.Structure):
    """Mirror of bl_quant_item."""
    _fields_ = [("x_dev", ctypes.c_void_p), ("dt", ctypes.c_int), ("M", ctypes.c_int64), ("K", ctypes.c_int64),
                ("ldx", ctypes.c_int64), ("q_dev", ctypes.c_void_p), ("a_scale_dev", ctypes.c_void_p),
                ("q_sum_dev", ctypes.c_void_p)]


class DecodeItem(ctypes.Structure):
    """Mirror of bl_decode_item."""
    _fields_ = [("x_dev", ctypes.c_void_p), ("dt", ctypes.c_int), ("ldx", ctypes.c_int64),
                ("packed_dev", ctypes.c_void_p), ("desc", ctypes.POINTER(PackedDesc)),
                ("out_dev", ctypes.c_void_p), ("acc_dev", ctypes.c_void_p), ("q_dev", ctypes.c_void_p),
                ("a_scale_dev", ctypes.c_void_p), ("q_sum_dev", ctypes.c_void_p)]


class NormQuantArgs(ctypes.Structure):
    """Mirror of bl_norm_quant_args."""
    _fields_ = [("mode", ctypes.c_int32), ("M", ctypes.c_int32), ("K", ctypes.c_int64), ("Kp", ctypes.c_int64),
                ("a_dev", ctypes.c_void_p), ("b_dev", ctypes.c_void_p), ("h_dev", ctypes.c_void_p),
                ("gamma_dev", ctypes.c_void_p), ("eps", ctypes.c_float), ("q_dev", ctypes.c_void_p),
                ("a_scale_dev", ctypes.c_void_p), ("q_sum_dev", ctypes.c_void_p), ("y_dev", ctypes.c_void_p),
                ("scratch_dev", ctypes.c_void_p), ("pieces", ctypes.c_int32)]


class AttnArgs(ctypes.Structure):
    """Mirror of bl_attn_args."""
    _fields_ = [("q_lin_dev", ctypes.c_void_p), ("k_lin_dev", ctypes.c_void_p), ("v_lin_dev", ctypes.c_void_p),
                ("pos_dev", ctypes.c_void_p), ("rope_table_dev", ctypes.c_void_p), ("k_cache_dev", ctypes.c_void_p),
                ("v_cache_dev", ctypes.c_void_p), ("out_dev", ctypes.c_void_p), ("scratch_dev", ctypes.c_void_p),
                ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("max_pos", ctypes.c_int32)]


class DecodeNormItem(ctypes.Structure):
    """Mirror of bl_decode_norm_item."""
    _fields_ = [("x_dev", ctypes.c_void_p), ("delta_dev", ctypes.c_void_p), ("h_out_dev", ctypes.c_void_p),
                ("gamma_dev", ctypes.c_void_p), ("eps", ctypes.c_float), ("packed_dev", ctypes.c_void_p),
                ("desc", ctypes.POINTER(PackedDesc)), ("out_dev", ctypes.c_void_p), ("acc_dev", ctypes.c_void_p),
                ("q_dev", ctypes.c_void_p), ("a_scale_dev", ctypes.c_void_p), ("q_sum_dev", ctypes.c_void_p),
                ("ss_in_dev", ctypes.c_void_p), ("ss_count", ctypes.c_int32), ("w_scale_up", ctypes.c_float),
                ("glu_gamma_dev", ctypes.c_void_p), ("ss_out_dev", ctypes.c_void_p)]


class AttnPrefillArgs(ctypes.Structure):
    """Mirror of bl_attn_prefill_args."""
    _fields_ = [("q_lin_dev", ctypes.c_void_p), ("k_lin_dev", ctypes.c_void_p), ("v_lin_dev", ctypes.c_void_p),
                ("rope_table_dev", ctypes.c_void_p), ("k_cache_dev", ctypes.c_void_p), ("v_cache_dev", ctypes.c_void_p),
                ("out_dev", ctypes.c_void_p), ("scratch_dev", ctypes.c_void_p), ("n_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("max_pos", ctypes.c_int32), ("pos0", ctypes.c_int32), ("M", ctypes.c_int32)]


_lib = None


def lib():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libbitlinear.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'` "
            "or `python paper_2410_16144_amd/build.py`. There is no CPU fallback." % LIB_PATH)
    # PyTorch first: its wheel carries the HIP runtime this library is linked against, and the
    # process must hold exactly one HIP runtime (streams and allocations are per runtime).
    import torch  # noqa: F401
    l = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    dp = ctypes.POINTER(PackedDesc)
    l.bl_padded_k.argtypes = [i64]
    l.bl_padded_k.restype = i64
    l.bl_padded_n.argtypes = [i64]
    l.bl_padded_n.restype = i64
    l.bl_packed_desc_init.argtypes = [i64, i64, ctypes.c_float, dp]
    l.bl_pack_ternary.argtypes = [vp, dp, vp, vp, vp]
    l.bl_unpack_ternary.argtypes = [vp, dp, vp, vp]
    l.bl_pack_gate_up.argtypes = [vp, vp, dp, vp, vp, vp]
    l.bl_quant_act.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp]
    l.bl_quant_act_batch.argtypes = [ctypes.POINTER(QuantItem), i32, vp]
    l.bl_gemv.argtypes = [vp, dp, vp, vp, vp, i64, vp, vp, vp]
    l.bl_gemv_batch.argtypes = [ctypes.POINTER(GemvItem), i32, i64, vp, vp]
    l.bl_gemv_batch_static.argtypes = [ctypes.POINTER(GemvItem), i32, i64, vp]
    l.bl_gemm_batch.argtypes = [ctypes.POINTER(GemvItem), i32, i64, vp]
    l.bl_decode_batch.argtypes = [ctypes.POINTER(DecodeItem), i32, i64, vp, vp]
    l.bl_gemm.argtypes = [vp, dp, vp, vp, vp, i64, vp, vp, vp]
    l.bl_tl2_padded_k.argtypes = [i64]
    l.bl_tl2_padded_k.restype = i64
    l.bl_tl2_desc_init.argtypes = [i64, i64, ctypes.c_float, dp]
    l.bl_tl2_pack.argtypes = [vp, dp, vp, vp, vp]
    l.bl_tl2_unpack.argtypes = [vp, dp, vp, vp]
    l.bl_tl2_gemv.argtypes = [vp, dp, vp, vp, vp, vp, vp]
    l.bl_tl2_gemv_batch.argtypes = [ctypes.POINTER(GemvItem), i32, vp, vp]
    l.bl_norm_quant.argtypes = [ctypes.POINTER(NormQuantArgs), vp]
    l.bl_rope_table.argtypes = [vp, i32, i32, ctypes.c_double, vp]
    l.bl_attn_scratch_bytes.argtypes = [i32, i32, i32]
    l.bl_attn_scratch_bytes.restype = ctypes.c_uint64
    l.bl_attn_decode.argtypes = [ctypes.POINTER(AttnArgs), vp]
    l.bl_pos_advance.argtypes = [vp, vp]
    l.bl_decode_norm_batch.argtypes = [ctypes.POINTER(DecodeNormItem), i32, vp, vp]
    l.bl_attn_prefill.argtypes = [ctypes.POINTER(AttnPrefillArgs), vp]
    l.bl_attn_prefill_scratch_bytes.argtypes = [i32, i32, i32, i32]
    l.bl_attn_prefill_scratch_bytes.restype = ctypes.c_uint64
    l.bl_set_tuning.argtypes = [ctypes.c_char_p, i32]
    l.bl_get_stat.argtypes = [ctypes.c_char_p]
    l.bl_get_stat.restype = i64
    l.bl_status_str.argtypes = [ctypes.c_int]
    l.bl_status_str.restype = ctypes.c_char_p
    l.bl_version.restype = ctypes.c_char_p
    l.bl_last_hip_error.restype = ctypes.c_char_p
    l.bl_last_kernel.restype = ctypes.c_char_p
    for name in ("bl_packed_desc_init", "bl_pack_ternary", "bl_unpack_ternary", "bl_quant_act", "bl_quant_act_batch", "bl_gemv",
                 "bl_gemv_batch", "bl_decode_batch", "bl_gemm", "bl_set_tuning", "bl_tl2_desc_init", "bl_tl2_pack",
                 "bl_tl2_unpack", "bl_tl2_gemv", "bl_tl2_gemv_batch", "bl_norm_quant", "bl_rope_table", "bl_attn_decode",
                 "bl_pos_advance", "bl_decode_norm_batch", "bl_attn_prefill", "bl_gemm_batch", "bl_gemv_batch_static", "bl_pack_gate_up"):
        getattr(l, name).restype = ctypes.c_int
    _lib = l
    return l


def _check(status, where):
    if status != BL_OK:
        raise BitLinearError(status, where)


def status_str(status: int) -> str:
    return lib().bl_status_str(int(status)).decode()


def version() -> str:
    return lib().bl_version().decode()


def bl_padded_k(K: int) -> int:
    return int(lib().bl_padded_k(K))


def bl_padded_n(N: int) -> int:
    return int(lib().bl_padded_n(N))


def bl_packed_desc_init(N: int, K: int, w_scale: float) -> PackedDesc:
    d = PackedDesc()
    _check(lib().bl_packed_desc_init(N, K, float(w_scale), ctypes.byref(d)), "bl_packed_desc_init")
    return d


def bl_pack_ternary(w_dev: int, desc: PackedDesc, packed_dev: int, bad_count_dev: int = 0, stream: int = 0):
    _check(lib().bl_pack_ternary(w_dev, ctypes.byref(desc), packed_dev, bad_count_dev or None, stream or None),
           "bl_pack_ternary")


def bl_pack_gate_up(gate_dev: int, up_dev: int, desc: PackedDesc, packed_dev: int, bad_count_dev: int = 0, stream: int = 0):
    _check(lib().bl_pack_gate_up(gate_dev, up_dev, ctypes.byref(desc), packed_dev, bad_count_dev or None, stream or None),
           "bl_pack_gate_up")


def bl_unpack_ternary(packed_dev: int, desc: PackedDesc, w_dev: int, stream: int = 0):
    _check(lib().bl_unpack_ternary(packed_dev, ctypes.byref(desc), w_dev, stream or None), "bl_unpack_ternary")


def bl_quant_act(x_dev: int, dtype: int, M: int, K: int, ldx: int, q_dev: int, a_scale_dev: int,
                 q_sum_dev: int = 0, stream: int = 0):
    _check(lib().bl_quant_act(x_dev, dtype, M, K, ldx, q_dev, a_scale_dev, q_sum_dev or None, stream or None),
           "bl_quant_act")


def make_quant_items(items):
    """items: iterable of (x_dev, dtype, M, K, ldx, q_dev, a_scale_dev, q_sum_dev) -> ctypes array."""
    items = list(items)
    arr = (QuantItem * len(items))()
    for i, (x, dt, M, K, ldx, q, a, s) in enumerate(items):
        arr[i] = QuantItem(x, dt, M, K, ldx, q, a, s or None)
    return arr


def bl_quant_act_batch(items, stream: int = 0):
    """items: a ctypes QuantItem array from make_quant_items (or an iterable of tuples)."""
    if not isinstance(items, ctypes.Array):
        items = make_quant_items(items)
    _check(lib().bl_quant_act_batch(items, len(items), stream or None), "bl_quant_act_batch")


def bl_gemv(packed_dev: int, desc: PackedDesc, q_dev: int, a_scale_dev: int, q_sum_dev: int, M: int,
            out_dev: int, acc_dev: int = 0, stream: int = 0):
    _check(lib().bl_gemv(packed_dev, ctypes.byref(desc), q_dev, a_scale_dev, q_sum_dev, M, out_dev,
                         acc_dev or None, stream or None), "bl_gemv")


def make_gemv_items(items):
    """items: iterable of (packed_dev, desc, q_dev, a_scale_dev, q_sum_dev, out_dev, acc_dev) -> ctypes array.
    The PackedDesc objects must outlive the array."""
    items = list(items)
    arr = (GemvItem * len(items))()
    for i, (packed, desc, q, a, s, out, acc) in enumerate(items):
        arr[i] = GemvItem(packed, ctypes.pointer(desc), q, a, s or None, out, acc or None)
    return arr


def bl_gemv_batch(items, M: int, workspace_dev: int = 0, stream: int = 0):
    """items: a ctypes GemvItem array from make_gemv_items (or an iterable of tuples)."""
    if not isinstance(items, ctypes.Array):
        items = make_gemv_items(items)
    _check(lib().bl_gemv_batch(items, len(items), M, workspace_dev or None, stream or None), "bl_gemv_batch")


def bl_gemv_batch_static(items, M: int, stream: int = 0):
    """bl_gemv_batch with the workspace in the library's static device array (nothing allocated, nothing passed)."""
    if not isinstance(items, ctypes.Array):
        items = make_gemv_items(items)
    _check(lib().bl_gemv_batch_static(items, len(items), M, stream or None), "bl_gemv_batch_static")


def bl_gemm_batch(items, M: int, stream: int = 0):
    """items: a ctypes GemvItem array from make_gemv_items (or an iterable of tuples), at most BL_MAX_GEMM_BATCH."""
    if not isinstance(items, ctypes.Array):
        items = make_gemv_items(items)
    _check(lib().bl_gemm_batch(items, len(items), M, stream or None), "bl_gemm_batch")


def make_decode_items(items):
    """items: iterable of (x_dev, dtype, ldx, packed_dev, desc, out_dev, acc_dev, q_dev, a_scale_dev, q_sum_dev)
    -> ctypes array.  The PackedDesc objects must outlive the array."""
    items = list(items)
    arr = (DecodeItem * len(items))()
    for i, (x, dt, ldx, packed, desc, out, acc, q, a, s) in enumerate(items):
        arr[i] = DecodeItem(x, dt, ldx, packed, ctypes.pointer(desc), out, acc or None, q or None, a or None,
                            s or None)
    return arr


def bl_decode_batch(items, M: int, workspace_dev: int = 0, stream: int = 0):
    """items: a ctypes DecodeItem array from make_decode_items (or an iterable of tuples)."""
    if not isinstance(items, ctypes.Array):
        items = make_decode_items(items)
    _check(lib().bl_decode_batch(items, len(items), M, workspace_dev or None, stream or None), "bl_decode_batch")


def bl_gemm(packed_dev: int, desc: PackedDesc, q_dev: int, a_scale_dev: int, q_sum_dev: int, M: int,
            out_dev: int, acc_dev: int = 0, stream: int = 0):
    _check(lib().bl_gemm(packed_dev, ctypes.byref(desc), q_dev, a_scale_dev, q_sum_dev, M, out_dev,
                         acc_dev or None, stream or None), "bl_gemm")


def bl_tl2_padded_k(K: int) -> int:
    return int(lib().bl_tl2_padded_k(K))


def bl_tl2_desc_init(N: int, K: int, w_scale: float) -> PackedDesc:
    d = PackedDesc()
    _check(lib().bl_tl2_desc_init(N, K, float(w_scale), ctypes.byref(d)), "bl_tl2_desc_init")
    return d


def bl_tl2_pack(w_dev: int, desc: PackedDesc, packed_dev: int, bad_count_dev: int = 0, stream: int = 0):
    _check(lib().bl_tl2_pack(w_dev, ctypes.byref(desc), packed_dev, bad_count_dev or None, stream or None),
           "bl_tl2_pack")


def bl_tl2_unpack(packed_dev: int, desc: PackedDesc, w_dev: int, stream: int = 0):
    _check(lib().bl_tl2_unpack(packed_dev, ctypes.byref(desc), w_dev, stream or None), "bl_tl2_unpack")


def bl_tl2_gemv(packed_dev: int, desc: PackedDesc, q_dev: int, a_scale_dev: int, out_dev: int, acc_dev: int = 0,
                stream: int = 0):
    _check(lib().bl_tl2_gemv(packed_dev, ctypes.byref(desc), q_dev, a_scale_dev, out_dev, acc_dev or None,
                             stream or None), "bl_tl2_gemv")


def bl_tl2_gemv_batch(items, workspace_dev: int = 0, stream: int = 0):
    """items: a ctypes GemvItem array from make_gemv_items (q_sum_dev may be 0), or an iterable of tuples."""
    if not isinstance(items, ctypes.Array):
        items = make_gemv_items(items)
    _check(lib().bl_tl2_gemv_batch(items, len(items), workspace_dev or None, stream or None), "bl_tl2_gemv_batch")


def make_norm_quant_args(mode: int, M: int, K: int, gamma_dev: int, eps: float, a_dev: int = 0, b_dev: int = 0,
                         h_dev: int = 0, q_dev: int = 0, a_scale_dev: int = 0, q_sum_dev: int = 0, Kp: int = 0,
                         y_dev: int = 0, scratch_dev: int = 0, pieces: int = 0) -> NormQuantArgs:
    return NormQuantArgs(mode, M, K, Kp, a_dev or None, b_dev or None, h_dev or None, gamma_dev or None, eps,
                         q_dev or None, a_scale_dev or None, q_sum_dev or None, y_dev or None, scratch_dev or None, pieces)


def bl_norm_quant(args: NormQuantArgs, stream: int = 0):
    _check(lib().bl_norm_quant(ctypes.byref(args), stream), "bl_norm_quant")


def bl_rope_table(table_dev: int, head_dim: int, max_pos: int, theta: float, stream: int = 0):
    _check(lib().bl_rope_table(table_dev, head_dim, max_pos, theta, stream), "bl_rope_table")


def bl_attn_scratch_bytes(n_heads: int, head_dim: int, max_pos: int) -> int:
    return int(lib().bl_attn_scratch_bytes(n_heads, head_dim, max_pos))


def make_attn_args(q_lin_dev: int, k_lin_dev: int, v_lin_dev: int, pos_dev: int, rope_table_dev: int, k_cache_dev: int,
                   v_cache_dev: int, out_dev: int, scratch_dev: int, n_heads: int, head_dim: int, max_pos: int) -> AttnArgs:
    return AttnArgs(q_lin_dev or None, k_lin_dev or None, v_lin_dev or None, pos_dev or None, rope_table_dev or None,
                    k_cache_dev or None, v_cache_dev or None, out_dev or None, scratch_dev or None, n_heads, head_dim,
                    max_pos)


def bl_attn_decode(args: AttnArgs, stream: int = 0):
    _check(lib().bl_attn_decode(ctypes.byref(args), stream), "bl_attn_decode")


def bl_attn_prefill_scratch_bytes(n_heads: int, head_dim: int, pos0: int, M: int) -> int:
    return int(lib().bl_attn_prefill_scratch_bytes(n_heads, head_dim, pos0, M))


def bl_attn_prefill(q_lin_dev: int, k_lin_dev: int, v_lin_dev: int, rope_table_dev: int, k_cache_dev: int, v_cache_dev: int,
                    out_dev: int, scratch_dev: int, n_heads: int, head_dim: int, max_pos: int, pos0: int, M: int, stream: int = 0):
    args = AttnPrefillArgs(q_lin_dev or None, k_lin_dev or None, v_lin_dev or None, rope_table_dev or None, k_cache_dev or None,
                           v_cache_dev or None, out_dev or None, scratch_dev or None, n_heads, head_dim, max_pos, pos0, M)
    _check(lib().bl_attn_prefill(ctypes.byref(args), stream), "bl_attn_prefill")


def bl_pos_advance(pos_dev: int, stream: int = 0):
    _check(lib().bl_pos_advance(pos_dev, stream), "bl_pos_advance")


def make_decode_norm_items(items):
    """items: iterable of dicts with the fields of bl_decode_norm_item without the _dev suffix (x, gamma, eps, packed,
    desc, out required as the form demands; the rest optional: 0 / absent = NULL).  Returns a ctypes array that keeps
    the descriptors alive."""
    items = list(items)
    arr = (DecodeNormItem * len(items))()
    for i, it in enumerate(items):
        g = lambda k: it.get(k) or None
        arr[i] = DecodeNormItem(g("x"), g("delta"), g("h_out"), g("gamma"), it.get("eps", 0.0), g("packed"),
                                ctypes.pointer(it["desc"]), g("out"), g("acc"), g("q"), g("a_scale"), g("q_sum"),
                                g("ss_in"), it.get("ss_count", 0), it.get("w_scale_up", 0.0), g("glu_gamma"), g("ss_out"))
    arr._descs = [it["desc"] for it in items]
    return arr


def bl_decode_norm_batch(items, workspace_dev: int = 0, stream: int = 0):
    _check(lib().bl_decode_norm_batch(items, len(items), workspace_dev or None, stream), "bl_decode_norm_batch")


def bl_set_tuning(key: str, value: int):
    _check(lib().bl_set_tuning(key.encode(), int(value)), "bl_set_tuning")


def bl_last_kernel() -> str:
    return lib().bl_last_kernel().decode()


def bl_get_stat(key: str) -> int:
    return int(lib().bl_get_stat(key.encode()))
