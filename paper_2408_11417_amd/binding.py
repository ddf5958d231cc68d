"""ctypes binding of libstreamk.so: the same names as the C ABI in include/streamk.h.

Argument marshalling only.  The library is loaded at import; if it has not been
built (python -m paper_2408_11417_amd.build, or __graft_entry__.build()) the
import fails: there is no fallback path.
"""
import ctypes
import os

try:
    # Device buffers and streams come from PyTorch, which ships its own HIP runtime.  Load it
    # first so that libstreamk.so binds to the same runtime instance instead of a second one.
    import torch  # noqa: F401
except ImportError:
    pass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstreamk.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libstreamk.so is not built: run `python -m paper_2408_11417_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

SK_OK, SK_ERR_INVALID_ARG, SK_ERR_UNSUPPORTED, SK_ERR_WORKSPACE = 0, -1, -2, -3
SK_ERR_HIP, SK_ERR_NOMEM, SK_ERR_TIMEOUT = -4, -5, -6
POLICY_NAMES = ("DP", "SK1_DP", "SK2_DP", "SK3_DP", "SK4_DP", "SK5_DP", "ALL_SK", "SK6_DP_EXT")
(SK_POLICY_DP, SK_POLICY_SK1_DP, SK_POLICY_SK2_DP, SK_POLICY_SK3_DP, SK_POLICY_SK4_DP,
 SK_POLICY_SK5_DP, SK_POLICY_ALL_SK, SK_POLICY_SK6_DP_EXT) = range(8)
SK_NUM_POLICIES = 7
SK_F16, SK_BF16, SK_FP8_E4M3, SK_F32 = 0, 1, 2, 3
SK_ROLE_FULL, SK_ROLE_OWNER, SK_ROLE_CONTRIB = 0, 1, 2
SK_ORDER_ROW_MAJOR, SK_ORDER_GROUPED = 0, 1
SK_FIXUP_FLAGS, SK_FIXUP_ATOMIC = 0, 1
SK_STREAMK_FIRST, SK_DATA_PARALLEL_FIRST = 0, 1
SK_SEGMENTS_ASCENDING, SK_SEGMENTS_K_ALIGNED = 0, 1

EXPORTS = ("sk_plan", "sk_plan_info", "sk_plan_ranges", "sk_plan_segments", "sk_plan_tile_coords", "sk_workspace_bytes",
           "sk_plan_set_fixup", "sk_plan_set_batch_order", "sk_plan_set_segment_order", "sk_plan_set_workspace", "sk_plan_set_spin_limit", "sk_plan_set_kernel_variant", "sk_gemm", "sk_gemm_static", "sk_plan_check", "sk_plan_kernel_info",
           "sk_plan_destroy", "sk_mfma_peak_operand_bytes", "sk_mfma_peak_launch", "sk_default_tile", "sk_plan_estimate_us", "bloom_winner_mask", "bloom_build", "bloom_insert", "bloom_query",
           "bloom_query_many", "bloom_bits", "bloom_serialize", "bloom_deserialize", "bloom_shape_key", "bloom_murmur3_32", "bloom_destroy", "sk_status_str", "sk_last_hip_error")


class sk_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("blk_m", "blk_n", "blk_k", "grid", "in_dtype", "out_dtype", "tile_order")]


class sk_plan_header(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("policy", ctypes.c_int32), ("blk_m", ctypes.c_int32), ("blk_n", ctypes.c_int32),
                ("blk_k", ctypes.c_int32), ("grid", ctypes.c_int32), ("in_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32), ("tiles_m", ctypes.c_int32), ("tiles_n", ctypes.c_int32),
                ("tiles", ctypes.c_int32), ("iters_per_tile", ctypes.c_int32),
                ("total_iters", ctypes.c_int64), ("sk_tiles", ctypes.c_int32), ("dp_tiles", ctypes.c_int32),
                ("sk_iters", ctypes.c_int64), ("iters_per_wg", ctypes.c_int32), ("dp_waves", ctypes.c_int32),
                ("has_kernel", ctypes.c_int32), ("tile_order", ctypes.c_int32),
                ("fixup", ctypes.c_int32), ("batch_order", ctypes.c_int32), ("segment_order", ctypes.c_int32),
                ("xcd_remap", ctypes.c_int32)]


class sk_wg_range(ctypes.Structure):
    _fields_ = [("sk_iter_begin", ctypes.c_int64), ("sk_iter_end", ctypes.c_int64),
                ("dp_tile_first", ctypes.c_int32), ("dp_tile_count", ctypes.c_int32)]


class sk_segment(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("wg", "tile", "k_begin", "k_end", "role")]


class sk_bloom_record(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("M", "N", "K", "policy_mask")]


class sk_bloom_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("m_bits", "k_probes", "n_filters")]


_vp, _i64, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
_lib.sk_plan.argtypes = [_i64, _i64, _i64, _int, ctypes.POINTER(sk_config), ctypes.POINTER(_vp)]
_lib.sk_plan_info.argtypes = [_vp, ctypes.POINTER(sk_plan_header)]
_lib.sk_plan_ranges.argtypes = [_vp, ctypes.POINTER(sk_wg_range)]
_lib.sk_plan_segments.argtypes = [_vp, ctypes.POINTER(sk_segment), ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
_lib.sk_plan_tile_coords.argtypes = [_vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
_lib.sk_workspace_bytes.argtypes = [_vp]
_lib.sk_workspace_bytes.restype = ctypes.c_size_t
_lib.sk_plan_set_workspace.argtypes = [_vp, _vp, ctypes.c_size_t]
_lib.sk_plan_set_spin_limit.argtypes = [_vp, ctypes.c_uint32]
_lib.sk_plan_set_kernel_variant.argtypes = [_vp, _int]
_lib.sk_plan_set_fixup.argtypes = [_vp, _int]
_lib.sk_plan_set_batch_order.argtypes = [_vp, _int]
_lib.sk_plan_set_segment_order.argtypes = [_vp, _int]
_lib.sk_plan_estimate_us.argtypes = [_vp, ctypes.POINTER(ctypes.c_double)]
_lib.sk_gemm.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.sk_mfma_peak_operand_bytes.restype = ctypes.c_size_t
_lib.sk_mfma_peak_launch.argtypes = [_int, _vp, _vp, _int, _int, _vp, ctypes.POINTER(ctypes.c_double)]
_lib.sk_gemm_static.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.sk_plan_check.argtypes = [_vp, _vp]
_lib.sk_plan_kernel_info.argtypes = [_vp] + [ctypes.POINTER(ctypes.c_int32)] * 3
_lib.sk_plan_destroy.argtypes = [_vp]
_lib.sk_plan_destroy.restype = None
_lib.sk_default_tile.argtypes = [_i64, _i64, _i64, _int, ctypes.POINTER(ctypes.c_int32)]
_lib.bloom_build.argtypes = [ctypes.POINTER(sk_bloom_record), ctypes.c_size_t, ctypes.POINTER(sk_bloom_params), ctypes.POINTER(_vp)]
_lib.bloom_insert.argtypes = [_vp, ctypes.POINTER(sk_bloom_record)]
_lib.bloom_query.argtypes = [_vp, _i64, _i64, _i64, ctypes.POINTER(ctypes.c_uint32)]
_lib.bloom_query_many.argtypes = [_vp, ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint32)]
_lib.bloom_bits.argtypes = [_vp, _int, ctypes.POINTER(ctypes.POINTER(ctypes.c_uint64)), ctypes.POINTER(ctypes.c_size_t)]
_lib.bloom_winner_mask.argtypes = [ctypes.POINTER(ctypes.c_int64), ctypes.c_size_t, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32)]
_lib.bloom_serialize.argtypes = [_vp, _vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
_lib.bloom_deserialize.argtypes = [_vp, ctypes.c_size_t, ctypes.POINTER(_vp)]
_lib.bloom_shape_key.argtypes = [_vp, ctypes.POINTER(ctypes.c_uint32)]
_lib.bloom_murmur3_32.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_uint32]
_lib.bloom_murmur3_32.restype = ctypes.c_uint32
_lib.bloom_destroy.argtypes = [_vp]
_lib.bloom_destroy.restype = None
_lib.sk_last_hip_error.restype = ctypes.c_char_p
_lib.sk_status_str.argtypes = [_int]
_lib.sk_status_str.restype = ctypes.c_char_p


class StreamKError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = " [%s]" % _lib.sk_last_hip_error().decode() if status == SK_ERR_HIP else ""
        super().__init__("%s: %s (%d)%s" % (where, sk_status_str(status), status, detail))


def _check(status, where):
    if status != SK_OK:
        raise StreamKError(status, where)


def sk_status_str(status):
    return _lib.sk_status_str(status).decode()


def sk_last_hip_error():
    return _lib.sk_last_hip_error().decode()


def sk_default_tile(M, N, K, in_dtype=SK_BF16):
    blk = (ctypes.c_int32 * 3)()
    _check(_lib.sk_default_tile(M, N, K, in_dtype, blk), "sk_default_tile")
    return tuple(blk)


def sk_plan(M, N, K, policy, blk=None, grid=0, in_dtype=None, out_dtype=None, tile_order=None):
    """Returns an opaque plan handle (int).  blk = (blk_m, blk_n, blk_k) or None for the default."""
    cfg = sk_config(*(blk or (0, 0, 0)), grid, 0 if in_dtype is None else in_dtype + 1,
                    0 if out_dtype is None else out_dtype + 1, 0 if tile_order is None else tile_order + 1)
    out = _vp()
    _check(_lib.sk_plan(M, N, K, policy, ctypes.byref(cfg), ctypes.byref(out)), "sk_plan")
    return out.value


def sk_plan_info(plan):
    h = sk_plan_header()
    _check(_lib.sk_plan_info(plan, ctypes.byref(h)), "sk_plan_info")
    return {n: getattr(h, n) for n, _ in sk_plan_header._fields_}


def sk_plan_ranges(plan):
    g = sk_plan_info(plan)["grid"]
    arr = (sk_wg_range * g)()
    _check(_lib.sk_plan_ranges(plan, arr), "sk_plan_ranges")
    return [(r.sk_iter_begin, r.sk_iter_end, r.dp_tile_first, r.dp_tile_count) for r in arr]


def sk_plan_segments(plan):
    n = ctypes.c_size_t()
    _lib.sk_plan_segments(plan, None, 0, ctypes.byref(n))
    arr = (sk_segment * max(n.value, 1))()
    _check(_lib.sk_plan_segments(plan, arr, n.value, ctypes.byref(n)), "sk_plan_segments")
    return [(s.wg, s.tile, s.k_begin, s.k_end, s.role) for s in arr[:n.value]]


def sk_plan_tile_coords(plan, tile):
    tm, tn = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.sk_plan_tile_coords(plan, tile, ctypes.byref(tm), ctypes.byref(tn)), "sk_plan_tile_coords")
    return tm.value, tn.value


def sk_workspace_bytes(plan):
    return _lib.sk_workspace_bytes(plan)


def sk_plan_set_workspace(plan, dev_ptr, nbytes):
    _check(_lib.sk_plan_set_workspace(plan, dev_ptr, nbytes), "sk_plan_set_workspace")


def sk_plan_set_fixup(plan, fixup):
    _check(_lib.sk_plan_set_fixup(plan, fixup), "sk_plan_set_fixup")


def sk_plan_set_batch_order(plan, batch_order):
    _check(_lib.sk_plan_set_batch_order(plan, batch_order), "sk_plan_set_batch_order")


def sk_plan_estimate_us(plan):
    us = ctypes.c_double()
    _check(_lib.sk_plan_estimate_us(plan, ctypes.byref(us)), "sk_plan_estimate_us")
    return us.value


def sk_plan_set_segment_order(plan, segment_order):
    _check(_lib.sk_plan_set_segment_order(plan, segment_order), "sk_plan_set_segment_order")


def sk_plan_set_spin_limit(plan, polls):
    _check(_lib.sk_plan_set_spin_limit(plan, polls), "sk_plan_set_spin_limit")


def sk_plan_set_kernel_variant(plan, variant):
    _check(_lib.sk_plan_set_kernel_variant(plan, variant), "sk_plan_set_kernel_variant")


def sk_gemm(A_ptr, B_ptr, D_ptr, plan, stream=0):
    """Device pointers (ints) and a hipStream_t (int).  Asynchronous."""
    _check(_lib.sk_gemm(A_ptr, B_ptr, D_ptr, plan, stream), "sk_gemm")


def sk_mfma_peak_operand_bytes():
    return _lib.sk_mfma_peak_operand_bytes()


def sk_mfma_peak_launch(in_dtype, operands_ptr, sink_ptr, workgroups, iters, stream=0):
    """Enqueues the register-resident matrix-core loop; returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check(_lib.sk_mfma_peak_launch(in_dtype, operands_ptr, sink_ptr, workgroups, iters, stream, ctypes.byref(flops)), "sk_mfma_peak_launch")
    return flops.value


def sk_gemm_static(A_ptr, B_ptr, D_ptr, plan, stream=0):
    """sk_gemm with the workspace inside the library (no allocation anywhere on the call path)."""
    _check(_lib.sk_gemm_static(A_ptr, B_ptr, D_ptr, plan, stream), "sk_gemm_static")


def sk_gemm_bind(A_ptr, B_ptr, D_ptr, plan, stream=0):
    """The same call with its arguments marshalled once: returns a function of no arguments that
    enqueues the launch and returns the status code.  For loops that launch one problem many times
    (the per-call conversion of five integers costs about as much as the launch itself)."""
    import functools
    return functools.partial(_lib.sk_gemm, _vp(A_ptr), _vp(B_ptr), _vp(D_ptr), _vp(plan), _vp(stream))


def sk_gemm_status(A_ptr, B_ptr, D_ptr, plan, stream=0):
    """As sk_gemm but returns the status code instead of raising."""
    return _lib.sk_gemm(A_ptr, B_ptr, D_ptr, plan, stream)


def sk_plan_check(plan, stream=0):
    return _lib.sk_plan_check(plan, stream)


def sk_plan_kernel_info(plan):
    """{"threads", "lds_bytes", "variant"} of the kernel a launch of this plan would use now."""
    v = (ctypes.c_int32 * 3)()
    p = [ctypes.cast(ctypes.byref(v, 4 * i), ctypes.POINTER(ctypes.c_int32)) for i in range(3)]
    _check(_lib.sk_plan_kernel_info(plan, *p), "sk_plan_kernel_info")
    return {"threads": v[0], "lds_bytes": v[1], "variant": v[2]}


def sk_plan_destroy(plan):
    _lib.sk_plan_destroy(plan)


def bloom_winner_mask(times_ns, tol_permille):
    """Bit p set iff times_ns[p] is within tol_permille / 1000 of the fastest."""
    arr = (ctypes.c_int64 * len(times_ns))(*[int(t) for t in times_ns])
    mask = ctypes.c_uint32()
    _check(_lib.bloom_winner_mask(arr, len(times_ns), tol_permille, ctypes.byref(mask)), "bloom_winner_mask")
    return mask.value


def bloom_build(records, m_bits=0, k_probes=0, n_filters=0):
    """records: iterable of (M, N, K, policy_mask).  Returns an opaque handle (int)."""
    records = list(records)
    arr = (sk_bloom_record * max(len(records), 1))(*[sk_bloom_record(*r) for r in records])
    params = sk_bloom_params(m_bits, k_probes, n_filters)
    out = _vp()
    _check(_lib.bloom_build(arr, len(records), ctypes.byref(params), ctypes.byref(out)), "bloom_build")
    return out.value


def bloom_insert(bloom, M, N, K, policy_mask):
    rec = sk_bloom_record(M, N, K, policy_mask)
    _check(_lib.bloom_insert(bloom, ctypes.byref(rec)), "bloom_insert")


def bloom_query(bloom, M, N, K):
    mask = ctypes.c_uint32()
    _check(_lib.bloom_query(bloom, M, N, K, ctypes.byref(mask)), "bloom_query")
    return mask.value


def bloom_query_many(bloom, sizes):
    """sizes: sequence of (M, N, K).  Returns the list of candidate masks."""
    flat = [int(v) for s in sizes for v in s]
    arr = (ctypes.c_uint32 * max(len(flat), 1))(*flat)
    out = (ctypes.c_uint32 * max(len(sizes), 1))()
    _check(_lib.bloom_query_many(bloom, arr, len(sizes), out), "bloom_query_many")
    return list(out[:len(sizes)])


def bloom_bits(bloom, filt):
    words = ctypes.POINTER(ctypes.c_uint64)()
    n = ctypes.c_size_t()
    _check(_lib.bloom_bits(bloom, filt, ctypes.byref(words), ctypes.byref(n)), "bloom_bits")
    return [words[i] for i in range(n.value)]


def bloom_serialize(bloom):
    """The filters as bytes."""
    n = ctypes.c_size_t()
    _check(_lib.bloom_serialize(bloom, None, 0, ctypes.byref(n)), "bloom_serialize")
    buf = (ctypes.c_ubyte * n.value)()
    _check(_lib.bloom_serialize(bloom, buf, n.value, ctypes.byref(n)), "bloom_serialize")
    return bytes(buf)


def bloom_deserialize(data):
    """New filters (opaque handle) from bloom_serialize's bytes."""
    out = _vp()
    buf = (ctypes.c_ubyte * len(data)).from_buffer_copy(data)
    _check(_lib.bloom_deserialize(buf, len(data), ctypes.byref(out)), "bloom_deserialize")
    return out.value


def bloom_shape_key(plan):
    key = (ctypes.c_uint32 * 3)()
    _check(_lib.bloom_shape_key(plan, key), "bloom_shape_key")
    return tuple(key)


def bloom_murmur3_32(key, seed):
    return _lib.bloom_murmur3_32(key, len(key), seed)


def bloom_destroy(bloom):
    _lib.bloom_destroy(bloom)
