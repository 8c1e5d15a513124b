"""ctypes binding of libtpla.so: argument marshalling only.

Every function has the name and argument order of its C counterpart in
include/tpla.h.  Tensor arguments may be torch tensors (their data_ptr() is
passed; they must be contiguous) or plain integers (raw addresses).  The
stream is torch's current stream unless given.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
# TPLA_LIBRARY selects another build of the same library (e.g. a measurement build made with
# TPLA_LIB_NAME=... python -m paper_2508_15881_amd.build); there is still no fallback.
_LIB_PATH = os.environ.get("TPLA_LIBRARY") or os.path.join(_PKG, "lib", "libtpla.so")

TPLA_F32, TPLA_BF16 = 0, 1
TPLA_U_IDENTITY, TPLA_U_HADAMARD, TPLA_U_DENSE = 0, 1, 2
TPLA_MAX_G = 8

EXPORTS = (
    "tpla_last_error", "tpla_version", "tpla_transform_latent", "tpla_transform_latent_paged",
    "tpla_write_mla_cache", "tpla_absorb_query", "tpla_workspace_bytes", "tpla_decode_shard",
    "tpla_combine_shards", "tpla_profile_enable", "tpla_profile_collect", "tpla_workspace_bytes_all",
    "tpla_decode_shards", "tpla_append_token_sliced", "tpla_output_projection",
    "tpla_output_projection_workspace_bytes", "tpla_latent_moments_workspace_bytes", "tpla_latent_moments",
    "tpla_pca_basis", "tpla_prefill_workspace_bytes", "tpla_prefill_attention", "tpla_stream_read",
    "tpla_decode_shards_combine", "tpla_validate_block_table", "tpla_decode_shards_combine_static",
    "tpla_combine_shards_to", "tpla_decode_shards_combine_to", "tpla_output_projection_to",
    "tpla_attention_block_workspace_bytes", "tpla_decode_shards_project",
)


class TplaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libtpla error %d: %s" % (code, msg))
        self.code = code


class TplaShape(ctypes.Structure):
    """Mirror of tpla_shape_t."""
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d_c", ctypes.c_int32), ("g", ctypes.c_int32),
        ("d_r", ctypes.c_int32), ("d_n", ctypes.c_int32), ("d_v", ctypes.c_int32),
        ("page_tokens", ctypes.c_int32), ("dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
    ]

    @property
    def dl(self):
        return self.d_c // self.g


_lib = None


def lib_path():
    return _LIB_PATH


def load_library():
    """Loads libtpla.so once.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libtpla.so not found at %s -- build it with `python -m paper_2508_15881_amd.build`" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, fp = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(ctypes.c_float)
    shp = ctypes.POINTER(TplaShape)
    lib.tpla_last_error.restype = ctypes.c_char_p
    lib.tpla_last_error.argtypes = []
    lib.tpla_version.restype = ctypes.c_int
    lib.tpla_version.argtypes = []
    lib.tpla_transform_latent.restype = ctypes.c_int
    lib.tpla_transform_latent.argtypes = [shp, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, i64, i64, vp]
    lib.tpla_transform_latent_paged.restype = ctypes.c_int
    lib.tpla_transform_latent_paged.argtypes = [shp, ctypes.c_int, vp, vp, vp, ctypes.POINTER(vp), vp, i64, vp]
    lib.tpla_write_mla_cache.restype = ctypes.c_int
    lib.tpla_write_mla_cache.argtypes = [shp, vp, vp, vp, i64, ctypes.c_float, vp, vp]
    lib.tpla_output_projection_workspace_bytes.restype = ctypes.c_size_t
    lib.tpla_output_projection_workspace_bytes.argtypes = [shp, i32]
    lib.tpla_output_projection.restype = ctypes.c_int
    lib.tpla_output_projection.argtypes = [shp, vp, vp, i32, vp, ctypes.c_size_t, vp, vp]
    lib.tpla_append_token_sliced.restype = ctypes.c_int
    lib.tpla_append_token_sliced.argtypes = [shp, vp, vp, fp, ctypes.c_float, vp, ctypes.POINTER(vp), vp]
    lib.tpla_absorb_query.restype = ctypes.c_int
    lib.tpla_absorb_query.argtypes = [shp, vp, vp, fp, vp, vp]
    lib.tpla_workspace_bytes.restype = ctypes.c_size_t
    lib.tpla_workspace_bytes.argtypes = [shp, i32, i32]
    lib.tpla_decode_shard.restype = ctypes.c_int
    lib.tpla_decode_shard.argtypes = [shp, vp, vp, vp, vp, i32, vp, i32, vp, ctypes.c_size_t, vp, vp, vp]
    lib.tpla_workspace_bytes_all.restype = ctypes.c_size_t
    lib.tpla_workspace_bytes_all.argtypes = [shp, i32, i32]
    lib.tpla_decode_shards.restype = ctypes.c_int
    lib.tpla_decode_shards.argtypes = [shp, vp, vp, ctypes.POINTER(vp), vp, i32, vp, i32, vp, ctypes.c_size_t, vp, vp, vp]
    lib.tpla_decode_shards_combine.restype = ctypes.c_int
    lib.tpla_decode_shards_combine.argtypes = [shp, vp, vp, ctypes.POINTER(vp), vp, i32, vp, i32, vp, ctypes.c_size_t,
                                               vp, vp, vp, vp, vp]
    lib.tpla_decode_shards_combine_static.restype = ctypes.c_int
    lib.tpla_decode_shards_combine_static.argtypes = [shp, vp, vp, ctypes.POINTER(vp), vp, i32, vp, i32,
                                                      vp, vp, vp, vp, vp]
    lib.tpla_combine_shards_to.restype = ctypes.c_int
    lib.tpla_combine_shards_to.argtypes = [shp, vp, vp, vp, i32, vp]
    lib.tpla_decode_shards_combine_to.restype = ctypes.c_int
    lib.tpla_decode_shards_combine_to.argtypes = [shp, vp, vp, ctypes.POINTER(vp), vp, i32, vp, i32, vp, ctypes.c_size_t,
                                                  vp, vp, i32, vp, vp, vp]
    lib.tpla_output_projection_to.restype = ctypes.c_int
    lib.tpla_output_projection_to.argtypes = [shp, vp, vp, i32, vp, ctypes.c_size_t, vp, i32, vp]
    lib.tpla_attention_block_workspace_bytes.restype = ctypes.c_size_t
    lib.tpla_attention_block_workspace_bytes.argtypes = [shp, i32, i32, i32]
    lib.tpla_decode_shards_project.restype = ctypes.c_int
    lib.tpla_decode_shards_project.argtypes = [shp, vp, vp, ctypes.POINTER(vp), vp, i32, vp, i32, vp, ctypes.c_size_t,
                                               vp, vp, i32, vp, i32, vp, vp, vp, vp]
    lib.tpla_combine_shards.restype = ctypes.c_int
    lib.tpla_combine_shards.argtypes = [shp, vp, vp, vp, vp]
    lib.tpla_profile_enable.restype = ctypes.c_int
    lib.tpla_profile_enable.argtypes = [i32]
    lib.tpla_profile_collect.restype = ctypes.c_int
    lib.tpla_profile_collect.argtypes = [fp, i32, ctypes.POINTER(i32)]
    lib.tpla_latent_moments_workspace_bytes.restype = ctypes.c_size_t
    lib.tpla_latent_moments_workspace_bytes.argtypes = [shp, i64]
    lib.tpla_latent_moments.restype = ctypes.c_int
    lib.tpla_latent_moments.argtypes = [shp, vp, vp, vp, i64, vp, ctypes.c_size_t, vp, vp, vp]
    lib.tpla_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.tpla_prefill_workspace_bytes.argtypes = [shp, i64]
    lib.tpla_prefill_attention.restype = ctypes.c_int
    lib.tpla_prefill_attention.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i64, i32, vp, ctypes.c_size_t, vp, vp]
    lib.tpla_stream_read.restype = ctypes.c_int
    lib.tpla_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.tpla_validate_block_table.restype = ctypes.c_int
    lib.tpla_validate_block_table.argtypes = [shp, vp, i32, vp, i64, ctypes.c_int]
    lib.tpla_pca_basis.restype = ctypes.c_int
    lib.tpla_pca_basis.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


def _ptr(x):
    """Address of a tensor / raw address / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise ValueError("libtpla needs contiguous tensors")
    return x.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    if torch.cuda.is_available():
        return torch.cuda.current_stream().cuda_stream
    return None


def _check(rc):
    if rc != 0:
        raise TplaError(rc, tpla_last_error())


def tpla_last_error():
    return load_library().tpla_last_error().decode()


def tpla_version():
    return load_library().tpla_version()


def tpla_transform_latent(shape, mode, inverse, signs, U, src, dst, n_outer, n_inner, stream=None):
    _check(load_library().tpla_transform_latent(
        ctypes.byref(shape), mode, inverse, _ptr(signs), _ptr(U), _ptr(src), _ptr(dst),
        n_outer, n_inner, _stream(stream)))


def tpla_transform_latent_paged(shape, mode, signs, U, mla_pool, shard_pools, page_ids, n_pages, stream=None):
    if shard_pools is None:
        arr = None
    else:
        # never read past g entries on the C side; sized generously so a
        # wrong-length list is reported by the library, not by ctypes
        arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
        for i, p in enumerate(shard_pools):
            arr[i] = _ptr(p)
    _check(load_library().tpla_transform_latent_paged(
        ctypes.byref(shape), mode, _ptr(signs), _ptr(U), _ptr(mla_pool), arr, _ptr(page_ids),
        n_pages, _stream(stream)))


def tpla_write_mla_cache(shape, c_raw, k_pe, slot_mapping, T, rms_eps, mla_pool, stream=None):
    _check(load_library().tpla_write_mla_cache(
        ctypes.byref(shape), _ptr(c_raw), _ptr(k_pe), _ptr(slot_mapping), T, rms_eps, _ptr(mla_pool),
        _stream(stream)))


def tpla_append_token_sliced(shape, c_t, k_pe, alpha, rms_eps, slots, shard_pools, stream=None):
    a_arr = None
    if alpha is not None:
        a_arr = (ctypes.c_float * max(TPLA_MAX_G, len(alpha)))(*[float(a) for a in alpha])
    if shard_pools is None:
        arr = None
    else:
        arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
        for i, p in enumerate(shard_pools):
            arr[i] = _ptr(p)
    _check(load_library().tpla_append_token_sliced(
        ctypes.byref(shape), _ptr(c_t), _ptr(k_pe), a_arr, rms_eps, _ptr(slots), arr, _stream(stream)))


def tpla_absorb_query(shape, q_nope, W_UK_t, mu, q_lat, stream=None):
    mu_arr = None
    if mu is not None:
        mu_arr = (ctypes.c_float * max(TPLA_MAX_G, len(mu)))(*[float(m) for m in mu])
    _check(load_library().tpla_absorb_query(
        ctypes.byref(shape), _ptr(q_nope), _ptr(W_UK_t), mu_arr, _ptr(q_lat), _stream(stream)))


def tpla_workspace_bytes(shape, max_pages_per_seq, n_splits):
    return int(load_library().tpla_workspace_bytes(ctypes.byref(shape), max_pages_per_seq, n_splits))


def tpla_decode_shard(shape, q_lat_i, q_pe, shard_pool, block_table, max_pages_per_seq, seq_lens,
                      n_splits, workspace, workspace_bytes, o_lat_i, lse_i, stream=None):
    _check(load_library().tpla_decode_shard(
        ctypes.byref(shape), _ptr(q_lat_i), _ptr(q_pe), _ptr(shard_pool), _ptr(block_table),
        max_pages_per_seq, _ptr(seq_lens), n_splits, _ptr(workspace), workspace_bytes,
        _ptr(o_lat_i), _ptr(lse_i), _stream(stream)))


def tpla_workspace_bytes_all(shape, max_pages_per_seq, n_splits):
    return int(load_library().tpla_workspace_bytes_all(ctypes.byref(shape), max_pages_per_seq, n_splits))


def tpla_decode_shards(shape, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                       n_splits, workspace, workspace_bytes, o_lat, lse, stream=None):
    if shard_pools is None:
        arr = None
    else:
        arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
        for i, p in enumerate(shard_pools):
            arr[i] = _ptr(p)
    _check(load_library().tpla_decode_shards(
        ctypes.byref(shape), _ptr(q_lat), _ptr(q_pe), arr, _ptr(block_table), max_pages_per_seq,
        _ptr(seq_lens), n_splits, _ptr(workspace), workspace_bytes, _ptr(o_lat), _ptr(lse), _stream(stream)))


def tpla_decode_shards_combine(shape, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                               n_splits, workspace, workspace_bytes, W_UV_t, o, o_lat, lse, stream=None):
    if shard_pools is None:
        arr = None
    else:
        arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
        for i, p in enumerate(shard_pools):
            arr[i] = _ptr(p)
    _check(load_library().tpla_decode_shards_combine(
        ctypes.byref(shape), _ptr(q_lat), _ptr(q_pe), arr, _ptr(block_table), max_pages_per_seq,
        _ptr(seq_lens), n_splits, _ptr(workspace), workspace_bytes, _ptr(W_UV_t), _ptr(o), _ptr(o_lat), _ptr(lse),
        _stream(stream)))


def tpla_decode_shards_combine_static(shape, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                                      n_splits, W_UV_t, o, o_lat, lse, stream=None):
    if shard_pools is None:
        arr = None
    else:
        arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
        for i, p in enumerate(shard_pools):
            arr[i] = _ptr(p)
    _check(load_library().tpla_decode_shards_combine_static(
        ctypes.byref(shape), _ptr(q_lat), _ptr(q_pe), arr, _ptr(block_table), max_pages_per_seq,
        _ptr(seq_lens), n_splits, _ptr(W_UV_t), _ptr(o), _ptr(o_lat), _ptr(lse), _stream(stream)))


def _pool_array(shard_pools):
    if shard_pools is None:
        return None
    arr = (ctypes.c_void_p * max(TPLA_MAX_G, len(shard_pools)))()
    for i, p in enumerate(shard_pools):
        arr[i] = _ptr(p)
    return arr


def tpla_combine_shards_to(shape, o_lat, W_UV_t, o, o_dtype, stream=None):
    _check(load_library().tpla_combine_shards_to(
        ctypes.byref(shape), _ptr(o_lat), _ptr(W_UV_t), _ptr(o), o_dtype, _stream(stream)))


def tpla_decode_shards_combine_to(shape, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                                  n_splits, workspace, workspace_bytes, W_UV_t, o, o_dtype, o_lat, lse, stream=None):
    _check(load_library().tpla_decode_shards_combine_to(
        ctypes.byref(shape), _ptr(q_lat), _ptr(q_pe), _pool_array(shard_pools), _ptr(block_table), max_pages_per_seq,
        _ptr(seq_lens), n_splits, _ptr(workspace), workspace_bytes, _ptr(W_UV_t), _ptr(o), o_dtype, _ptr(o_lat),
        _ptr(lse), _stream(stream)))


def tpla_output_projection_to(shape, o, W_O, D, workspace, workspace_bytes, out, out_dtype, stream=None):
    _check(load_library().tpla_output_projection_to(
        ctypes.byref(shape), _ptr(o), _ptr(W_O), D, _ptr(workspace), workspace_bytes, _ptr(out), out_dtype,
        _stream(stream)))


def tpla_attention_block_workspace_bytes(shape, max_pages_per_seq, n_splits, D):
    return int(load_library().tpla_attention_block_workspace_bytes(ctypes.byref(shape), max_pages_per_seq, n_splits, D))


def tpla_decode_shards_project(shape, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens, n_splits,
                               workspace, workspace_bytes, W_UV_t, W_O, D, out, out_dtype, o, o_lat, lse, stream=None):
    _check(load_library().tpla_decode_shards_project(
        ctypes.byref(shape), _ptr(q_lat), _ptr(q_pe), _pool_array(shard_pools), _ptr(block_table), max_pages_per_seq,
        _ptr(seq_lens), n_splits, _ptr(workspace), workspace_bytes, _ptr(W_UV_t), _ptr(W_O), D, _ptr(out), out_dtype,
        _ptr(o), _ptr(o_lat), _ptr(lse), _stream(stream)))


def tpla_combine_shards(shape, o_lat, W_UV_t, o, stream=None):
    _check(load_library().tpla_combine_shards(
        ctypes.byref(shape), _ptr(o_lat), _ptr(W_UV_t), _ptr(o), _stream(stream)))


def tpla_output_projection_workspace_bytes(shape, D):
    return int(load_library().tpla_output_projection_workspace_bytes(ctypes.byref(shape), D))


def tpla_output_projection(shape, o, W_O, D, workspace, workspace_bytes, out, stream=None):
    _check(load_library().tpla_output_projection(
        ctypes.byref(shape), _ptr(o), _ptr(W_O), D, _ptr(workspace), workspace_bytes, _ptr(out), _stream(stream)))


def tpla_prefill_workspace_bytes(shape, T):
    return int(load_library().tpla_prefill_workspace_bytes(ctypes.byref(shape), T))


def tpla_prefill_attention(shape, q_nope, q_pe, c, k_pe, W_UK, W_UV, cu_seqlens, T, max_seq_len, workspace,
                           workspace_bytes, o, stream=None):
    _check(load_library().tpla_prefill_attention(
        ctypes.byref(shape), _ptr(q_nope), _ptr(q_pe), _ptr(c), _ptr(k_pe), _ptr(W_UK), _ptr(W_UV), _ptr(cu_seqlens),
        T, max_seq_len, _ptr(workspace), workspace_bytes, _ptr(o), _stream(stream)))


def tpla_latent_moments_workspace_bytes(shape, n_pages):
    return int(load_library().tpla_latent_moments_workspace_bytes(ctypes.byref(shape), n_pages))


def tpla_latent_moments(shape, mla_pool, page_ids, page_fill, n_pages, workspace, workspace_bytes, sum_out, gram_out,
                        stream=None):
    _check(load_library().tpla_latent_moments(
        ctypes.byref(shape), _ptr(mla_pool), _ptr(page_ids), _ptr(page_fill), n_pages, _ptr(workspace),
        workspace_bytes, _ptr(sum_out), _ptr(gram_out), _stream(stream)))


def tpla_pca_basis(d_c, g, n_rows, sum_host, gram_host):
    """Host call.  sum_host [d_c], gram_host [d_c, d_c]: C-contiguous float64 numpy arrays.
    Returns (U float32 [d_c, d_c], eigenvalues float64 [d_c], fractions float64 [g])."""
    import numpy as np
    sum_host = np.ascontiguousarray(sum_host, dtype=np.float64)
    gram_host = np.ascontiguousarray(gram_host, dtype=np.float64)
    if sum_host.shape != (d_c,) or gram_host.shape != (d_c, d_c):
        raise ValueError("sum must be [d_c] and gram [d_c, d_c]")
    U = np.empty((d_c, d_c), dtype=np.float32)
    eig = np.empty(d_c, dtype=np.float64)
    frac = np.empty(g, dtype=np.float64)
    _check(load_library().tpla_pca_basis(d_c, g, n_rows, sum_host.ctypes.data, gram_host.ctypes.data,
                                         U.ctypes.data, eig.ctypes.data, frac.ctypes.data))
    return U, eig, frac


def tpla_validate_block_table(shape, block_table_host, max_pages_per_seq, seq_lens_host, n_pool_pages,
                              forbid_shared=False):
    """Host call.  block_table_host [B, max_pages_per_seq], seq_lens_host [B]: int32 numpy arrays
    (or None, to exercise the argument checks).  Raises TplaError naming the first bad entry."""
    import numpy as np
    bt = None if block_table_host is None else np.ascontiguousarray(block_table_host, dtype=np.int32)
    ln = None if seq_lens_host is None else np.ascontiguousarray(seq_lens_host, dtype=np.int32)
    if bt is not None and ln is not None and (bt.shape != (shape.B, max_pages_per_seq) or ln.shape != (shape.B,)):
        raise ValueError("block_table must be [B, max_pages_per_seq] and seq_lens [B]")
    _check(load_library().tpla_validate_block_table(
        ctypes.byref(shape), None if bt is None else bt.ctypes.data, max_pages_per_seq,
        None if ln is None else ln.ctypes.data, n_pool_pages, 1 if forbid_shared else 0))


def tpla_stream_read(buf, nbytes, sink, stream=None):
    _check(load_library().tpla_stream_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream)))


def tpla_profile_enable(max_records):
    _check(load_library().tpla_profile_enable(max_records))


def tpla_profile_collect(capacity):
    """Elapsed milliseconds of every bracketed split kernel since the last collect."""
    buf = (ctypes.c_float * max(1, capacity))()
    n = ctypes.c_int32(0)
    _check(load_library().tpla_profile_collect(buf, capacity, ctypes.byref(n)))
    return [buf[i] for i in range(n.value)]
