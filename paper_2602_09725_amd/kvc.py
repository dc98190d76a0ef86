"""ctypes binding of libkvc.so: same names and argument order as include/kvc.h.

Tensors are passed as device pointers (`tensor.data_ptr()`), streams as
`torch.cuda.Stream.cuda_stream` handles; torch is used for nothing else.
"""
import ctypes as C
import os

KVC_F16, KVC_BF16 = 0, 1
KVC_Q_PER_CHANNEL, KVC_Q_PER_TOKEN = 0, 1
KVC_ORDER_CHUNK, KVC_ORDER_LAYER = 0, 1
KVC_ABI_VERSION = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvc.so")
_lib = None


class KvcError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {status_str(status)} (kvc_status {status})")
        self.status = status


class Layout(C.Structure):
    """kvc_layout"""
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32)] + [
        (n, C.c_int32) for n in ("num_layers", "num_kv_heads", "head_dim", "dtype", "chunk_tokens", "tile_h", "tile_w",
                                 "tiles_x", "tiles_y", "k_mode", "v_mode", "tile_seg")]

    def __init__(self, num_layers, num_kv_heads, head_dim, dtype, chunk_tokens, tile_h, tile_w, tiles_x, tiles_y,
                 k_mode=KVC_Q_PER_CHANNEL, v_mode=KVC_Q_PER_TOKEN, tile_seg=0):
        super().__init__(C.sizeof(Layout), KVC_ABI_VERSION, num_layers, num_kv_heads, head_dim, dtype, chunk_tokens,
                         tile_h, tile_w, tiles_x, tiles_y, k_mode, v_mode, tile_seg)


class Strides(C.Structure):
    """kvc_strides (elements)"""
    _fields_ = [("layer_stride", C.c_int64), ("kv_stride", C.c_int64), ("token_stride", C.c_int64)]


class HostChunk(C.Structure):
    """kvc_host_chunk"""
    _fields_ = [("host_blob", C.c_void_p), ("bytes", C.c_size_t), ("n_tokens", C.c_int64)]


def lib_path():
    return _LIB_PATH


def load(path=None):
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    p = path or _LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it with `python -m paper_2602_09725_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(p)
    LP, vp, i64, i32, sz = C.POINTER(Layout), C.c_void_p, C.c_int64, C.c_int32, C.c_size_t
    lib.kvc_status_str.argtypes = [C.c_int]
    lib.kvc_status_str.restype = C.c_char_p
    lib.kvc_build_id.argtypes = []
    lib.kvc_build_id.restype = C.c_char_p
    lib.kvc_layout_validate.argtypes = [LP]
    lib.kvc_chunk_sizes.argtypes = [LP, C.POINTER(sz), C.POINTER(sz), C.POINTER(i32)]
    lib.kvc_blob_meta_offset.argtypes = [LP]
    lib.kvc_blob_meta_offset.restype = sz
    lib.kvc_pack.argtypes = [LP, vp, Strides, i64, vp, sz, vp, sz, vp]
    lib.kvc_pack_plan.argtypes = [LP, Strides, C.POINTER(i32), C.POINTER(i32)]
    lib.kvc_restore.argtypes = [LP, vp, vp, i64, vp, Strides, vp]
    lib.kvc_restore_paged.argtypes = [LP, vp, vp, i64, i64, vp, i64, i32, vp, i64, vp, vp]
    lib.kvc_fetch_pipeline.argtypes = [LP, C.POINTER(HostChunk), i32, C.POINTER(vp), sz, i32, vp, i64, i32, vp, i64,
                                       vp, vp, vp, C.POINTER(C.c_float)]
    lib.kvc_restore_paged_frame.argtypes = [LP, vp, vp, i32, i32, i32, i64, i64, vp, i64, i32, vp, i64, vp, vp]
    lib.kvc_restore_paged_frames.argtypes = [LP, vp, vp, i64, i64, i64, i64, vp, i64, i32, vp, i64, vp, vp]
    lib.kvc_frame_size.argtypes = [LP]
    lib.kvc_frame_size.restype = sz
    lib.kvc_frame_offset.argtypes = [LP, i32, i32, i32]
    lib.kvc_frame_offset.restype = sz
    lib.kvc_fetch_pipeline_frames.argtypes = [LP, C.POINTER(HostChunk), i32, C.POINTER(vp), sz, i32, C.POINTER(vp), sz, i32,
                                              vp, i64, i32, vp, i64, vp, vp, vp, i32, C.POINTER(vp),
                                              C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.kvc_meta_staging_size.argtypes = [LP, i32]
    lib.kvc_meta_staging_size.restype = sz
    dp = C.POINTER(C.c_double)
    lib.kvc_select_resolution.argtypes = [dp, dp, dp, i32, i32, i32, i32, C.c_double, dp]
    lib.kvc_select_resolution.restype = i32
    lib.kvc_est_bandwidth.argtypes = [C.c_double, C.c_double]
    lib.kvc_est_bandwidth.restype = C.c_double
    lib.kvc_layout_set_resolution.argtypes = [LP, i32, i32]
    lib.kvc_admission_ok.argtypes = [dp, dp, i32, i32]
    lib.kvc_admission_ok.restype = i32
    lib.kvc_admission_min_buffered.argtypes = [dp, dp, i32]
    lib.kvc_admission_min_buffered.restype = i32
    lib.kvc_residual_histograms_size.argtypes = [LP, i64]
    lib.kvc_residual_histograms_size.restype = sz
    lib.kvc_residual_histograms.argtypes = [LP, vp, i64, vp, sz, vp]
    lib.kvc_proxy_cost_bits.argtypes = [LP, vp, i64]
    lib.kvc_proxy_cost_bits.restype = C.c_double
    ip = C.POINTER(i32)
    lib.kvc_tile_candidates.argtypes = [i32, i32, ip, ip, ip, i32]
    lib.kvc_tile_candidates.restype = i32
    lib.kvc_probe_expand.argtypes = [vp, vp, sz, vp, sz, i32, i32, vp]
    if path is None:
        _lib = lib
    return lib


def build_id():
    return load().kvc_build_id().decode()


def status_str(status):
    return load().kvc_status_str(int(status)).decode()


def _check(status, what):
    if status != 0:
        raise KvcError(status, what)


def layout_validate(layout):
    return load().kvc_layout_validate(C.byref(layout))


def chunk_sizes(layout):
    """-> (frame_bytes, meta_bytes, frames_per_group) of one chunk section."""
    fb, mb, f = C.c_size_t(), C.c_size_t(), C.c_int32()
    _check(load().kvc_chunk_sizes(C.byref(layout), C.byref(fb), C.byref(mb), C.byref(f)), "kvc_chunk_sizes")
    return fb.value, mb.value, f.value


def pack_plan(layout, strides):
    """-> (resident, threads): how kvc_pack would run (host arithmetic only)."""
    r, t = C.c_int32(), C.c_int32()
    _check(load().kvc_pack_plan(C.byref(layout), Strides(*strides), C.byref(r), C.byref(t)), "kvc_pack_plan")
    return r.value, t.value


def blob_meta_offset(layout):
    return load().kvc_blob_meta_offset(C.byref(layout))


def kvc_pack(layout, kv_ptr, strides, n_tokens, frames_ptr, frames_cap, meta_ptr, meta_cap, stream=0):
    _check(load().kvc_pack(C.byref(layout), kv_ptr, Strides(*strides), n_tokens, frames_ptr, frames_cap, meta_ptr,
                           meta_cap, stream), "kvc_pack")


def kvc_restore(layout, frames_ptr, meta_ptr, n_tokens, out_ptr, strides, stream=0):
    _check(load().kvc_restore(C.byref(layout), frames_ptr, meta_ptr, n_tokens, out_ptr, Strides(*strides), stream),
           "kvc_restore")


def kvc_restore_paged(layout, frames_ptr, meta_ptr, first_token, n_tokens, layer_cache_ptrs_dev, num_blocks,
                      block_size, block_table_ptr, table_len, err_ptr=None, stream=0):
    _check(load().kvc_restore_paged(C.byref(layout), frames_ptr, meta_ptr, first_token, n_tokens,
                                    layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr, table_len, err_ptr,
                                    stream), "kvc_restore_paged")


PROBE_ONE_XCD_PER_PIECE, PROBE_LINE_READS = 1, 2


def kvc_probe_expand(src_ptr, dst_ptr, out_bytes, piece_map_ptr, piece_bytes, wg_bytes, stream=0, shape=0):
    _check(load().kvc_probe_expand(src_ptr, dst_ptr, out_bytes, piece_map_ptr, piece_bytes, wg_bytes, shape, stream),
           "kvc_probe_expand")


N_RESIDUALS = 5


def residual_histograms_size(layout, n_chunks):
    return load().kvc_residual_histograms_size(C.byref(layout), n_chunks)


def kvc_residual_histograms(layout, frames_ptr, n_chunks, hist_ptr, hist_cap, stream=0):
    _check(load().kvc_residual_histograms(C.byref(layout), frames_ptr, n_chunks, hist_ptr, hist_cap, stream),
           "kvc_residual_histograms")


def proxy_cost_bits(layout, hist_host_ptr, n_chunks):
    """hist_host_ptr: address of the uint64 histogram array in host memory."""
    return load().kvc_proxy_cost_bits(C.byref(layout), hist_host_ptr, n_chunks)


def tile_candidates(num_kv_heads, head_dim):
    """-> [(tile_h, tile_w, tile_seg)] of the tilings rules i-iii of Sec. 3.2.2 leave."""
    n = load().kvc_tile_candidates(num_kv_heads, head_dim, None, None, None, 0)
    if n < 0:
        raise KvcError(1, "kvc_tile_candidates")
    th, tw, seg = (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_int32 * n)()
    load().kvc_tile_candidates(num_kv_heads, head_dim, th, tw, seg, n)
    return [(th[i], tw[i], seg[i]) for i in range(n)]


def kvc_fetch_pipeline(layout, chunks, staging_ptrs, staging_bytes, layer_cache_ptrs_dev, num_blocks, block_size,
                       block_table_ptr, table_len, err_ptr, copy_stream, compute_stream, timed=True):
    """chunks: list of (host_ptr, bytes, n_tokens).  Returns fetch-to-ready ms when timed, else None."""
    arr = (HostChunk * len(chunks))(*[HostChunk(p, b, n) for p, b, n in chunks])
    st = (C.c_void_p * len(staging_ptrs))(*staging_ptrs)
    ms = C.c_float(0.0)
    _check(load().kvc_fetch_pipeline(C.byref(layout), arr, len(chunks), st, staging_bytes, len(staging_ptrs),
                                     layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr, table_len, err_ptr,
                                     copy_stream, compute_stream, C.byref(ms) if timed else None),
           "kvc_fetch_pipeline")
    return ms.value if timed else None


def frame_size(layout):
    return load().kvc_frame_size(C.byref(layout))


def frame_offset(layout, kind, layer_group, frame_index):
    return load().kvc_frame_offset(C.byref(layout), kind, layer_group, frame_index)


def kvc_restore_paged_frame(layout, frame_ptr, meta_ptr, kind, layer_group, frame_index, first_token, n_tokens,
                            layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr, table_len, err_ptr=None,
                            stream=0):
    _check(load().kvc_restore_paged_frame(C.byref(layout), frame_ptr, meta_ptr, kind, layer_group, frame_index,
                                          first_token, n_tokens, layer_cache_ptrs_dev, num_blocks, block_size,
                                          block_table_ptr, table_len, err_ptr, stream), "kvc_restore_paged_frame")


def kvc_restore_paged_frames(layout, frames_ptr, meta_ptr, first_frame, n_frames, first_token, n_tokens,
                             layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr, table_len, err_ptr=None,
                             stream=0):
    _check(load().kvc_restore_paged_frames(C.byref(layout), frames_ptr, meta_ptr, first_frame, n_frames, first_token,
                                           n_tokens, layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr,
                                           table_len, err_ptr, stream), "kvc_restore_paged_frames")


def meta_staging_size(layout, order):
    return load().kvc_meta_staging_size(C.byref(layout), order)


def kvc_fetch_pipeline_frames(layout, chunks, frame_staging_ptrs, frame_staging_bytes, meta_staging_ptrs,
                              meta_staging_bytes, layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr,
                              table_len, err_ptr, copy_stream, compute_stream, order=KVC_ORDER_CHUNK,
                              group_ready_events=None, timed=True, group_times=False):
    """chunks: list of (host_ptr, bytes, n_tokens); group_ready_events: list of LG hipEvent_t handles or None.
    Returns fetch-to-ready ms when timed (with the list of per-layer-group ready times when group_times), else None."""
    arr = (HostChunk * len(chunks))(*[HostChunk(p, b, n) for p, b, n in chunks])
    fs = (C.c_void_p * len(frame_staging_ptrs))(*frame_staging_ptrs)
    ms_ = (C.c_void_p * len(meta_staging_ptrs))(*meta_staging_ptrs)
    ev = (C.c_void_p * len(group_ready_events))(*group_ready_events) if group_ready_events is not None else None
    LG = (layout.num_layers + 2) // 3
    ms = C.c_float(0.0)
    gms = (C.c_float * max(LG, 1))() if group_times else None
    _check(load().kvc_fetch_pipeline_frames(C.byref(layout), arr, len(chunks), fs, frame_staging_bytes,
                                            len(frame_staging_ptrs), ms_, meta_staging_bytes, len(meta_staging_ptrs),
                                            layer_cache_ptrs_dev, num_blocks, block_size, block_table_ptr, table_len,
                                            err_ptr, copy_stream, compute_stream, order, ev, gms,
                                            C.byref(ms) if timed else None),
           "kvc_fetch_pipeline_frames")
    if group_times:
        return (ms.value if timed else None), [gms[i] for i in range(LG)]
    return ms.value if timed else None


def _doubles(xs):
    return (C.c_double * len(xs))(*[float(x) for x in xs])


def admission_ok(t_fetch, t_comp, n_buffered):
    """Appx A.3 non-blocking condition; 1 / 0, or -1 on a bad argument."""
    n = len(t_fetch)
    if len(t_comp) != n:
        return -1
    return load().kvc_admission_ok(_doubles(t_fetch), _doubles(t_comp), n, n_buffered)


def admission_min_buffered(t_fetch, t_comp):
    n = len(t_fetch)
    if len(t_comp) != n:
        return -1
    return load().kvc_admission_min_buffered(_doubles(t_fetch), _doubles(t_comp), n)


def select_resolution(sizes, latency_rows, penalty, pool_load, active_res, bandwidth):
    """Alg. 1.  latency_rows[load - 1][r].  Returns (r_opt, bubble), or (-1, None) on a bad argument."""
    n_res, n_loads = len(sizes), len(latency_rows)
    if len(penalty) != n_res or any(len(row) != n_res for row in latency_rows):
        return -1, None
    flat = [x for row in latency_rows for x in row]
    bubble = C.c_double(0.0)
    r = load().kvc_select_resolution(_doubles(sizes), _doubles(flat), _doubles(penalty), n_res, n_loads, pool_load,
                                     active_res, float(bandwidth), C.byref(bubble))
    return (r, bubble.value) if r >= 0 else (-1, None)


def est_bandwidth(last_chunk_size, last_transmission_delay):
    return load().kvc_est_bandwidth(float(last_chunk_size), float(last_transmission_delay))


def layout_set_resolution(layout, width, height):
    """Sets the tile grid of `layout` for frames of at most width x height pixels; returns the status."""
    return load().kvc_layout_set_resolution(C.byref(layout), width, height)
