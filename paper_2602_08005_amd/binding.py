"""ctypes binding of libdeltakv.so: the same names as include/deltakv.h.

Argument marshalling only -- every step of the hot path runs inside the HIP
library.  There is no fallback: if the library is missing, import fails.
PyTorch tensors are used for device memory and streams (`data_ptr()`,
`torch.cuda.current_stream().cuda_stream`).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  imported BEFORE the library is loaded: libdeltakv must bind to the HIP runtime
              # that PyTorch ships (the streams and device pointers it is handed belong to that runtime)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeltakv.so")

OK, E_INVALID_ARG, E_UNSUPPORTED, E_WORKSPACE, E_HIP = 0, -1, -2, -3, -4
SPLIT, JOINT = 0, 1
METRIC_COSINE = 0
METRIC_L2 = 1


class Dims(C.Structure):
    _fields_ = [("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("rank", C.c_int32), ("latent_mode", C.c_int32), ("ref_stride", C.c_int32),
                ("page_tokens", C.c_int32), ("metric", C.c_int32),
                ("n_pages", C.c_int64), ("n_ref_slots", C.c_int64),
                ("latent_bits", C.c_int32), ("top_k", C.c_int32)]


class Mlp(C.Structure):
    """deltakv_mlp: the non-linear compressor's weights (device pointers)."""
    _fields_ = [("kind", C.c_int32), ("hidden", C.c_int32), ("w1", C.c_void_p), ("wg", C.c_void_p),
                ("b1", C.c_void_p), ("w2", C.c_void_p)]


MLP_GELU, MLP_SWIGLU = 0, 1


class Layout(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "latent_pool_bytes", "idx_pool_bytes", "ref_pool_bytes", "ref_norm_pool_bytes",
        "latent_page_stride", "latent_head_stride", "latent_stream_stride",
        "idx_page_stride", "idx_head_stride", "idx_slot_stride",
        "ref_head_stride", "ref_kv_stride", "ref_slot_stride", "ref_norm_head_stride",
        "compress_ws_bytes", "decode_ws_bytes")] + [("n_streams", C.c_int32), ("alignment", C.c_int32)]


class DeltaKVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code == E_HIP or (code == E_WORKSPACE and where == "deltakv_decode_attn_static"):
            detail = _lib.deltakv_last_error_detail().decode()
        super().__init__(f"{where}: {strerror(code)} ({code}) {detail}")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    with open("/proc/self/maps") as f:
        runtimes = {ln.split()[-1] for ln in f if "libamdhip64" in ln}
    if len(runtimes) > 1:
        raise ImportError(f"two HIP runtimes are loaded ({sorted(runtimes)}); libdeltakv and PyTorch must share one")
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.deltakv_version.restype = C.c_int
    lib.deltakv_strerror.restype = C.c_char_p
    lib.deltakv_strerror.argtypes = [C.c_int]
    lib.deltakv_last_error_detail.restype = C.c_char_p
    lib.deltakv_tune.restype = C.c_int
    lib.deltakv_tune.argtypes = [C.c_char_p, i32]
    lib.deltakv_timing_begin.restype = C.c_int
    lib.deltakv_timing_end.restype = C.c_int
    lib.deltakv_timing_end.argtypes = [vp, vp, i32]
    lib.deltakv_paged_layout.restype = C.c_int
    lib.deltakv_paged_layout.argtypes = [C.POINTER(Dims), i32, i64, i64, C.POINTER(Layout)]
    lib.deltakv_latent_block_offsets.restype = C.c_int
    lib.deltakv_latent_block_offsets.argtypes = [C.POINTER(Dims), i32, vp]
    lib.deltakv_keep_ratio.restype = C.c_double
    lib.deltakv_keep_ratio.argtypes = [C.POINTER(Dims)]
    lib.deltakv_q4_block_offsets.restype = C.c_int
    lib.deltakv_q4_block_offsets.argtypes = [C.POINTER(Dims), i32, vp, vp, vp, vp]
    lib.deltakv_compress.restype = C.c_int
    lib.deltakv_compress.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, vp, i32, vp, i32,
                                     vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i64, vp]
    lib.deltakv_compress_mlp.restype = C.c_int
    lib.deltakv_compress_mlp.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, vp, i32, vp, i32,
                                         C.POINTER(Mlp), vp, vp, vp, vp, vp, vp, i32, vp, i64, vp]
    lib.deltakv_decode_attn.restype = C.c_int
    lib.deltakv_decode_attn.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, i32, vp, i32,
                                        vp, vp, vp, vp, vp, i32, C.c_float, vp, vp, vp, i64, vp]
    lib.deltakv_decode_attn_rope.restype = C.c_int
    lib.deltakv_decode_attn_rope.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, i32, vp, i32,
                                             vp, vp, vp, vp, vp, i32, C.c_float, C.c_float, vp, vp, vp, i64, vp]
    lib.deltakv_decode_attn_static.restype = C.c_int
    lib.deltakv_decode_attn_static.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, i32, vp, i32,
                                               vp, vp, vp, vp, vp, i32, C.c_float, vp, vp, vp]
    lib.deltakv_decode_attn_subset.restype = C.c_int
    lib.deltakv_decode_attn_subset.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, i32, vp, i32,
                                               vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, C.c_float, vp, vp,
                                               vp, i64, vp]
    lib.deltakv_decode_attn_raw.restype = C.c_int
    lib.deltakv_decode_attn_raw.argtypes = [C.POINTER(Dims), C.POINTER(Layout), vp, vp, vp, vp, i32, vp, i32,
                                            vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, C.c_float,
                                            vp, vp, vp, i64, vp]
    return lib


_lib = _load()
KERNEL_NAMES = ("ref_scores", "stream", "ref_values", "finalize", "admit_refs", "sim_top2", "resolve", "exact",
                "project", "raw_attn")
EXPORTS = ("deltakv_version", "deltakv_strerror", "deltakv_last_error_detail", "deltakv_timing_begin",
           "deltakv_timing_end", "deltakv_tune", "deltakv_paged_layout", "deltakv_latent_block_offsets",
           "deltakv_keep_ratio", "deltakv_compress", "deltakv_decode_attn", "deltakv_decode_attn_subset",
           "deltakv_decode_attn_raw", "deltakv_decode_attn_static", "deltakv_decode_attn_rope", "deltakv_compress_mlp", "deltakv_q4_block_offsets")
STATIC_WS_BYTES = 64 << 20


def version() -> int:
    return int(_lib.deltakv_version())


def strerror(code: int) -> str:
    return _lib.deltakv_strerror(int(code)).decode()


def tune(name: str, value: int) -> None:
    rc = _lib.deltakv_tune(name.encode(), int(value))
    if rc != OK:
        raise DeltaKVError(rc, f"deltakv_tune({name})")


def timing_begin() -> None:
    rc = _lib.deltakv_timing_begin()
    if rc != OK:
        raise DeltaKVError(rc, "deltakv_timing_begin")


def timing_end() -> dict:
    """{kernel name: (total ms, launches)} for the calls since timing_begin()."""
    ms = np.zeros(len(KERNEL_NAMES), dtype=np.float32)
    cnt = np.zeros(len(KERNEL_NAMES), dtype=np.int32)
    rc = _lib.deltakv_timing_end(ms.ctypes.data, cnt.ctypes.data, len(KERNEL_NAMES))
    if rc != OK:
        raise DeltaKVError(rc, "deltakv_timing_end")
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNEL_NAMES)}


def make_dims(n_kv_heads, n_q_heads, rank, n_pages, n_ref_slots, latent_mode=SPLIT, ref_stride=16,
              head_dim=128, page_tokens=16, metric=METRIC_COSINE, latent_bits=16, top_k=1) -> Dims:
    return Dims(n_kv_heads, n_q_heads, head_dim, rank, latent_mode, ref_stride, page_tokens, metric,
                n_pages, n_ref_slots, latent_bits, top_k)


def paged_layout(dims: Dims, max_batch: int, max_new_tokens: int, max_seq_len: int) -> Layout:
    out = Layout()
    rc = _lib.deltakv_paged_layout(C.byref(dims), max_batch, max_new_tokens, max_seq_len, C.byref(out))
    if rc != OK:
        raise DeltaKVError(rc, "deltakv_paged_layout")
    return out


def latent_block_offsets(dims: Dims, stream: int) -> np.ndarray:
    out = np.empty((dims.page_tokens, dims.rank), dtype=np.int32)
    rc = _lib.deltakv_latent_block_offsets(C.byref(dims), stream, out.ctypes.data)
    if rc != OK:
        raise DeltaKVError(rc, "deltakv_latent_block_offsets")
    return out


def q4_block_offsets(dims: Dims, stream: int):
    """(code_elem [P, r], code_shift [P, r], scale_elem [P], zero_elem [P]) of the 4-bit record layout."""
    P, r = dims.page_tokens, dims.rank
    ce, cs = np.zeros((P, r), dtype=np.int32), np.zeros((P, r), dtype=np.int32)
    se, ze = np.zeros(P, dtype=np.int32), np.zeros(P, dtype=np.int32)
    rc = _lib.deltakv_q4_block_offsets(C.byref(dims), stream, ce.ctypes.data, cs.ctypes.data, se.ctypes.data, ze.ctypes.data)
    if rc != OK:
        raise DeltaKVError(rc, "deltakv_q4_block_offsets")
    return ce, cs, se, ze


def keep_ratio(dims: Dims) -> float:
    return float(_lib.deltakv_keep_ratio(C.byref(dims)))


def _dp(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream_handle(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _host_i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def compress(dims, layout, latent_pool, idx_pool, ref_pool, ref_inv_norm, block_tables, ref_tables,
             w_down_k, w_down_v, k_new, v_new, cu_new, cu_new_host, len_before, len_before_host,
             workspace, stream=None, check=True) -> int:
    cu_h, lb_h = _host_i32(cu_new_host), _host_i32(len_before_host)
    batch = len(lb_h)
    rc = _lib.deltakv_compress(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool), _dp(ref_inv_norm),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_down_k), _dp(w_down_v), _dp(k_new), _dp(v_new), _dp(cu_new), cu_h.ctypes.data,
        _dp(len_before), lb_h.ctypes.data, batch, _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_compress")
    return rc


def compress_mlp(dims, layout, latent_pool, idx_pool, ref_pool, ref_inv_norm, block_tables, ref_tables,
                 kind, w1, wg, b1, w2, k_new, v_new, cu_new, cu_new_host, len_before, len_before_host,
                 workspace, stream=None, check=True) -> int:
    """deltakv_compress with the non-linear compressor: w1 / wg bf16 [2 * head_dim][hidden], b1 fp32 [hidden],
    w2 bf16 [hidden][rank] (device tensors; wg None unless kind is MLP_SWIGLU)."""
    cu_h, lb_h = _host_i32(cu_new_host), _host_i32(len_before_host)
    mlp = Mlp(int(kind), int(w1.shape[1]), _dp(w1), _dp(wg), _dp(b1), _dp(w2))
    rc = _lib.deltakv_compress_mlp(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool), _dp(ref_inv_norm),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        C.byref(mlp), _dp(k_new), _dp(v_new), _dp(cu_new), cu_h.ctypes.data,
        _dp(len_before), lb_h.ctypes.data, len(lb_h), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_compress_mlp")
    return rc


def decode_attn(dims, layout, latent_pool, idx_pool, ref_pool, block_tables, ref_tables, w_up_k, w_up_v, q,
                seq_lens, seq_lens_host, scale, out, lse, workspace, stream=None, check=True) -> int:
    sl_h = _host_i32(seq_lens_host)
    rc = _lib.deltakv_decode_attn(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_up_k), _dp(w_up_v), _dp(q), _dp(seq_lens), sl_h.ctypes.data, len(sl_h), float(scale),
        _dp(out), _dp(lse), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_decode_attn")
    return rc


def decode_attn_rope(dims, layout, latent_pool, idx_pool, ref_pool, block_tables, ref_tables, w_up_k, w_up_v, q_rot,
                     seq_lens, seq_lens_host, scale, rope_base, out, lse, workspace, stream=None, check=True) -> int:
    """Decode attention with rotary position embedding on the reconstructed keys (q_rot: already rotated)."""
    sl_h = _host_i32(seq_lens_host)
    rc = _lib.deltakv_decode_attn_rope(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_up_k), _dp(w_up_v), _dp(q_rot), _dp(seq_lens), sl_h.ctypes.data, len(sl_h), float(scale), float(rope_base),
        _dp(out), _dp(lse), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_decode_attn_rope")
    return rc


def decode_attn_static(dims, layout, latent_pool, idx_pool, ref_pool, block_tables, ref_tables, w_up_k, w_up_v, q,
                       seq_lens, seq_lens_host, scale, out, lse, stream=None, check=True) -> int:
    """deltakv_decode_attn on the library's own static workspace (the call allocates nothing)."""
    sl_h = _host_i32(seq_lens_host)
    rc = _lib.deltakv_decode_attn_static(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_up_k), _dp(w_up_v), _dp(q), _dp(seq_lens), sl_h.ctypes.data, len(sl_h), float(scale),
        _dp(out), _dp(lse), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_decode_attn_static")
    return rc


def decode_attn_subset(dims, layout, latent_pool, idx_pool, ref_pool, block_tables, ref_tables, w_up_k, w_up_v, q,
                       seq_lens, seq_lens_host, sel_pages, sel_masks, n_sel, n_sel_host, scale, out, lse, workspace,
                       stream=None, check=True) -> int:
    sl_h, ns_h = _host_i32(seq_lens_host), _host_i32(n_sel_host)
    rc = _lib.deltakv_decode_attn_subset(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_up_k), _dp(w_up_v), _dp(q), _dp(seq_lens), sl_h.ctypes.data,
        _dp(sel_pages), _dp(sel_masks), sel_pages.shape[1], _dp(n_sel), ns_h.ctypes.data, len(sl_h), float(scale),
        _dp(out), _dp(lse), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_decode_attn_subset")
    return rc


def decode_attn_raw(dims, layout, latent_pool, idx_pool, ref_pool, block_tables, ref_tables, w_up_k, w_up_v, q,
                    seq_lens, seq_lens_host, raw_k, raw_v, raw_lens, scale, out, lse, workspace, selection=None,
                    stream=None, check=True) -> int:
    """raw_k / raw_v: [batch, raw_cap, n_kv_heads, head_dim] bf16 bits (or None for no raw segment);
    selection: None for the whole cache, else (sel_pages, sel_masks, n_sel, n_sel_host)."""
    sl_h = _host_i32(seq_lens_host)
    sp, sm, n_dev, n_host = selection if selection is not None else (None, None, None, None)
    ns_h = _host_i32(n_host) if selection is not None else None
    rc = _lib.deltakv_decode_attn_raw(
        C.byref(dims), C.byref(layout), _dp(latent_pool), _dp(idx_pool), _dp(ref_pool),
        _dp(block_tables), block_tables.shape[1], _dp(ref_tables), ref_tables.shape[1],
        _dp(w_up_k), _dp(w_up_v), _dp(q), _dp(seq_lens), sl_h.ctypes.data,
        _dp(sp), _dp(sm), 0 if sp is None else sp.shape[1], _dp(n_dev), None if ns_h is None else ns_h.ctypes.data,
        _dp(raw_k), _dp(raw_v), _dp(raw_lens), 0 if raw_k is None else raw_k.shape[1], len(sl_h), float(scale),
        _dp(out), _dp(lse), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if check and rc != OK:
        raise DeltaKVError(rc, "deltakv_decode_attn_raw")
    return rc
