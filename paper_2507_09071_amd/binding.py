"""ctypes binding with the same names as the C ABI declared in include/blindsight.h.

PyTorch is used only by callers, for device memory and streams: this module takes raw
device pointers (or objects with .data_ptr()) and never computes anything itself.  If the
shared library is missing it is built once; if it cannot be loaded the import of a symbol
fails loudly — there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

BS_BF16, BS_F32 = 0, 1
DENSE, SINK, INTRA, INTRA_SINK = 0, 1, 2, 3

EXPORTS = ("bs_build_tilemap", "bs_build_tilemap_ex", "bs_build_tilemap_model", "bs_build_tilemap_suffix", "bs_tilemap_destroy", "bs_tilemap_dims", "bs_tilemap_row_order", "bs_tilemap_layout", "bs_tilemap_key_order", "bs_tilemap_tile_states",
           "bs_tilemap_stats", "bs_tilemap_pair_plan", "bs_tilemap_upload", "bs_tilemap_rebind", "bs_tilemap_prepare",
           "bs_attn_prefill", "bs_attn_prefill_ex", "bs_attn_prefill_static", "bs_static_scratch_bytes",
           "bs_characterize_prompt", "bs_head_sq_error", "bs_aggregate_head_type", "bs_aggregate_layer", "bs_alpha_layer", "bs_strerror",
           "bs_last_error")


class BlindsightError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = load_library().bs_last_error().decode() if code in (-3, -4) or "static" in where else ""
        super().__init__(f"{where}: {_strerror(code)} ({code})" + (f" [{detail}]" if detail else ""))


class _Span(ctypes.Structure):
    _fields_ = [("start", ctypes.c_int32), ("end", ctypes.c_int32), ("sink", ctypes.c_int32)]


_lib = None


def _preload_process_hip_runtime():
    """One process must use ONE HIP runtime.  PyTorch ships its own libamdhip64; callers hand us
    device pointers and streams that belong to it, so load that copy first (by path) and let the
    dynamic linker resolve our library's libamdhip64 dependency to it by soname.  Without PyTorch
    the system runtime under /opt/rocm is used."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.origin:
        return
    cand = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def library_path() -> str:
    return _build.LIB


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(verbose=False)
    _preload_process_hip_runtime()
    lib = ctypes.CDLL(_build.LIB)
    i32, i64p = ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
    i32p, u8p, vp = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8), ctypes.c_void_p
    lib.bs_build_tilemap.argtypes = [ctypes.POINTER(_Span), i32, i32, u8p, i32, i32, i32, i32,
                                     ctypes.POINTER(vp)]
    lib.bs_build_tilemap.restype = ctypes.c_int
    lib.bs_build_tilemap_ex.argtypes = [ctypes.POINTER(_Span), i32, i32, u8p, i32, i32, i32, i32, ctypes.c_uint32,
                                        ctypes.POINTER(ctypes.c_void_p)]
    lib.bs_build_tilemap_ex.restype = ctypes.c_int
    lib.bs_build_tilemap_model.argtypes = [ctypes.POINTER(_Span), i32, i32, u8p, i32, i32, i32, i32, ctypes.c_uint32,
                                           i32p, i32, i32, ctypes.POINTER(ctypes.c_void_p)]
    lib.bs_build_tilemap_model.restype = ctypes.c_int
    lib.bs_build_tilemap_suffix.argtypes = [ctypes.POINTER(_Span), i32, i32, u8p, i32, i32, i32, i32, ctypes.c_uint32,
                                            i32p, i32, i32, i32, ctypes.POINTER(ctypes.c_void_p)]
    lib.bs_build_tilemap_suffix.restype = ctypes.c_int
    lib.bs_tilemap_row_order.argtypes = [vp, i32p]
    lib.bs_tilemap_row_order.restype = ctypes.c_int
    lib.bs_tilemap_layout.argtypes = [vp, i32p, i32p, i32p]
    lib.bs_tilemap_layout.restype = ctypes.c_int
    lib.bs_tilemap_key_order.argtypes = [vp, i32p, i32p]
    lib.bs_tilemap_key_order.restype = ctypes.c_int
    lib.bs_tilemap_destroy.argtypes = [vp]
    lib.bs_tilemap_destroy.restype = None
    lib.bs_tilemap_dims.argtypes = [vp, i32p, i32p, i32p, i32p]
    lib.bs_tilemap_dims.restype = ctypes.c_int
    lib.bs_tilemap_tile_states.argtypes = [vp, i32, i32, i32, u8p]
    lib.bs_tilemap_tile_states.restype = ctypes.c_int
    lib.bs_tilemap_stats.argtypes = [vp, i32, i64p, i64p, i64p, i64p, i64p, i64p]
    lib.bs_tilemap_stats.restype = ctypes.c_int
    lib.bs_tilemap_pair_plan.argtypes = [vp, i32, i64p, i64p, i64p]
    lib.bs_tilemap_pair_plan.restype = ctypes.c_int
    lib.bs_tilemap_upload.argtypes = [vp]
    lib.bs_tilemap_upload.restype = ctypes.c_int
    lib.bs_tilemap_rebind.argtypes = [vp, u8p, i32]
    lib.bs_tilemap_rebind.restype = ctypes.c_int
    lib.bs_tilemap_prepare.argtypes = [vp, i32, i32, vp]
    lib.bs_tilemap_prepare.restype = ctypes.c_int
    lib.bs_attn_prefill_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, ctypes.c_float, vp]
    lib.bs_attn_prefill_static.restype = ctypes.c_int
    lib.bs_static_scratch_bytes.argtypes = []
    lib.bs_static_scratch_bytes.restype = ctypes.c_int64
    lib.bs_attn_prefill.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, vp]
    lib.bs_attn_prefill.restype = ctypes.c_int
    lib.bs_attn_prefill_ex.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_float, vp, vp, vp]
    lib.bs_attn_prefill_ex.restype = ctypes.c_int
    f64, f64p = ctypes.c_double, ctypes.POINTER(ctypes.c_double)
    lib.bs_characterize_prompt.argtypes = [vp, vp, vp, ctypes.POINTER(_Span), i32, i32, i32, i32, i32, i32, i32,
                                           ctypes.c_float, f64, ctypes.c_uint32, i32p, i32, i32, u8p, f64p, vp]
    lib.bs_characterize_prompt.restype = ctypes.c_int
    lib.bs_head_sq_error.argtypes = [vp, vp, i32, i32, ctypes.c_int64, vp, vp]
    lib.bs_head_sq_error.restype = ctypes.c_int
    lib.bs_aggregate_head_type.argtypes = [f64p, f64, f64, f64]
    lib.bs_aggregate_head_type.restype = ctypes.c_int
    lib.bs_aggregate_layer.argtypes = [u8p, i32, i32, f64, f64, f64, u8p, f64p]
    lib.bs_aggregate_layer.restype = ctypes.c_int
    lib.bs_alpha_layer.argtypes = [f64, f64, i32, i32]
    lib.bs_alpha_layer.restype = ctypes.c_double
    lib.bs_strerror.argtypes = [ctypes.c_int]
    lib.bs_strerror.restype = ctypes.c_char_p
    lib.bs_last_error.argtypes = []
    lib.bs_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _strerror(code: int) -> str:
    return load_library().bs_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code != 0:
        raise BlindsightError(code, where)


class TileMap:
    """Owner of one bs_tilemap*.  Immutable after construction; reusable for every call on
    the same prompt and class vector."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)
        lib = load_library()
        vals = [ctypes.c_int32() for _ in range(4)]
        _check(lib.bs_tilemap_dims(self._h, *[ctypes.byref(v) for v in vals]), "bs_tilemap_dims")
        self.seq_len, self.n_q_tiles, self.n_k_tiles, self.n_q_heads = (int(v.value) for v in vals)

    @property
    def handle(self):
        return self._h

    def tile_states(self, cls: int, q_tile_begin: int = 0, q_tile_count: int | None = None) -> np.ndarray:
        if q_tile_count is None:
            q_tile_count = self.n_q_tiles - q_tile_begin
        out = np.empty((max(q_tile_count, 0), self.n_k_tiles), dtype=np.uint8)
        _check(load_library().bs_tilemap_tile_states(
            self._h, cls, q_tile_begin, q_tile_count,
            out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))), "bs_tilemap_tile_states")
        return out

    def row_order(self, block_m: int = 128) -> np.ndarray:
        """int32 [n_q_tiles, block_m]: position of every row of every query tile, -1 = no row."""
        out = np.empty((self.n_q_tiles, block_m), dtype=np.int32)
        _check(load_library().bs_tilemap_row_order(self._h, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))),
               "bs_tilemap_row_order")
        return out

    def layout(self) -> dict:
        v = [ctypes.c_int32() for _ in range(3)]
        _check(load_library().bs_tilemap_layout(self._h, *[ctypes.byref(x) for x in v]), "bs_tilemap_layout")
        return {n: bool(x.value) for n, x in zip(("regrouped", "packed", "intra_compact"), v)}

    def key_order(self, block_n: int = 64):
        """(int32 [n_k_tiles, block_n] position of the key in every tile slot, -1 = none;
        number of leading tiles that are the prompt in position order)."""
        out = np.empty((self.n_k_tiles, block_n), dtype=np.int32)
        n0 = ctypes.c_int32()
        _check(load_library().bs_tilemap_key_order(self._h, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                                   ctypes.byref(n0)), "bs_tilemap_key_order")
        return out, int(n0.value)

    def stats(self, cls: int) -> dict:
        v = [ctypes.c_int64() for _ in range(6)]
        _check(load_library().bs_tilemap_stats(self._h, cls, *[ctypes.byref(x) for x in v]),
               "bs_tilemap_stats")
        names = ("visited", "full", "partial", "allowed_pairs", "empty_rows", "n_ranges")
        return {n: int(x.value) for n, x in zip(names, v)}

    def pair_plan(self, gqa_group: int) -> dict:
        v = [ctypes.c_int64() for _ in range(3)]
        _check(load_library().bs_tilemap_pair_plan(self._h, int(gqa_group), *[ctypes.byref(x) for x in v]),
               "bs_tilemap_pair_plan")
        return {n: int(x.value) for n, x in zip(("n_units", "unit_tiles", "skip_steps"), v)}

    def upload(self):
        _check(load_library().bs_tilemap_upload(self._h), "bs_tilemap_upload")

    def rebind(self, head_class):
        """Bind the map to another class vector (one per layer); the per-class lists are kept."""
        hc = np.ascontiguousarray(head_class, dtype=np.uint8)
        _check(load_library().bs_tilemap_rebind(self._h, hc.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), len(hc)),
               "bs_tilemap_rebind")
        self.n_q_heads = len(hc)

    def prepare(self, dtype: int, gqa_group: int, stream=None):
        """Upload and plan ahead of time, so that bs_attn_prefill_static allocates nothing."""
        _check(load_library().bs_tilemap_prepare(self._h, int(dtype), int(gqa_group),
                                                 ctypes.c_void_p(int(stream) if stream else 0)), "bs_tilemap_prepare")

    def close(self):
        if self._h is not None and self._h.value:
            load_library().bs_tilemap_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


BS_MAP_REGROUP_ROWS = 1
BS_MAP_PACK_KEYS = 2
BS_MAP_BIDIR_IMAGES = 4


def bs_build_tilemap(spans, seq_len: int, head_class, sink_len: int = 0,
                     block_m: int = 128, block_n: int = 64, flags: int = 0, sink_offsets=None,
                     window: int = 0, q_begin: int = 0) -> TileMap:
    """spans: int array [G,3] of (start, end, sink); head_class: uint8 [n_q_heads];
    flags: 0 or BS_MAP_* bits (goes through bs_build_tilemap_ex); sink_offsets: in-image offsets that
    are sink keys in every image, window: sliding window of the layer (both go through
    bs_build_tilemap_model); q_begin: the query rows are positions q_begin .. seq_len - 1 only
    (bs_build_tilemap_suffix)."""
    lib = load_library()
    sp = np.ascontiguousarray(np.asarray(spans, dtype=np.int32).reshape(-1, 3))
    hc = np.ascontiguousarray(head_class, dtype=np.uint8)
    handle = ctypes.c_void_p()
    sp_ptr = sp.ctypes.data_as(ctypes.POINTER(_Span)) if len(sp) else None
    hc_ptr = hc.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    if q_begin:
        so = np.ascontiguousarray([] if sink_offsets is None else sink_offsets, dtype=np.int32).reshape(-1)
        rc = lib.bs_build_tilemap_suffix(sp_ptr, len(sp), int(seq_len), hc_ptr, len(hc), int(sink_len),
                                         int(block_m), int(block_n), int(flags),
                                         so.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if len(so) else None, len(so),
                                         int(window), int(q_begin), ctypes.byref(handle))
        _check(rc, "bs_build_tilemap_suffix")
    elif (sink_offsets is not None and len(sink_offsets)) or window:
        so = np.ascontiguousarray([] if sink_offsets is None else sink_offsets, dtype=np.int32).reshape(-1)
        rc = lib.bs_build_tilemap_model(sp_ptr, len(sp), int(seq_len), hc_ptr, len(hc), int(sink_len),
                                        int(block_m), int(block_n), int(flags),
                                        so.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if len(so) else None, len(so),
                                        int(window), ctypes.byref(handle))
        _check(rc, "bs_build_tilemap_model")
    elif flags:
        rc = lib.bs_build_tilemap_ex(sp_ptr, len(sp), int(seq_len), hc_ptr, len(hc), int(sink_len),
                                     int(block_m), int(block_n), int(flags), ctypes.byref(handle))
        _check(rc, "bs_build_tilemap_ex")
    else:
        rc = lib.bs_build_tilemap(sp_ptr, len(sp), int(seq_len), hc_ptr, len(hc), int(sink_len),
                                  int(block_m), int(block_n), ctypes.byref(handle))
        _check(rc, "bs_build_tilemap")
    return TileMap(handle.value)


def _ptr(x) -> int:
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def bs_attn_prefill_ex(q, k, v, out, tilemap: TileMap, dtype: int, n_q_heads: int, gqa_group: int,
                       head_dim: int, scale: float, stream=None, ev_main_start=None, ev_main_stop=None) -> None:
    """bs_attn_prefill that also records two caller-owned hipEvent_t handles (ints) around the
    attention kernel itself."""
    rc = load_library().bs_attn_prefill_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(out), tilemap.handle,
                                           int(dtype), int(n_q_heads), int(gqa_group), int(head_dim),
                                           float(scale), ctypes.c_void_p(int(stream) if stream else 0),
                                           ctypes.c_void_p(int(ev_main_start) if ev_main_start else 0),
                                           ctypes.c_void_p(int(ev_main_stop) if ev_main_stop else 0))
    _check(rc, "bs_attn_prefill_ex")


def bs_attn_prefill(q, k, v, out, tilemap: TileMap, dtype: int, n_q_heads: int, gqa_group: int,
                    head_dim: int, scale: float, stream=None) -> None:
    """q/k/v/out: device pointers (ints) or tensors exposing .data_ptr(); stream: hipStream_t
    handle as int (e.g. torch.cuda.current_stream().cuda_stream) or None for the default stream.
    Enqueues only."""
    rc = load_library().bs_attn_prefill(_ptr(q), _ptr(k), _ptr(v), _ptr(out), tilemap.handle,
                                        int(dtype), int(n_q_heads), int(gqa_group), int(head_dim),
                                        float(scale), ctypes.c_void_p(int(stream) if stream else 0))
    _check(rc, "bs_attn_prefill")


def bs_attn_prefill_static(q, k, v, out, tilemap: TileMap, n_q_heads: int, gqa_group: int, head_dim: int,
                           scale: float, stream=None) -> None:
    """bf16 prefill that allocates nothing (static scratch inside the library); the map must have been
    prepared with TileMap.prepare(BS_BF16, gqa_group)."""
    rc = load_library().bs_attn_prefill_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), tilemap.handle, int(n_q_heads),
                                               int(gqa_group), int(head_dim), float(scale),
                                               ctypes.c_void_p(int(stream) if stream else 0))
    _check(rc, "bs_attn_prefill_static")


def bs_static_scratch_bytes() -> int:
    return int(load_library().bs_static_scratch_bytes())


def bs_characterize_prompt(q, k, v, spans, seq_len: int, sink_len: int, dtype: int, n_q_heads: int,
                           gqa_group: int, head_dim: int, scale: float, alpha: float, map_flags: int = 0,
                           stream=None, sink_offsets=None, window: int = 0):
    """Alg. 1 for every query head of one layer.  Returns (head_type uint8 [Hq], nmse float64 [3, Hq]);
    waits for the stream."""
    sp = np.ascontiguousarray(np.asarray(spans, dtype=np.int32).reshape(-1, 3))
    sp_ptr = sp.ctypes.data_as(ctypes.POINTER(_Span)) if len(sp) else None
    head_type = np.zeros(int(n_q_heads), dtype=np.uint8)
    nmse = np.zeros((3, int(n_q_heads)), dtype=np.float64)
    so = np.ascontiguousarray([] if sink_offsets is None else sink_offsets, dtype=np.int32).reshape(-1)
    so_ptr = so.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if len(so) else None
    rc = load_library().bs_characterize_prompt(
        _ptr(q), _ptr(k), _ptr(v), sp_ptr, len(sp), int(seq_len), int(sink_len), int(dtype), int(n_q_heads),
        int(gqa_group), int(head_dim), float(scale), float(alpha), int(map_flags), so_ptr, len(so), int(window),
        head_type.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
        nmse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ctypes.c_void_p(int(stream) if stream else 0))
    _check(rc, "bs_characterize_prompt")
    return head_type, nmse


def bs_head_sq_error(attn_mask, attn_ref, dtype: int, n_heads: int, elems_per_head: int, sums, stream=None) -> None:
    """sums: device buffer of 2 * n_heads float64 (pointer or tensor).  Enqueues only."""
    rc = load_library().bs_head_sq_error(_ptr(attn_mask), _ptr(attn_ref), int(dtype), int(n_heads),
                                         int(elems_per_head), _ptr(sums),
                                         ctypes.c_void_p(int(stream) if stream else 0))
    _check(rc, "bs_head_sq_error")


def bs_aggregate_head_type(fraction, gamma_d: float, gamma_s: float, gamma_i: float) -> int:
    """Alg. 2 for one head: fraction = 4 shares (Dense, Sink, Intra-Image, Intra-Image+Sink)."""
    f = np.ascontiguousarray(fraction, dtype=np.float64)
    if f.shape != (4,):
        raise ValueError("fraction must hold 4 values")
    rc = load_library().bs_aggregate_head_type(f.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                               float(gamma_d), float(gamma_s), float(gamma_i))
    if rc < 0:
        _check(rc, "bs_aggregate_head_type")
    return rc


def bs_aggregate_layer(head_types, gamma_d: float, gamma_s: float, gamma_i: float):
    """Alg. 2 for a layer: head_types uint8 [n_prompts, n_q_heads] -> (head_class uint8 [n_q_heads],
    fraction float64 [n_q_heads, 4])."""
    t = np.ascontiguousarray(head_types, dtype=np.uint8)
    if t.ndim != 2:
        raise ValueError("head_types must be [n_prompts, n_q_heads]")
    out = np.zeros(t.shape[1], dtype=np.uint8)
    frac = np.zeros((t.shape[1], 4), dtype=np.float64)
    rc = load_library().bs_aggregate_layer(t.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), t.shape[0], t.shape[1],
                                           float(gamma_d), float(gamma_s), float(gamma_i),
                                           out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                           frac.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "bs_aggregate_layer")
    return out, frac


def bs_alpha_layer(alpha_first: float, alpha_last: float, layer_idx: int, num_layers: int) -> float:
    """Linear alpha_layer schedule of the paper (fixed threshold when both ends are equal)."""
    return float(load_library().bs_alpha_layer(float(alpha_first), float(alpha_last), int(layer_idx), int(num_layers)))
