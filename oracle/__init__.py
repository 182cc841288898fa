"""ctypes front end of the CPU oracle (oracle/bs_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
CPU-baseline leg.  The product path never imports this package, and this package never
imports the product path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bs_oracle.c")
_LIB = os.path.join(_HERE, "libbs_oracle.so")

DENSE, SINK, INTRA, INTRA_SINK = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, AVX2 at most so the binary runs on any recent host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared",
               "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, i64, u8p = ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(ctypes.c_uint8)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p, f64p = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        lib.bso_token_arrays.argtypes = [i32p, i32, i32, i32, i32p, i32, i32p, u8p]
        lib.bso_token_arrays.restype = ctypes.c_int
        lib.bso_allowed.argtypes = [ctypes.c_int, i32, i32, i32p, u8p, ctypes.c_int, i32]
        lib.bso_allowed.restype = ctypes.c_int
        lib.bso_mask.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32, u8p]
        lib.bso_mask.restype = None
        lib.bso_pair_count.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32]
        lib.bso_pair_count.restype = i64
        lib.bso_mask_rows.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32, i32p, i32, u8p]
        lib.bso_mask_rows.restype = None
        lib.bso_pair_count_rows.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32, i32p, i32]
        lib.bso_pair_count_rows.restype = i64
        lib.bso_tile_states.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32, i32, i32, i32p, i32, u8p]
        lib.bso_tile_states.restype = None
        lib.bso_tile_states_rows.argtypes = [ctypes.c_int, i32, i32p, u8p, ctypes.c_int, i32, i32, i32, i32p, i32, u8p]
        lib.bso_tile_states_rows.restype = None
        lib.bso_attention.argtypes = [f32p, f32p, f32p, i32, i32, i32, i32, u8p, i32p, u8p, ctypes.c_int, i32,
                                      ctypes.c_double, i32p, i32, f64p]
        lib.bso_attention.restype = ctypes.c_int
        lib.bso_num_threads.argtypes = []
        lib.bso_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def num_threads() -> int:
    return int(_load().bso_num_threads())


def token_arrays(spans, seq_len: int, sink_len: int = 0, sink_offsets=None):
    """(imgid int32[L], issink uint8[L]) from the span table; raises ValueError on a bad table.
    sink_offsets: offsets inside every image that are sink keys as well (Gemma-3-style sinks)."""
    sp = np.ascontiguousarray(np.asarray(spans, dtype=np.int32).reshape(-1, 3))
    so = np.ascontiguousarray([] if sink_offsets is None else sink_offsets, dtype=np.int32).reshape(-1)
    imgid = np.empty(max(seq_len, 0), dtype=np.int32)
    issink = np.empty(max(seq_len, 0), dtype=np.uint8)
    rc = _load().bso_token_arrays(_p(sp, ctypes.c_int32), sp.shape[0], seq_len, sink_len,
                                  _p(so, ctypes.c_int32), len(so),
                                  _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8))
    if rc != 0:
        raise ValueError(f"bad span table (code {rc})")
    return imgid, issink


def allowed(cls: int, i: int, j: int, imgid, issink, img_bidir: bool = False, window: int = 0) -> bool:
    """img_bidir: the model's dense mask also lets a token see the later tokens of its own image;
    window > 0: the dense mask keeps only keys with i - j < window (sliding-window layers)."""
    return bool(_load().bso_allowed(int(cls), int(i), int(j), _p(imgid, ctypes.c_int32),
                                    _p(issink, ctypes.c_uint8), int(bool(img_bidir)), int(window)))


def mask(cls: int, imgid, issink, img_bidir: bool = False, window: int = 0) -> np.ndarray:
    L = len(imgid)
    out = np.empty((L, L), dtype=np.uint8)
    _load().bso_mask(int(cls), L, _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8),
                     int(bool(img_bidir)), int(window), _p(out, ctypes.c_uint8))
    return out


def pair_count(cls: int, imgid, issink, img_bidir: bool = False, window: int = 0) -> int:
    return int(_load().bso_pair_count(int(cls), len(imgid), _p(imgid, ctypes.c_int32),
                                      _p(issink, ctypes.c_uint8), int(bool(img_bidir)), int(window)))


def mask_rows(cls: int, imgid, issink, rows, img_bidir: bool = False, window: int = 0) -> np.ndarray:
    """uint8 [len(rows), L]: the listed rows of the bitmap (for prompts too long for mask())."""
    L = len(imgid)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1)
    assert len(rows) == 0 or (rows.min() >= 0 and rows.max() < L)
    out = np.empty((len(rows), L), dtype=np.uint8)
    _load().bso_mask_rows(int(cls), L, _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8), int(bool(img_bidir)),
                          int(window), _p(rows, ctypes.c_int32), len(rows), _p(out, ctypes.c_uint8))
    return out


def pair_count_rows(cls: int, imgid, issink, rows, img_bidir: bool = False, window: int = 0) -> int:
    """Allowed pairs of the listed query rows, by enumeration."""
    L = len(imgid)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1)
    assert len(rows) == 0 or (rows.min() >= 0 and rows.max() < L)
    return int(_load().bso_pair_count_rows(int(cls), L, _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8),
                                           int(bool(img_bidir)), int(window), _p(rows, ctypes.c_int32), len(rows)))


def tile_states(cls: int, imgid, issink, block_m: int, block_n: int, q_tiles=None,
                img_bidir: bool = False, window: int = 0) -> np.ndarray:
    """uint8 [len(q_tiles), N] of 0 skip / 1 partial / 2 full, by enumeration of the elements."""
    L = len(imgid)
    M = -(-L // block_m)
    N = -(-L // block_n)
    qt = np.arange(M, dtype=np.int32) if q_tiles is None else np.ascontiguousarray(q_tiles, dtype=np.int32)
    out = np.empty((len(qt), N), dtype=np.uint8)
    _load().bso_tile_states(int(cls), L, _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8),
                            int(bool(img_bidir)), int(window), block_m, block_n, _p(qt, ctypes.c_int32), len(qt), _p(out, ctypes.c_uint8))
    return out


def tile_states_rows(cls: int, imgid, issink, rows, block_n: int, img_bidir: bool = False,
                     window: int = 0) -> np.ndarray:
    """Tile states for query tiles given as row lists: rows int32 [n_tiles, block_m], -1 = no row."""
    L = len(imgid)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert rows.ndim == 2
    N = -(-L // block_n)
    out = np.empty((rows.shape[0], N), dtype=np.uint8)
    _load().bso_tile_states_rows(int(cls), L, _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8),
                                 int(bool(img_bidir)), int(window), rows.shape[1], block_n, _p(rows, ctypes.c_int32), rows.shape[0],
                                 _p(out, ctypes.c_uint8))
    return out


def attention(q, k, v, head_class, imgid, issink, scale: float, rows=None, img_bidir: bool = False,
              window: int = 0) -> np.ndarray:
    """fp64 masked-softmax attention.  q [Hq,L,d], k/v [Hkv,L,d] as float32 numpy arrays
    (widen bf16 exactly before calling).  Returns [Hq, n_rows, d] float64."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    k = np.ascontiguousarray(k, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    Hq, L, d = q.shape
    Hkv = k.shape[0]
    assert k.shape == (Hkv, L, d) and v.shape == (Hkv, L, d) and Hq % Hkv == 0
    hc = np.ascontiguousarray(head_class, dtype=np.uint8)
    assert hc.shape == (Hq,) and len(imgid) == L and len(issink) == L
    if rows is None:
        rp, n_rows = None, L
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.ndim == 1 and (len(rows) == 0 or (rows.min() >= 0 and rows.max() < L))
        rp, n_rows = _p(rows, ctypes.c_int32), len(rows)
    out = np.empty((Hq, n_rows, d), dtype=np.float64)
    if n_rows == 0:
        return out
    rc = _load().bso_attention(_p(q, ctypes.c_float), _p(k, ctypes.c_float), _p(v, ctypes.c_float),
                               Hq, Hq // Hkv, L, d, _p(hc, ctypes.c_uint8),
                               _p(imgid, ctypes.c_int32), _p(issink, ctypes.c_uint8), int(bool(img_bidir)),
                               int(window), float(scale), rp, n_rows, _p(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"oracle attention failed (code {rc})")
    return out


def attention_for_prompt(p, q, k, v, rows=None) -> np.ndarray:
    """Convenience: p is any object with spans / seq_len / sink_len / head_class / scale
    (e.g. workloads.Prompt); q, k, v torch tensors or numpy arrays."""
    def to_np(t):
        if hasattr(t, "detach"):
            t = t.detach().float().cpu().numpy()
        return t
    imgid, issink = token_arrays(p.spans, p.seq_len, p.sink_len, getattr(p, "sink_offsets", None))
    return attention(to_np(q), to_np(k), to_np(v), p.head_class, imgid, issink, p.scale, rows,
                     bool(getattr(p, "img_bidir", False)), int(getattr(p, "window", 0)))
