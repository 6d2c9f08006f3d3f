"""CPU oracle for the HDC hot path: TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It does not import the HIP library or its
Python binding, and the product never imports it.

The arithmetic lives in ``hdc_oracle.c`` (plain C, one byte per hypervector
dimension, written from Sec. III of arXiv 2206.04746).  The functions below only
marshal numpy arrays, call the C routines through ctypes, and convert between the
byte-per-dimension form the oracle computes in and the packed 32-bit words the
library boundary uses (Sec. IV-B1: LSB first, pad bits zero).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hdc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fused multiply-add, OpenMP over samples)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


I64, I32 = ctypes.c_int64, ctypes.c_int32


def threads() -> int:
    """Host threads the sample-parallel oracle loops use."""
    return int(_load().orc_threads())


def unpack(words: np.ndarray, D: int) -> np.ndarray:
    """u32 words ``[..., W]`` -> {0,1} bytes ``[..., D]``."""
    words = _c(words, np.uint32)
    W = (D + 31) // 32
    assert words.shape[-1] == W
    rows = words.size // W
    bits = np.empty(words.shape[:-1] + (D,), dtype=np.uint8)
    _load().orc_unpack(_p(words), I64(rows), I32(D), _p(bits))
    return bits


def pack(bits: np.ndarray) -> np.ndarray:
    """{0,1} bytes ``[..., D]`` -> u32 words ``[..., W]`` with zero pad bits."""
    bits = _c(bits, np.uint8)
    D = bits.shape[-1]
    W = (D + 31) // 32
    rows = bits.size // D if D else 0
    words = np.empty(bits.shape[:-1] + (W,), dtype=np.uint32)
    _load().orc_pack(_p(bits), I64(rows), I32(D), _p(words))
    return words


def quantize(feats: np.ndarray, L: int, lo: Optional[np.ndarray] = None,
             scale: Optional[np.ndarray] = None) -> np.ndarray:
    """Bin index ``[N][F]`` (int32) of every feature; fp32 features need lo/scale."""
    N, F = feats.shape
    q = np.empty((N, F), dtype=np.int32)
    if feats.dtype == np.uint8:
        x = _c(feats, np.uint8)
        _load().orc_quantize_u8(_p(x), I64(N), I32(F), I32(L), _p(q))
    else:
        x = _c(feats, np.float32)
        lo32, sc32 = _c(lo, np.float32), _c(scale, np.float32)
        assert lo32.shape == (F,) and sc32.shape == (F,)
        _load().orc_quantize_f32(_p(x), I64(N), I32(F), _p(lo32), _p(sc32), I32(L), _p(q))
    return q


def encode_bits(q: np.ndarray, item_bits: np.ndarray, level_bits: np.ndarray,
                tie_bits: np.ndarray) -> np.ndarray:
    """Eq. (1) on byte-per-dimension tables; returns ``[N][D]`` bytes."""
    q = _c(q, np.int32)
    N, F = q.shape
    item_bits, level_bits, tie_bits = (_c(a, np.uint8) for a in (item_bits, level_bits, tie_bits))
    D = item_bits.shape[1]
    assert item_bits.shape == (F, D) and level_bits.shape[1] == D and tie_bits.shape == (D,)
    assert q.size == 0 or (q.min() >= 0 and q.max() < level_bits.shape[0])
    hv = np.empty((N, D), dtype=np.uint8)
    _load().orc_encode(_p(q), I64(N), I32(F), I32(D), _p(item_bits), _p(level_bits),
                       _p(tie_bits), _p(hv))
    return hv


def encode(feats: np.ndarray, D: int, L: int, item: np.ndarray, level: np.ndarray,
           tie: np.ndarray, lo=None, scale=None) -> np.ndarray:
    """Features ``[N][F]`` -> packed hypervectors u32 ``[N][W]`` (packed tables in)."""
    q = quantize(feats, L, lo, scale)
    hv = encode_bits(q, unpack(item, D), unpack(level, D), unpack(tie, D))
    return pack(hv)


def train_classical(hv: np.ndarray, labels: np.ndarray, D: int, C: int,
                    acc: Optional[np.ndarray] = None, class_n: Optional[np.ndarray] = None
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """Adds packed rows ``hv [N][W]`` into ``acc i32[C][D]`` / ``class_n i64[C]``."""
    bits = unpack(hv, D)
    labels = _c(labels, np.int32)
    N = bits.shape[0]
    assert labels.shape == (N,)
    acc = np.zeros((C, D), dtype=np.int32) if acc is None else _c(acc, np.int32).copy()
    class_n = np.zeros(C, dtype=np.int64) if class_n is None else _c(class_n, np.int64).copy()
    _load().orc_train_classical(_p(bits), _p(labels), I64(N), I32(D), I32(C), _p(acc), _p(class_n))
    return acc, class_n


def binarize_classical(acc: np.ndarray, class_n: np.ndarray, tie: np.ndarray) -> np.ndarray:
    acc, class_n = _c(acc, np.int32), _c(class_n, np.int64)
    C, D = acc.shape
    tie_bits = unpack(tie, D)
    out = np.empty((C, D), dtype=np.uint8)
    _load().orc_binarize_classical(_p(acc), _p(class_n), I32(C), I32(D), _p(tie_bits), _p(out))
    return pack(out)


def train_online(hv: np.ndarray, labels: np.ndarray, D: int, C: int, epochs: int = 1,
                 lr: float = 1.0, acc: Optional[np.ndarray] = None, log: bool = False):
    """Sequential similarity-weighted updates, Eqs. (2),(3).  Returns ``acc f32[C][D]``
    (and, with ``log``, the per-step predictions and top-2 cosine margins)."""
    bits = unpack(hv, D)
    labels = _c(labels, np.int32)
    N = bits.shape[0]
    assert labels.shape == (N,)
    acc = np.zeros((C, D), dtype=np.float32) if acc is None else _c(acc, np.float32).copy()
    pred = np.empty(N * epochs, dtype=np.int32) if log else None
    margin = np.empty(N * epochs, dtype=np.float64) if log else None
    _load().orc_train_online(_p(bits), _p(labels), I64(N), I32(D), I32(C), I32(epochs),
                             ctypes.c_float(lr), _p(acc), _p(pred), _p(margin))
    return (acc, pred, margin) if log else acc


def hsum(hv: np.ndarray, D: int) -> np.ndarray:
    """Horizontal summation (Sec. IV-B2): set dimensions per row, ``int32 [N]``."""
    bits = unpack(hv, D)
    out = np.empty(bits.shape[0], dtype=np.int32)
    _load().orc_hsum(_p(bits), I64(bits.shape[0]), I32(D), _p(out))
    return out


def vsum(hv: np.ndarray, D: int) -> np.ndarray:
    """Vertical summation (Sec. IV-B2): rows with the dimension set, ``int32 [D]``."""
    bits = unpack(hv, D)
    out = np.empty(D, dtype=np.int32)
    _load().orc_vsum(_p(bits), I64(bits.shape[0]), I32(D), _p(out))
    return out


def search_cosine(hv: np.ndarray, m: np.ndarray, D: int) -> Tuple[np.ndarray, np.ndarray]:
    """Cosine inference against real-valued class rows ``m f32[C][D]`` (Sec. III):
    ``(cos f64[N][C], pred int32[N])``."""
    bits = unpack(hv, D)
    m = _c(m, np.float32)
    N, C = bits.shape[0], m.shape[0]
    assert m.shape == (C, D)
    cosv = np.empty((N, C), dtype=np.float64)
    pred = np.empty(N, dtype=np.int32)
    _load().orc_search_cosine(_p(bits), I64(N), I32(D), _p(m), I32(C), _p(cosv), _p(pred))
    return cosv, pred


def train_online_batched(hv: np.ndarray, labels: np.ndarray, D: int, C: int, batch: int,
                         epochs: int = 1, lr: float = 1.0, acc: Optional[np.ndarray] = None) -> np.ndarray:
    """Online training with the class rows frozen over each batch of ``batch`` samples
    (Sec. VI-D2).  Returns ``acc f32[C][D]``."""
    bits = unpack(hv, D)
    labels = _c(labels, np.int32)
    N = bits.shape[0]
    assert labels.shape == (N,) and batch >= 1
    acc = np.zeros((C, D), dtype=np.float32) if acc is None else _c(acc, np.float32).copy()
    _load().orc_train_online_batched(_p(bits), _p(labels), I64(N), I32(D), I32(C), I32(epochs),
                                     ctypes.c_float(lr), I64(batch), _p(acc))
    return acc


def binarize_online(acc: np.ndarray, tie: np.ndarray) -> np.ndarray:
    acc = _c(acc, np.float32)
    C, D = acc.shape
    tie_bits = unpack(tie, D)
    out = np.empty((C, D), dtype=np.uint8)
    _load().orc_binarize_online(_p(acc), I32(C), I32(D), _p(tie_bits), _p(out))
    return pack(out)


def search(hv: np.ndarray, class_hv: np.ndarray, D: int) -> Tuple[np.ndarray, np.ndarray]:
    """Hamming distances u32 ``[N][C]`` and nearest class i32 ``[N]``."""
    q_bits, c_bits = unpack(hv, D), unpack(class_hv, D)
    N, C = q_bits.shape[0], c_bits.shape[0]
    dist = np.empty((N, C), dtype=np.uint32)
    pred = np.empty(N, dtype=np.int32)
    _load().orc_search(_p(q_bits), I64(N), _p(c_bits), I32(C), I32(D), _p(dist), _p(pred))
    return dist, pred
