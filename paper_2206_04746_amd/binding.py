"""ctypes binding of the C ABI in ``include/hdc.h`` - same names, argument marshalling only.

Tensors must live on the GPU, be contiguous and have the dtype the ABI states; nothing is
copied or converted here.  All calls enqueue on ``torch.cuda.current_stream()`` unless a
stream is given; the caller synchronises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# HDC_LIBRARY may point at another build of the same ABI (e.g. a tuning variant)
LIB_PATH = os.environ.get("HDC_LIBRARY") or os.path.join(_HERE, "libhdc.so")

HDC_OK, HDC_EINVAL, HDC_ENOMEM, HDC_EHIP, HDC_ELIMIT, HDC_ELABEL = 0, -1, -2, -3, -4, -5
HDC_RESERVE_ONLINE, HDC_RESERVE_ONLINE_BATCHED, HDC_RESERVE_SEARCH_COSINE, HDC_RESERVE_ENCODE_SPARSE = 1, 2, 4, 8
HDC_F32, HDC_U8 = 0, 1

# every symbol include/hdc.h declares
SYMBOLS = ["hdc_create", "hdc_destroy", "hdc_encode", "hdc_encode_sparse", "hdc_train_classical",
           "hdc_binarize_classical", "hdc_train_online", "hdc_train_online_batched", "hdc_binarize_online", "hdc_search",
           "hdc_search_cosine", "hdc_pack", "hdc_unpack", "hdc_hsum", "hdc_vsum", "hdc_vsum_static", "hdc_encoded_words", "hdc_set_label_check", "hdc_reserve",
           "hdc_profile_enable", "hdc_profile_read",
           "hdc_strerror", "hdc_last_hip_error", "hdc_version"]

KERNEL_IDS = {"encode": 0, "quantize": 1, "accumulate": 2, "online": 3, "search": 4,
              "online_fwd": 5, "online_bwd": 6, "encode_contract": 7, "encode_wide": 8}


class HdcParams(ctypes.Structure):
    _fields_ = [("D", ctypes.c_int32), ("F", ctypes.c_int32), ("L", ctypes.c_int32),
                ("C", ctypes.c_int32), ("feat_dtype", ctypes.c_int)]


class HdcError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libhdc error {code}: {text}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2206_04746_amd.build` "
            "(there is no CPU fallback for the HDC kernels)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.hdc_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(HdcParams), vp, vp, vp, vp, vp]
    lib.hdc_destroy.argtypes = [vp]
    lib.hdc_encode.argtypes = [vp, vp, i64, vp, vp]
    lib.hdc_encode_sparse.argtypes = [vp, vp, i64, vp, vp]
    lib.hdc_train_classical.argtypes = [vp, vp, vp, i64, vp, vp, vp]
    lib.hdc_binarize_classical.argtypes = [vp, vp, vp, vp, vp]
    lib.hdc_train_online.argtypes = [vp, vp, vp, i64, i32, ctypes.c_float, vp, vp]
    lib.hdc_train_online_batched.argtypes = [vp, vp, vp, i64, i32, ctypes.c_float, i64, vp, vp]
    lib.hdc_binarize_online.argtypes = [vp, vp, vp, vp]
    lib.hdc_search_cosine.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    lib.hdc_encoded_words.argtypes = [vp]
    lib.hdc_encoded_words.restype = ctypes.c_int32
    for name in ("hdc_pack", "hdc_unpack", "hdc_hsum", "hdc_vsum"):
        getattr(lib, name).argtypes = [vp, vp, i64, vp, vp]
    lib.hdc_search.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    lib.hdc_vsum_static.argtypes = [i32, vp, i64, vp, vp]
    lib.hdc_set_label_check.argtypes = [vp, ctypes.c_int]
    lib.hdc_set_label_check.restype = ctypes.c_int
    lib.hdc_reserve.argtypes = [vp, ctypes.c_uint, i64, i64, vp]
    lib.hdc_reserve.restype = ctypes.c_int
    lib.hdc_vsum_static.restype = ctypes.c_int
    lib.hdc_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.hdc_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_int64)]
    lib.hdc_profile_enable.restype = ctypes.c_int
    lib.hdc_profile_read.restype = ctypes.c_int
    for name in ("hdc_create", "hdc_destroy", "hdc_encode", "hdc_encode_sparse", "hdc_train_classical",
                 "hdc_binarize_classical", "hdc_train_online", "hdc_train_online_batched",
                 "hdc_binarize_online", "hdc_search", "hdc_search_cosine", "hdc_pack", "hdc_unpack",
                 "hdc_hsum", "hdc_vsum"):
        getattr(lib, name).restype = ctypes.c_int
    lib.hdc_strerror.argtypes = [ctypes.c_int]
    lib.hdc_strerror.restype = ctypes.c_char_p
    lib.hdc_last_hip_error.restype = ctypes.c_char_p
    lib.hdc_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def strerror(code: int) -> str:
    return lib.hdc_strerror(code).decode()


def _check(code: int) -> None:
    if code != HDC_OK:
        text = strerror(code)
        if code == HDC_EHIP:
            text += ": " + lib.hdc_last_hip_error().decode()
        raise HdcError(code, text)


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, shape=None) -> Optional[int]:
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


class Context:
    """Owns an ``hdc_ctx`` (device copies of the item / level / tie tables)."""

    def __init__(self, D: int, F: int, L: int, C: int, item, level, tie, lo=None, scale=None,
                 feat_dtype: str = "f32"):
        self.D, self.F, self.L, self.C = int(D), int(F), int(L), int(C)
        self.W = (self.D + 31) // 32
        self.feat_dtype = feat_dtype
        self._torch_feat = torch.float32 if feat_dtype == "f32" else torch.uint8
        p = HdcParams(self.D, self.F, self.L, self.C, HDC_F32 if feat_dtype == "f32" else HDC_U8)
        item_h, level_h, tie_h = _host(item, np.uint32), _host(level, np.uint32), _host(tie, np.uint32)
        if item_h.shape != (self.F, self.W) or level_h.shape != (self.L, self.W) or tie_h.shape != (self.W,):
            raise ValueError("table shapes must be item[F][W], level[L][W], tie[W]")
        lo_h = None if lo is None else _host(lo, np.float32)
        sc_h = None if scale is None else _host(scale, np.float32)
        torch.cuda.init()
        self._h = ctypes.c_void_p()
        _check(lib.hdc_create(ctypes.byref(self._h), ctypes.byref(p), item_h.ctypes.data,
                              level_h.ctypes.data, tie_h.ctypes.data,
                              None if lo_h is None else lo_h.ctypes.data,
                              None if sc_h is None else sc_h.ctypes.data))

    def close(self) -> None:
        if getattr(self, "_h", None):
            h, self._h = self._h, None
            _check(lib.hdc_destroy(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the entry points, same names as the C ABI ---------------------------------------
    def hdc_encode(self, feats: torch.Tensor, hv: torch.Tensor, stream=None) -> None:
        N = feats.shape[0]
        _check(lib.hdc_encode(self._h, _dev(feats, self._torch_feat, (N, self.F)), N,
                              _dev(hv, torch.int32, (N, self.W)), _stream(stream)))

    def hdc_encode_sparse(self, feats: torch.Tensor, hv: torch.Tensor, stream=None) -> None:
        N = feats.shape[0]
        _check(lib.hdc_encode_sparse(self._h, _dev(feats, self._torch_feat, (N, self.F)), N,
                                     _dev(hv, torch.int32, (N, self.W)), _stream(stream)))

    def hdc_train_classical(self, hv, labels, acc, class_n, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_train_classical(self._h, _dev(hv, torch.int32, (N, self.W)),
                                       _dev(labels, torch.int32, (N,)), N,
                                       _dev(acc, torch.int32, (self.C, self.D)),
                                       _dev(class_n, torch.int64, (self.C,)), _stream(stream)))

    def hdc_binarize_classical(self, acc, class_n, class_hv, stream=None) -> None:
        _check(lib.hdc_binarize_classical(self._h, _dev(acc, torch.int32, (self.C, self.D)),
                                          _dev(class_n, torch.int64, (self.C,)),
                                          _dev(class_hv, torch.int32, (self.C, self.W)), _stream(stream)))

    def hdc_train_online(self, hv, labels, acc, epochs: int = 1, lr: float = 1.0, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_train_online(self._h, _dev(hv, torch.int32, (N, self.W)),
                                    _dev(labels, torch.int32, (N,)), N, int(epochs), float(lr),
                                    _dev(acc, torch.float32, (self.C, self.D)), _stream(stream)))

    def hdc_train_online_batched(self, hv, labels, acc, batch: int, epochs: int = 1, lr: float = 1.0,
                                 stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_train_online_batched(self._h, _dev(hv, torch.int32, (N, self.W)),
                                            _dev(labels, torch.int32, (N,)), N, int(epochs), float(lr),
                                            int(batch), _dev(acc, torch.float32, (self.C, self.D)),
                                            _stream(stream)))

    def hdc_binarize_online(self, acc, class_hv, stream=None) -> None:
        _check(lib.hdc_binarize_online(self._h, _dev(acc, torch.float32, (self.C, self.D)),
                                       _dev(class_hv, torch.int32, (self.C, self.W)), _stream(stream)))

    def hdc_encoded_words(self) -> int:
        return int(lib.hdc_encoded_words(self._h))

    def hdc_search_cosine(self, hv, acc, pred, cos=None, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_search_cosine(self._h, _dev(hv, torch.int32, (N, self.W)), N,
                                     _dev(acc, torch.float32, (self.C, self.D)),
                                     None if cos is None else _dev(cos, torch.float32, (N, self.C)),
                                     _dev(pred, torch.int32, (N,)), _stream(stream)))

    def hdc_pack(self, bits, hv, stream=None) -> None:
        N = bits.shape[0]
        _check(lib.hdc_pack(self._h, _dev(bits, torch.uint8, (N, self.D)), N,
                            _dev(hv, torch.int32, (N, self.W)), _stream(stream)))

    def hdc_unpack(self, hv, bits, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_unpack(self._h, _dev(hv, torch.int32, (N, self.W)), N,
                              _dev(bits, torch.uint8, (N, self.D)), _stream(stream)))

    def hdc_hsum(self, hv, out, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_hsum(self._h, _dev(hv, torch.int32, (N, self.W)), N,
                            _dev(out, torch.int32, (N,)), _stream(stream)))

    def hdc_vsum(self, hv, out, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_vsum(self._h, _dev(hv, torch.int32, (N, self.W)), N,
                            _dev(out, torch.int32, (self.D,)), _stream(stream)))

    def hdc_search(self, hv, class_hv, pred, dist=None, stream=None) -> None:
        N = hv.shape[0]
        _check(lib.hdc_search(self._h, _dev(hv, torch.int32, (N, self.W)), N,
                              _dev(class_hv, torch.int32, (self.C, self.W)),
                              _dev(dist, torch.int32, (N, self.C)), _dev(pred, torch.int32, (N,)),
                              _stream(stream)))


    def hdc_set_label_check(self, enable: bool = True) -> None:
        _check(lib.hdc_set_label_check(self._h, int(bool(enable))))

    def hdc_reserve(self, what: int, max_batch: int = 0, max_queries: int = 0, stream=None) -> None:
        _check(lib.hdc_reserve(self._h, int(what), int(max_batch), int(max_queries), _stream(stream)))

    def hdc_profile_enable(self, enable: bool = True) -> None:
        _check(lib.hdc_profile_enable(self._h, int(bool(enable))))

    def hdc_profile_read(self, kernel: str):
        """(total device milliseconds, timed launches) of one hot kernel since the last read."""
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(lib.hdc_profile_read(self._h, KERNEL_IDS[kernel], ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value


def hdc_vsum_static(D: int, hv: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """hdc_vsum without a context and without any allocation (D <= 16384)."""
    N, W = hv.shape[0], (int(D) + 31) // 32
    _check(lib.hdc_vsum_static(int(D), _dev(hv, torch.int32, (N, W)), N, _dev(out, torch.int32, (int(D),)),
                               _stream(stream)))


def version() -> str:
    return lib.hdc_version().decode()
