"""ctypes binding of libadadim.so: same names as the C ABI (include/adadim.h).

Argument marshalling only.  Tensors are torch CUDA(ROCm) tensors used purely as
device memory; every step of the search runs in the library's HIP kernels.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadadim.so")

OK, EINVAL, ENULL, EALIGN, EHIP = 0, -1, -2, -3, -4
DIM_OC, DIM_IC = 0, 1
DW_F32, DW_F16, DW_F16_SCALED = 0, 1, 2

EXPORTS = (
    "adadim_create", "adadim_destroy", "adadim_last_error", "adadim_version", "adadim_score_elems",
    "adadim_hessian", "adadim_quantize", "adadim_hessian_prepare",
    "adadim_layer_error", "adadim_layer_error_prepared", "adadim_layer_error_batch", "adadim_select",
    "adadim_gemv_ic", "adadim_gptq_prepare", "adadim_gptq_quantize",
    "adadim_quantize_meta16", "adadim_gemv_ic_meta16",
    "adadim_hessian_prepared", "adadim_layer_error_batch_select", "adadim_quantize_both", "adadim_gptq_quantize_meta16", "adadim_capture_begin", "adadim_capture_end", "adadim_graph_launch", "adadim_graph_destroy",
    "adadim_profile", "adadim_profile_only", "adadim_profile_read", "adadim_profile_read_spread",
    "adadim_probe_gram_timeline", "adadim_probe_gemv_read",
    "adadim_layer_error_batch_select_noalloc", "adadim_noalloc_scratch_bytes", "adadim_probe_mfma", "adadim_probe_mfma_f64",
)

_lib = None


def score_elems(rows: int, cols: int) -> int:
    """Elements a scoring-layout buffer for an [rows, cols] operand must hold (adadim_score_elems)."""
    return int(load_library().adadim_score_elems(rows, cols))


def from_score_layout(a, rows: int, cols: int):
    """Row-major [rows, cols] view of a numpy array held in the library's scoring layout
    (ADADIM_DW_F16_SCALED dW and the prepared Hs): [row tile of 256][column block of 32]
    [256 rows][32 columns] when cols is a multiple of 32, the last row tile padded; row-major
    otherwise.  Index shuffling only."""
    import numpy as np
    a = np.asarray(a).reshape(-1)
    if cols % 32:
        return a[:rows * cols].reshape(rows, cols)
    tiles = (rows + 255) // 256
    t = a[:tiles * 256 * cols].reshape(tiles, cols // 32, 256, 32).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(t).reshape(tiles * 256, cols)[:rows]


class AdaDimError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"adadim error {code}: {text}")
        self.code = code


def load_library(path: str | None = None) -> ctypes.CDLL:
    """Loads the built shared library; raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} is missing: build it with `python -m paper_2309_15531_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(p)
    lib.adadim_create.argtypes = [POINTER(c_void_p), c_void_p]
    lib.adadim_create.restype = c_int
    lib.adadim_destroy.argtypes = [c_void_p]
    lib.adadim_destroy.restype = None
    lib.adadim_last_error.argtypes = [c_void_p]
    lib.adadim_last_error.restype = c_char_p
    lib.adadim_version.argtypes = []
    lib.adadim_version.restype = c_char_p
    lib.adadim_score_elems.argtypes = [c_int64, c_int64]
    lib.adadim_score_elems.restype = c_int64
    lib.adadim_hessian.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int]
    lib.adadim_hessian.restype = c_int
    lib.adadim_quantize.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_float,
                                    c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    lib.adadim_quantize.restype = c_int
    lib.adadim_quantize_meta16.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_float,
                                           c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p]
    lib.adadim_quantize_meta16.restype = c_int
    lib.adadim_gemv_ic_meta16.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int, c_int,
                                          c_void_p]
    lib.adadim_gemv_ic_meta16.restype = c_int
    lib.adadim_quantize_both.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_float, c_int, c_void_p] + \
        [c_void_p] * 10
    lib.adadim_quantize_both.restype = c_int
    lib.adadim_hessian_prepared.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
    lib.adadim_hessian_prepared.restype = c_int
    lib.adadim_capture_begin.argtypes = [c_void_p]
    lib.adadim_capture_begin.restype = c_int
    lib.adadim_capture_end.argtypes = [c_void_p, POINTER(c_void_p)]
    lib.adadim_capture_end.restype = c_int
    lib.adadim_graph_launch.argtypes = [c_void_p, c_void_p]
    lib.adadim_graph_launch.restype = c_int
    lib.adadim_graph_destroy.argtypes = [c_void_p]
    lib.adadim_graph_destroy.restype = None
    lib.adadim_hessian_prepare.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_void_p]
    lib.adadim_hessian_prepare.restype = c_int
    lib.adadim_layer_error.argtypes = [c_void_p, c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
    lib.adadim_layer_error.restype = c_int
    lib.adadim_layer_error_prepared.argtypes = [c_void_p, c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p,
                                                c_void_p, c_void_p]
    lib.adadim_layer_error_prepared.restype = c_int
    lib.adadim_layer_error_batch.argtypes = [c_void_p, c_int, POINTER(c_void_p), c_int, c_int64, c_int64, c_void_p,
                                             c_void_p, c_void_p, c_void_p]
    lib.adadim_layer_error_batch.restype = c_int
    lib.adadim_layer_error_batch_select.argtypes = [c_void_p, c_int, POINTER(c_void_p), c_int, c_int64, c_int64,
                                                    c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.adadim_layer_error_batch_select.restype = c_int
    lib.adadim_layer_error_batch_select_noalloc.argtypes = [c_void_p, c_int, POINTER(c_void_p), c_int64, c_int64,
                                                            c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.adadim_layer_error_batch_select_noalloc.restype = c_int
    lib.adadim_noalloc_scratch_bytes.argtypes = [c_int, c_int64, c_int64]
    lib.adadim_noalloc_scratch_bytes.restype = c_int64
    lib.adadim_probe_mfma.argtypes = [c_void_p, c_int, c_int, POINTER(ctypes.c_double), POINTER(ctypes.c_double)]
    lib.adadim_probe_mfma.restype = c_int
    lib.adadim_probe_mfma_f64.argtypes = [c_void_p, c_int, POINTER(ctypes.c_double), POINTER(ctypes.c_double)]
    lib.adadim_probe_mfma_f64.restype = c_int
    lib.adadim_select.argtypes = [c_void_p, c_void_p, c_int, c_void_p, POINTER(c_int32)]
    lib.adadim_select.restype = c_int
    lib.adadim_profile.argtypes = [c_void_p, c_int]
    lib.adadim_profile.restype = c_int
    lib.adadim_profile_only.argtypes = [c_void_p, ctypes.c_char_p]
    lib.adadim_profile_only.restype = c_int
    lib.adadim_profile_read.argtypes = [c_void_p, c_int, ctypes.c_char_p, c_int, POINTER(ctypes.c_double),
                                        POINTER(c_int64)]
    lib.adadim_profile_read.restype = c_int
    lib.adadim_probe_gemv_read.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, POINTER(ctypes.c_double)]
    lib.adadim_probe_gemv_read.restype = c_int
    lib.adadim_probe_gram_timeline.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int,
                                               POINTER(ctypes.c_float), c_int, POINTER(c_int), POINTER(c_int)]
    lib.adadim_probe_gram_timeline.restype = c_int
    lib.adadim_profile_read_spread.argtypes = [c_void_p, c_int] + [POINTER(ctypes.c_double)] * 3
    lib.adadim_profile_read_spread.restype = c_int
    lib.adadim_gemv_ic.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int, c_int,
                                   c_void_p]
    lib.adadim_gemv_ic.restype = c_int
    lib.adadim_gptq_prepare.argtypes = [c_void_p, c_void_p, c_int64, c_float, c_int, c_void_p, c_void_p, c_void_p]
    lib.adadim_gptq_prepare.restype = c_int
    lib.adadim_gptq_quantize.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_void_p, c_void_p,
                                         c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.adadim_gptq_quantize.restype = c_int
    lib.adadim_gptq_quantize_meta16.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_void_p, c_void_p,
                                                c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.adadim_gptq_quantize_meta16.restype = c_int
    if path is None:
        _lib = lib
    return lib


def _ptr(t):
    """Device address of a torch tensor (None -> NULL); plain ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return c_void_p(t)
    return c_void_p(t.data_ptr())


def _need(t, what: str, dtype: str | None = None, pitched: bool = False):
    """Raises unless the torch tensor `t` can be handed to the library as `what`: on the GPU, of the element type
    the ABI documents (`dtype`: "float16", "float32", ...; None = any), unit stride along the last axis and, unless
    `pitched` (X: the row pitch travels as ldx), contiguous.  The library sees only an address: a transposed view
    or a tensor of another type would be read as something it is not.  None and raw addresses pass."""
    if t is None or isinstance(t, int):
        return
    if not t.is_cuda:
        raise TypeError(f"{what}: expected a device tensor, got one on {t.device}")
    if dtype is not None and str(t.dtype) != "torch." + dtype:
        raise TypeError(f"{what}: expected {dtype}, got {t.dtype}")
    if t.dim() >= 1 and t.numel() > 0 and t.stride(-1) != 1:
        raise ValueError(f"{what}: the last axis must have unit stride (strides {tuple(t.stride())}); pass a contiguous "
                         "tensor, not a transposed view")
    if not pitched and not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous (shape {tuple(t.shape)}, strides {tuple(t.stride())})")


class Context:
    """One adadim_ctx bound to a HIP stream (default: torch's current stream)."""

    def __init__(self, stream: int | None = None):
        self._lib = load_library()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
        self.stream = stream
        h = c_void_p()
        rc = self._lib.adadim_create(byref(h), c_void_p(stream))
        if rc != OK:
            raise AdaDimError(rc, self._lib.adadim_last_error(None).decode())
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.adadim_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self._lib.adadim_last_error(self._h).decode()

    def _check(self, rc: int):
        if rc != OK:
            raise AdaDimError(rc, self.last_error())

    # -- raw calls: return the status code, never raise ------------------
    def raw(self, name: str, *args) -> int:
        return getattr(self._lib, name)(self._h, *args)

    # -- the ABI, one method per entry point ----------------------------
    def adadim_hessian(self, X, H, accumulate: bool = False, tokens: int | None = None):
        t = X.shape[0] if tokens is None else tokens
        _need(X, "X", "float16", pitched=True)
        _need(H, "H", "float32")
        self._check(self._lib.adadim_hessian(self._h, _ptr(X), t, X.shape[1], X.stride(0), _ptr(H),
                                             1 if accumulate else 0))

    def adadim_quantize(self, W, dim: int, bits: int, group: int, clip: float = 1.0, codes=None, scales=None,
                        zeros=None, dW=None, dW_dtype: int = DW_F32, colscale=None, packed=None):
        out_f, in_f = W.shape
        _need(W, "W", "float16")
        _need(codes, "codes", "uint8"); _need(scales, "scales", "float32"); _need(zeros, "zeros", "uint8")
        _need(dW, "dW", "float32" if dW_dtype == DW_F32 else "float16"); _need(colscale, "colscale", "float32")
        _need(packed, "packed")
        self._check(self._lib.adadim_quantize(self._h, _ptr(W), out_f, in_f, dim, bits, group, c_float(clip),
                                              _ptr(codes), _ptr(scales), _ptr(zeros), _ptr(dW), dW_dtype,
                                              _ptr(colscale), _ptr(packed)))

    def adadim_quantize_meta16(self, W, dim: int, bits: int, group: int, clip: float = 1.0, codes=None, meta=None,
                               dW=None, dW_dtype: int = DW_F32, colscale=None, packed=None):
        out_f, in_f = W.shape
        _need(W, "W", "float16")
        _need(codes, "codes", "uint8"); _need(meta, "meta")
        _need(dW, "dW", "float32" if dW_dtype == DW_F32 else "float16"); _need(colscale, "colscale", "float32")
        _need(packed, "packed")
        self._check(self._lib.adadim_quantize_meta16(self._h, _ptr(W), out_f, in_f, dim, bits, group, c_float(clip),
                                                     _ptr(codes), _ptr(meta), _ptr(dW), dW_dtype, _ptr(colscale),
                                                     _ptr(packed)))

    def adadim_quantize_both(self, W, bits: int, group: int, colscale, oc: dict, ic: dict, clip: float = 1.0,
                             meta16: bool = False):
        """oc / ic: dicts with any of codes, scales (or meta when meta16), zeros, dW, packed."""
        out_f, in_f = W.shape
        _need(W, "W", "float16")
        _need(colscale, "colscale", "float32")
        for d in (oc, ic):
            _need(d.get("codes"), "codes", "uint8"); _need(d.get("dW"), "dW", "float16"); _need(d.get("packed"), "packed")
            _need(d.get("zeros"), "zeros", "uint8")
            _need(d.get("meta") if meta16 else d.get("scales"), "scales", None if meta16 else "float32")

        def five(d):
            return [_ptr(d.get("codes")), _ptr(d.get("meta") if meta16 else d.get("scales")), _ptr(d.get("zeros")),
                    _ptr(d.get("dW")), _ptr(d.get("packed"))]
        self._check(self._lib.adadim_quantize_both(self._h, _ptr(W), out_f, in_f, bits, group, c_float(clip),
                                                   1 if meta16 else 0, _ptr(colscale), *five(oc), *five(ic)))

    def alloc_score(self, rows: int, cols: int, device="cuda"):
        """Flat fp16 device buffer large enough for an [rows, cols] operand in the scoring layout."""
        import torch
        return torch.empty(score_elems(rows, cols), dtype=torch.float16, device=device)

    def adadim_hessian_prepared(self, X, H, Hs, hmeta, tokens: int | None = None):
        t = X.shape[0] if tokens is None else tokens
        _need(X, "X", "float16", pitched=True)
        _need(H, "H", "float32"); _need(Hs, "Hs", "float16"); _need(hmeta, "hmeta", "float32")
        self._check(self._lib.adadim_hessian_prepared(self._h, _ptr(X), t, X.shape[1], X.stride(0), _ptr(H), _ptr(Hs),
                                                      _ptr(hmeta)))

    def adadim_hessian_prepare(self, H, Hs, hmeta):
        _need(H, "H", "float32"); _need(Hs, "Hs", "float16"); _need(hmeta, "hmeta", "float32")
        self._check(self._lib.adadim_hessian_prepare(self._h, _ptr(H), H.shape[0], _ptr(Hs), _ptr(hmeta)))

    def adadim_layer_error(self, dW, dW_dtype: int, H, loss, loss_rows=None):
        out_f, in_f = dW.shape
        _need(dW, "dW", "float32" if dW_dtype == DW_F32 else "float16"); _need(H, "H", "float32")
        _need(loss, "loss", "float32"); _need(loss_rows, "loss_rows", "float32")
        self._check(self._lib.adadim_layer_error(self._h, _ptr(dW), dW_dtype, out_f, in_f, _ptr(H),
                                                 _ptr(loss_rows), _ptr(loss)))

    def adadim_layer_error_prepared(self, dW, dW_dtype: int, Hs, hmeta, loss, loss_rows=None, shape=None):
        """shape = (out, in) when dW is a flat scoring-layout buffer (see alloc_score)."""
        out_f, in_f = dW.shape if shape is None else shape
        _need(dW, "dW", "float32" if dW_dtype == DW_F32 else "float16"); _need(Hs, "Hs", "float16")
        _need(hmeta, "hmeta", "float32"); _need(loss, "loss", "float32"); _need(loss_rows, "loss_rows", "float32")
        self._check(self._lib.adadim_layer_error_prepared(self._h, _ptr(dW), dW_dtype, out_f, in_f, _ptr(Hs),
                                                          _ptr(hmeta), _ptr(loss_rows), _ptr(loss)))

    def adadim_layer_error_batch(self, dWs, dW_dtype: int, Hs, hmeta, losses, loss_rows=None, shape=None):
        out_f, in_f = dWs[0].shape if shape is None else shape
        for t in dWs:
            _need(t, "dW", "float32" if dW_dtype == DW_F32 else "float16")
        _need(Hs, "Hs", "float16"); _need(hmeta, "hmeta", "float32"); _need(losses, "losses", "float32")
        _need(loss_rows, "loss_rows", "float32")
        arr = (c_void_p * len(dWs))(*[t.data_ptr() for t in dWs])
        self._check(self._lib.adadim_layer_error_batch(self._h, len(dWs), arr, dW_dtype, out_f, in_f, _ptr(Hs),
                                                       _ptr(hmeta), _ptr(loss_rows), _ptr(losses)))

    def adadim_layer_error_batch_select(self, dWs, dW_dtype: int, Hs, hmeta, losses, best_dev, loss_rows=None, shape=None):
        out_f, in_f = dWs[0].shape if shape is None else shape
        for t in dWs:
            _need(t, "dW", "float32" if dW_dtype == DW_F32 else "float16")
        _need(Hs, "Hs", "float16"); _need(hmeta, "hmeta", "float32"); _need(losses, "losses", "float32")
        _need(loss_rows, "loss_rows", "float32")
        arr = (c_void_p * len(dWs))(*[t.data_ptr() for t in dWs])
        self._check(self._lib.adadim_layer_error_batch_select(self._h, len(dWs), arr, dW_dtype, out_f, in_f, _ptr(Hs),
                                                              _ptr(hmeta), _ptr(loss_rows), _ptr(losses), _ptr(best_dev)))

    def adadim_layer_error_batch_select_noalloc(self, dWs, Hs, hmeta, losses, best_dev, loss_rows=None, shape=None):
        """The same call with its scratch in the library's fixed device array (no allocation); dWs are
        column-scaled fp16 buffers in the scoring layout, at most eight."""
        out_f, in_f = dWs[0].shape if shape is None else shape
        arr = (c_void_p * len(dWs))(*[t.data_ptr() for t in dWs])
        self._check(self._lib.adadim_layer_error_batch_select_noalloc(self._h, len(dWs), arr, out_f, in_f, _ptr(Hs),
                                                                      _ptr(hmeta), _ptr(loss_rows), _ptr(losses),
                                                                      _ptr(best_dev)))

    def adadim_select(self, losses, n: int | None = None, best_dev=None, to_host: bool = True):
        n = losses.numel() if n is None else n
        host = c_int32(-1)
        self._check(self._lib.adadim_select(self._h, _ptr(losses), n, _ptr(best_dev),
                                            byref(host) if to_host else None))
        return host.value if to_host else None

    def adadim_gemv_ic(self, packed, scales, zeros, x, out_f: int, in_f: int, bits: int, group: int, y):
        self._check(self._lib.adadim_gemv_ic(self._h, _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(x), out_f, in_f,
                                             bits, group, _ptr(y)))

    def adadim_gemv_ic_meta16(self, packed, meta, x, out_f: int, in_f: int, bits: int, group: int, y):
        self._check(self._lib.adadim_gemv_ic_meta16(self._h, _ptr(packed), _ptr(meta), _ptr(x), out_f, in_f, bits, group,
                                                    _ptr(y)))

    def adadim_capture_begin(self):
        self._check(self._lib.adadim_capture_begin(self._h))

    def adadim_capture_end(self):
        """Returns the graph handle (an int); free it with adadim_graph_destroy."""
        g = c_void_p()
        self._check(self._lib.adadim_capture_end(self._h, byref(g)))
        return g.value

    def adadim_graph_launch(self, graph: int):
        self._check(self._lib.adadim_graph_launch(self._h, c_void_p(graph)))

    def adadim_graph_destroy(self, graph):
        if graph:
            self._lib.adadim_graph_destroy(c_void_p(graph))

    def adadim_gptq_prepare(self, H, perm, dead, U, percdamp: float = 0.01, act_order: bool = True):
        self._check(self._lib.adadim_gptq_prepare(self._h, _ptr(H), H.shape[0], c_float(percdamp), 1 if act_order else 0,
                                                  _ptr(perm), _ptr(dead), _ptr(U)))

    def adadim_gptq_quantize_meta16(self, W, dim: int, bits: int, group: int, U, perm, dead, codes, static_meta=None,
                                    meta=None, dW=None, packed=None):
        out_f, in_f = W.shape
        self._check(self._lib.adadim_gptq_quantize_meta16(self._h, _ptr(W), out_f, in_f, dim, bits, group, _ptr(U),
                                                          _ptr(perm), _ptr(dead), _ptr(static_meta), _ptr(codes),
                                                          _ptr(meta), _ptr(dW), _ptr(packed)))

    def adadim_gptq_quantize(self, W, dim: int, bits: int, group: int, U, perm, dead, codes, static_scales=None,
                             static_zeros=None, scales=None, zeros=None, dW=None, packed=None):
        out_f, in_f = W.shape
        self._check(self._lib.adadim_gptq_quantize(self._h, _ptr(W), out_f, in_f, dim, bits, group, _ptr(U), _ptr(perm),
                                                   _ptr(dead), _ptr(static_scales), _ptr(static_zeros), _ptr(codes),
                                                   _ptr(scales), _ptr(zeros), _ptr(dW), _ptr(packed)))

    def adadim_probe_mfma_f64(self, iters: int = 20000):
        """(TFLOP/s, shader clock in MHz) of a register-resident fp64 MFMA loop; waits for the stream."""
        tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
        self._check(self._lib.adadim_probe_mfma_f64(self._h, iters, byref(tf), byref(mhz)))
        return tf.value, mhz.value

    def adadim_probe_gemv_read(self, packed, out_f: int, in_f: int, bits: int) -> float:
        """Microseconds of one launch that only reads the code stream the way the matrix-vector kernel does."""
        _need(packed, "packed", "int32")
        us = ctypes.c_double(0.0)
        self._check(self._lib.adadim_probe_gemv_read(self._h, _ptr(packed), out_f, in_f, bits, byref(us)))
        return us.value

    def adadim_probe_gram_timeline(self, X, dispatcher: bool = False):
        """(records [pieces, 8] as a numpy array, plan as 8 ints) of one time-stamped launch of the Gram tile kernel."""
        import numpy as np
        _need(X, "X", "float16", pitched=True)
        cap = 8192
        rec = np.zeros((cap, 8), dtype=np.float32)
        n, plan = c_int(0), (c_int * 8)()
        self._check(self._lib.adadim_probe_gram_timeline(
            self._h, _ptr(X), X.shape[0], X.shape[1], X.stride(0), 1 if dispatcher else 0,
            rec.ctypes.data_as(POINTER(ctypes.c_float)), cap, byref(n), plan))
        return rec[:n.value].copy(), [int(v) for v in plan]

    def adadim_probe_mfma(self, random_operands: bool, iters: int = 4000):
        """(TFLOP/s, shader clock in MHz) of a register-resident MFMA loop; waits for the stream."""
        tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
        self._check(self._lib.adadim_probe_mfma(self._h, 1 if random_operands else 0, iters, byref(tf), byref(mhz)))
        return tf.value, mhz.value

    def adadim_profile(self, enable: bool):
        self._check(self._lib.adadim_profile(self._h, 1 if enable else 0))

    def adadim_profile_only(self, name: str | None):
        """Bracket only the kernel of that name with events (None: every kernel again)."""
        self._check(self._lib.adadim_profile_only(self._h, name.encode() if name else None))

    def adadim_profile_read(self, spread: bool = False) -> dict:
        """All per-kernel records: {kernel name: (total ms, launches)}; with spread, (total ms, launches, smallest,
        median and largest ms of a launch)."""
        out, idx = {}, 0
        while True:
            name = ctypes.create_string_buffer(64)
            ms, n = ctypes.c_double(0.0), c_int64(0)
            rc = self._lib.adadim_profile_read(self._h, idx, name, 64, byref(ms), byref(n))
            if rc == EINVAL:
                return out
            self._check(rc)
            rec = (ms.value, n.value)
            if spread:
                lo, mid, hi = ctypes.c_double(0.0), ctypes.c_double(0.0), ctypes.c_double(0.0)
                self._check(self._lib.adadim_profile_read_spread(self._h, idx, byref(lo), byref(mid), byref(hi)))
                rec += (lo.value, mid.value, hi.value)
            out[name.value.decode()] = rec
            idx += 1
