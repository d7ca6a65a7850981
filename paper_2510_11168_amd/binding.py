"""Thin ctypes binding of libelmo_head.so: argument marshalling only.

Every step of the head's hot path runs in the library's HIP kernels.  PyTorch is used for device
memory and streams and nothing else.  There is no fallback: if the shared library is missing the
import of this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from .build import LIB_PATH

ELMO_BF16 = 0
ELMO_FP8_E4M3 = 1
ELMO_FP32 = 2
ELMO_SR = 1
ELMO_KAHAN = 2
ELMO_VALIDATE = 4


class ElmoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"elmo_head error {code}: {text}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(the HIP library is the only implementation, there is no CPU path)")

_lib = C.CDLL(LIB_PATH)


class elmo_head_opts(C.Structure):
    _fields_ = [
        ("flags", C.c_uint32), ("max_B", C.c_int32), ("max_nnz", C.c_int64),
        ("W", C.c_void_p), ("W_bytes", C.c_size_t),
        ("comp", C.c_void_p), ("comp_bytes", C.c_size_t), ("kahan_rows", C.c_int64), ("weight_decay", C.c_float),
        ("dropout_p", C.c_float),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


_lib.elmo_last_error.restype = C.c_char_p
_lib.elmo_last_error.argtypes = []
_lib.elmo_logit_buffer_bytes.restype = C.c_size_t
_lib.elmo_logit_buffer_bytes.argtypes = [C.c_int64, C.c_int64]
_lib.elmo_head_sizes.restype = C.c_int
_lib.elmo_head_sizes.argtypes = [C.c_int64, C.c_int32, C.c_int, C.c_int64, C.c_int32, C.c_int64, C.c_uint32, C.c_int64,
                                 C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
_lib.elmo_head_create.restype = C.c_int
_lib.elmo_head_create.argtypes = [C.c_int64, C.c_int32, C.c_int, C.c_int64, C.POINTER(elmo_head_opts),
                                  C.POINTER(C.c_void_p)]
_lib.elmo_head_step.restype = C.c_int
_lib.elmo_head_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.elmo_quantize_em.restype = C.c_int
_lib.elmo_quantize_em.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_uint64, C.c_uint64,
                                  C.c_void_p, C.c_void_p]
_lib.elmo_precision_hits.restype = C.c_int
_lib.elmo_precision_hits.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.elmo_head_topk.restype = C.c_int
_lib.elmo_head_topk.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.elmo_topk_static.restype = C.c_int
_lib.elmo_topk_static.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                  C.c_void_p, C.c_void_p]
_lib.elmo_head_destroy.restype = C.c_int
_lib.elmo_head_destroy.argtypes = [C.c_void_p]
_lib.elmo_head_profile.restype = C.c_int
_lib.elmo_head_profile.argtypes = [C.c_void_p, C.c_int]
_lib.elmo_head_profile_read.restype = C.c_int
_lib.elmo_head_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
_lib.elmo_quantize.restype = C.c_int
_lib.elmo_quantize.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_uint64, C.c_uint64,
                               C.c_void_p, C.c_void_p]
_lib.elmo_philox4x32_10.restype = None
_lib.elmo_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
_lib.elmo_kahan_adamw.restype = C.c_int
_lib.elmo_kahan_adamw.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_float,
                                  C.c_double, C.c_double, C.c_float, C.c_float, C.c_int64, C.c_void_p]
_lib.elmo_dropout_keep16.restype = C.c_uint32
_lib.elmo_dropout_keep16.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32]

EXPORTS = ("elmo_last_error", "elmo_logit_buffer_bytes", "elmo_head_sizes", "elmo_head_create",
           "elmo_head_step", "elmo_head_topk", "elmo_head_destroy", "elmo_quantize", "elmo_philox4x32_10",
           "elmo_head_profile", "elmo_head_profile_read", "elmo_precision_hits", "elmo_quantize_em",
           "elmo_dropout_keep16", "elmo_kahan_adamw", "elmo_topk_static")


def _check(rc: int) -> None:
    if rc != 0:
        raise ElmoError(rc, elmo_last_error())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        if not torch.cuda.is_available():
            return 0          # no device: only argument checks can run, on the null stream
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


# ------------------------------------------------------------------ the C entry points, same names
def elmo_last_error() -> str:
    return _lib.elmo_last_error().decode()


def elmo_logit_buffer_bytes(batch: int, labels: int) -> int:
    return int(_lib.elmo_logit_buffer_bytes(batch, labels))


def elmo_head_sizes(L, d, weight_dtype, chunk, max_B, max_nnz, flags, kahan_rows=0):
    w, c, s = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(_lib.elmo_head_sizes(L, d, weight_dtype, chunk, max_B, max_nnz, flags, kahan_rows, C.byref(w), C.byref(c), C.byref(s)))
    return w.value, c.value, s.value


def elmo_head_create(L, d, weight_dtype, chunk, *, flags, max_B, max_nnz, W, comp, workspace, kahan_rows=0,
                     weight_decay=0.0, dropout_p=0.0) -> int:
    """W, comp, workspace: 1-D torch.uint8 device tensors (comp may be None).  Returns the handle."""
    o = elmo_head_opts(flags=flags, max_B=max_B, max_nnz=max_nnz,
                       W=_ptr(W), W_bytes=0 if W is None else W.numel() * W.element_size(),
                       comp=_ptr(comp), comp_bytes=0 if comp is None else comp.numel() * comp.element_size(),
                       kahan_rows=kahan_rows, weight_decay=weight_decay, dropout_p=dropout_p,
                       workspace=_ptr(workspace),
                       workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size())
    h = C.c_void_p()
    _check(_lib.elmo_head_create(L, d, weight_dtype, chunk, C.byref(o), C.byref(h)))
    return h.value


def elmo_head_step(h, X, B, indptr, indices, nnz, lr, seed, step, dX_out=None, loss_out=None, stream=None) -> None:
    _check(_lib.elmo_head_step(h, _ptr(X), B, _ptr(indptr), _ptr(indices), nnz, lr, seed, step,
                               _ptr(dX_out), _ptr(loss_out), _stream(stream)))


def elmo_head_topk(h, X, B, k, idx_out=None, score_out=None, stream=None) -> None:
    _check(_lib.elmo_head_topk(h, _ptr(X), B, k, _ptr(idx_out), _ptr(score_out), _stream(stream)))


def elmo_topk_static(W, L, d, weight_dtype, X, B, k, idx_out=None, score_out=None, stream=None) -> None:
    _check(_lib.elmo_topk_static(_ptr(W), L, d, weight_dtype, _ptr(X), B, k, _ptr(idx_out), _ptr(score_out), _stream(stream)))


def elmo_quantize_em(src, n, exp_bits, man_bits, mode, seed, step, first_elem, dst, stream=None) -> None:
    _check(_lib.elmo_quantize_em(_ptr(src), n, exp_bits, man_bits, mode, seed, step, first_elem, _ptr(dst), _stream(stream)))


def elmo_precision_hits(idx, B, k, indptr, indices, hits_out, stream=None) -> None:
    """hits_out: torch.int64 device tensor of k entries; P@j = hits_out[j-1] / (j * B)."""
    _check(_lib.elmo_precision_hits(_ptr(idx), B, k, _ptr(indptr), _ptr(indices), _ptr(hits_out), _stream(stream)))


def elmo_head_destroy(h) -> None:
    _check(_lib.elmo_head_destroy(h))


PROFILE_CLASSES = ("setup", "logits", "dx", "update", "finalize", "topk")


def elmo_head_profile(h, enable: bool) -> None:
    _check(_lib.elmo_head_profile(h, int(enable)))


def elmo_head_profile_read(h):
    """{class: (milliseconds, spans)} accumulated since profiling was enabled / last read."""
    ms = (C.c_double * 6)()
    n = (C.c_int64 * 6)()
    _check(_lib.elmo_head_profile_read(h, ms, n))
    return {name: (ms[i], n[i]) for i, name in enumerate(PROFILE_CLASSES)}


def elmo_quantize(src, n, dtype, mode, seed, step, first_elem, dst, stream=None) -> None:
    _check(_lib.elmo_quantize(_ptr(src), n, dtype, mode, seed, step, first_elem, _ptr(dst), _stream(stream)))


def elmo_kahan_adamw(param, comp, m, v, grad, n, state_dtype, lr, beta1, beta2, eps, weight_decay, t, stream=None) -> None:
    _check(_lib.elmo_kahan_adamw(_ptr(param), _ptr(comp), _ptr(m), _ptr(v), _ptr(grad), n, state_dtype, lr, beta1, beta2, eps,
                                 weight_decay, t, _stream(stream)))


def elmo_dropout_keep16(seed, step, block, threshold) -> int:
    return int(_lib.elmo_dropout_keep16(seed, step, block, threshold))


def elmo_philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    _lib.elmo_philox4x32_10(c, k, o)
    return list(o)


# ------------------------------------------------------------------ convenience owner of the buffers
class Head:
    """Allocates W / comp / workspace as torch device tensors and keeps the handle alive."""

    def __init__(self, L, d, weight_dtype, chunk, flags, max_B, max_nnz, device="cuda:0", kahan_rows=0, weight_decay=0.0,
                 dropout_p=0.0):
        self.L, self.d, self.fmt, self.chunk, self.flags = L, d, weight_dtype, chunk, flags
        self.max_B, self.max_nnz = max_B, max_nnz
        self.kahan_rows = (kahan_rows or L) if flags & ELMO_KAHAN else 0   # label rows that carry compensation
        wb, cb, sb = elmo_head_sizes(L, d, weight_dtype, chunk, max_B, max_nnz, flags, kahan_rows)
        self.W = torch.zeros(wb, dtype=torch.uint8, device=device)
        self.comp = torch.zeros(cb, dtype=torch.uint8, device=device) if cb else None
        self.workspace = torch.empty(sb, dtype=torch.uint8, device=device)
        self.bytes = (wb, cb, sb)
        self.h = elmo_head_create(L, d, weight_dtype, chunk, flags=flags, max_B=max_B, max_nnz=max_nnz,
                                  W=self.W, comp=self.comp, workspace=self.workspace, kahan_rows=kahan_rows,
                                  weight_decay=weight_decay, dropout_p=dropout_p)

    def weights(self):
        """[L, d] view of the raw weight bits: uint8 codes (E4M3) or int16 patterns (BF16)."""
        if self.fmt == ELMO_FP8_E4M3:
            return self.W.view(self.L, self.d)
        return self.W.view(torch.int16).view(self.L, self.d)

    def compensation(self):
        return None if self.comp is None else self.comp.view(torch.int16).view(self.kahan_rows, self.d)

    def step(self, X, indptr, indices, lr, seed, step, dX_out=None, loss_out=None, stream=None):
        elmo_head_step(self.h, X, X.shape[0], indptr, indices, int(indices.numel()), lr, seed, step,
                       dX_out, loss_out, stream)

    def topk(self, X, k, idx_out, score_out, stream=None):
        elmo_head_topk(self.h, X, X.shape[0], k, idx_out, score_out, stream)

    def close(self):
        if self.h is not None:
            elmo_head_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
