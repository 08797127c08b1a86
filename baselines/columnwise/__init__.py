"""ctypes front end of cw_sampler.c, the CPU sampler in the paper's column-wise layout (Sec. 5.1).
BASELINE / TEST INFRASTRUCTURE ONLY, not the oracle (that is oracle/): imported by tests/ and by
bench.py's CPU leg.  ``build()`` compiles it with gcc; ``load()`` builds it if it is missing."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cw_sampler.c")
LIB = os.path.join(HERE, "libcw.so")
# no fused multiply-add out of separately rounded operations: the penalties are defined in
# IEEE fp32, one rounding per operation
FLAGS = ["-O3", "-fopenmp", "-mavx2", "-mfma", "-ffp-contract=off", "-fPIC", "-shared", "-Wall"]
_FIELDS = ("temperature", "top_k", "top_p", "min_p", "repetition_penalty", "frequency_penalty",
           "presence_penalty", "row_id")
_DTYPES = dict(temperature=np.float32, top_k=np.int32, top_p=np.float32, min_p=np.float32,
               repetition_penalty=np.float32, frequency_penalty=np.float32, presence_penalty=np.float32,
               row_id=np.int64)


class _Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in _FIELDS]


def build() -> str:
    res = subprocess.run(["gcc"] + FLAGS + ["-o", LIB + ".tmp", SRC, "-lm"], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        lib = ctypes.CDLL(LIB)
        lib.cw_create.restype = ctypes.c_void_p
        lib.cw_create.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.cw_destroy.argtypes = [ctypes.c_void_p]
        lib.cw_threads.restype = ctypes.c_int
        lib.cw_threads.argtypes = [ctypes.c_void_p]
        lib.cw_push_tokens.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        lib.cw_set_history.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64]
        lib.cw_load_f32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        lib.cw_load_bf16.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        lib.cw_sample.restype = ctypes.c_int
        lib.cw_sample.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Params), ctypes.c_uint64, ctypes.c_uint64,
                                  ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


class ColumnwiseSampler:
    """Persistent column-wise state of one batch of B sequences over a vocabulary of V."""

    def __init__(self, B: int, V: int, threads: int = 0):
        self.lib = load()
        self.B, self.V = B, V
        self.h = self.lib.cw_create(B, V, threads)
        if not self.h:
            raise MemoryError("cw_create failed")
        self.threads = int(self.lib.cw_threads(self.h))

    def close(self):
        if self.h:
            self.lib.cw_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def set_history(self, b: int, tokens) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        self.lib.cw_set_history(self.h, b, t.ctypes.data, t.size)

    def push_tokens(self, tokens) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        assert t.size == self.B
        self.lib.cw_push_tokens(self.h, t.ctypes.data)

    def load_logits(self, logits: np.ndarray, v0: int = 0) -> None:
        """``logits``: row-major [B, n] float32, or uint16 holding bf16 bit patterns; goes to
        vocabulary ids v0 .. v0 + n - 1."""
        assert logits.ndim == 2 and logits.shape[0] == self.B and logits.strides[1] == logits.itemsize
        assert v0 + logits.shape[1] <= self.V
        stride = logits.strides[0] // logits.itemsize
        if logits.dtype == np.float32:
            self.lib.cw_load_f32(self.h, logits.ctypes.data, stride, v0, logits.shape[1])
        elif logits.dtype == np.uint16:
            self.lib.cw_load_bf16(self.h, logits.ctypes.data, stride, v0, logits.shape[1])
        else:
            raise TypeError("float32 or uint16 (bf16 bits)")

    def sample(self, params: Dict[str, Optional[np.ndarray]], seed: int, step: int, n_logprobs: int = 0,
               row_ids: Optional[np.ndarray] = None):
        p = _Params()
        keep = []
        for name in _FIELDS:
            arr = row_ids if name == "row_id" else params.get(name)
            if arr is not None:
                arr = np.ascontiguousarray(arr, dtype=_DTYPES[name])
                assert arr.size == self.B
                keep.append(arr)
                setattr(p, name, arr.ctypes.data)
        ids = np.empty(self.B, dtype=np.int32)
        lp_ids = np.empty((self.B, 1 + n_logprobs), dtype=np.int32)
        lp = np.empty((self.B, 1 + n_logprobs), dtype=np.float32)
        rc = self.lib.cw_sample(self.h, ctypes.byref(p), seed, step, n_logprobs, ids.ctypes.data,
                                lp_ids.ctypes.data, lp.ctypes.data)
        if rc != 0:
            raise RuntimeError(f"cw_sample returned {rc}")
        return ids, lp_ids, lp
