"""ctypes binding of libsip.so: the same entry points as include/sip.h, with torch tensors
standing in for device pointers.  Argument marshalling only -- every step of the sampling
path runs in the library's kernels.  There is no fallback: without the compiled library
(or without a GPU) the calls raise."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsip.so")

SIP_F32, SIP_BF16 = 0, 1
SIP_OK, SIP_ERR_INVALID_ARG, SIP_ERR_UNSUPPORTED, SIP_ERR_WORKSPACE, SIP_ERR_HIP, SIP_ERR_TIMEOUT, SIP_ERR_SCRATCH = range(7)
SIP_MAX_V = 1 << 19
SIP_MAX_K_LOGPROBS = 64
SIP_MAX_SLOTS = 1 << 20
SIP_MAX_SHARDS = 8
SIP_MAX_L = 1 << 17

PARAM_FIELDS = ("temperature", "top_k", "top_p", "min_p", "repetition_penalty",
                "frequency_penalty", "presence_penalty", "row_id")
_PARAM_DTYPES = {"temperature": torch.float32, "top_k": torch.int32, "top_p": torch.float32,
                 "min_p": torch.float32, "repetition_penalty": torch.float32,
                 "frequency_penalty": torch.float32, "presence_penalty": torch.float32,
                 "row_id": torch.int64}


class SipParams(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in PARAM_FIELDS]


class SipCall(ctypes.Structure):
    """sip_call of include/sip.h, field for field."""
    _fields_ = [("logits", ctypes.c_void_p), ("row_stride", ctypes.c_int64), ("V", ctypes.c_int32),
                ("shard_logits", ctypes.POINTER(ctypes.c_void_p)), ("t_shards", ctypes.c_int32),
                ("V_shard", ctypes.c_int32), ("shard_stride", ctypes.c_int64), ("B", ctypes.c_int32),
                ("dtype", ctypes.c_int), ("params", ctypes.POINTER(SipParams)),
                ("hist_indptr", ctypes.c_void_p), ("hist_tokens", ctypes.c_void_p), ("hist_nnz", ctypes.c_int64),
                ("state", ctypes.c_void_p), ("state_bytes", ctypes.c_size_t), ("slots", ctypes.c_int32),
                ("L_max", ctypes.c_int32), ("slot_of_row", ctypes.c_void_p),
                ("seed", ctypes.c_uint64), ("step", ctypes.c_uint64),
                ("out_ids", ctypes.c_void_p), ("out_lp_ids", ctypes.c_void_p), ("out_lp", ctypes.c_void_p),
                ("k_logprobs", ctypes.c_int32),
                ("host_ids", ctypes.c_void_p), ("host_flag", ctypes.c_void_p), ("ticket", ctypes.c_uint64),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t), ("hip_stream", ctypes.c_void_p),
                ("prompt_indptr", ctypes.c_void_p), ("prompt_tokens", ctypes.c_void_p), ("prompt_nnz", ctypes.c_int64)]


class SipError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"sip_sample failed: {sip_status_string(status)} (status {status})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libsip.so (built by paper_2506_22033_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2506_22033_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        lib.sip_workspace_bytes.restype = ctypes.c_size_t
        lib.sip_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_int64,
                                            ctypes.c_int32]
        lib.sip_sample.restype = ctypes.c_int
        lib.sip_sample.argtypes = [
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int,
            ctypes.POINTER(SipParams), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.sip_init.restype = ctypes.c_int
        lib.sip_init.argtypes = []
        lib.sip_noalloc_scratch_bytes.restype = ctypes.c_size_t
        lib.sip_noalloc_scratch_bytes.argtypes = []
        lib.sip_sample_noalloc.restype = ctypes.c_int
        lib.sip_sample_noalloc.argtypes = [
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int,
            ctypes.POINTER(SipParams), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_void_p]
        lib.sip_workspace_bytes_sharded.restype = ctypes.c_size_t
        lib.sip_workspace_bytes_sharded.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
                                                    ctypes.c_int64, ctypes.c_int32]
        lib.sip_sample_sharded.restype = ctypes.c_int
        lib.sip_sample_sharded.argtypes = [
            ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
            ctypes.c_int, ctypes.POINTER(SipParams), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.sip_publish_ids.restype = ctypes.c_int
        lib.sip_publish_ids.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_uint64, ctypes.c_void_p]
        lib.sip_wait_ids.restype = ctypes.c_int
        lib.sip_wait_ids.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64]
        lib.sip_probe_read.restype = ctypes.c_int
        lib.sip_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_void_p,
                                       ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.sip_call_workspace_bytes.restype = ctypes.c_size_t
        lib.sip_call_workspace_bytes.argtypes = [ctypes.POINTER(SipCall)]
        lib.sip_sample_call.restype = ctypes.c_int
        lib.sip_sample_call.argtypes = [ctypes.POINTER(SipCall)]
        lib.sip_plan_chunks.restype = ctypes.c_int32
        lib.sip_plan_chunks.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_int32]
        lib.sip_state_bytes.restype = ctypes.c_size_t
        lib.sip_state_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
        lib.sip_state_init.restype = ctypes.c_int
        lib.sip_state_init.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_void_p]
        lib.sip_state_assign.restype = ctypes.c_int
        lib.sip_state_assign.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int64, ctypes.c_void_p]
        lib.sip_sample_state.restype = ctypes.c_int
        lib.sip_sample_state.argtypes = [
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int,
            ctypes.POINTER(SipParams), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.sip_status_string.restype = ctypes.c_char_p
        lib.sip_status_string.argtypes = [ctypes.c_int]
        lib.sip_profile_kernel_events.restype = None
        lib.sip_profile_kernel_events.argtypes = [ctypes.c_void_p] * 6
        lib.sip_version.restype = ctypes.c_int
        lib.sip_version.argtypes = []
        _lib = lib
    return _lib


def sip_version() -> int:
    return int(load().sip_version())


def sip_profile_kernel_events(stream_start: Optional[int], stream_stop: Optional[int],
                              finish_start: Optional[int] = None, finish_stop: Optional[int] = None,
                              rescue_start: Optional[int] = None, rescue_stop: Optional[int] = None) -> None:
    """Arm the one-shot profiling hook with raw hipEvent_t handles (all None disarms)."""
    load().sip_profile_kernel_events(stream_start, stream_stop, finish_start, finish_stop, rescue_start, rescue_stop)


def sip_status_string(status: int) -> str:
    return load().sip_status_string(int(status)).decode()


def sip_workspace_bytes(B: int, V: int, dtype: int, hist_nnz: int, k_logprobs: int) -> int:
    return int(load().sip_workspace_bytes(B, V, dtype, hist_nnz, k_logprobs))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def dtype_code(logits: torch.Tensor) -> int:
    if logits.dtype == torch.float32:
        return SIP_F32
    if logits.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return SIP_BF16
    raise TypeError(f"logits must be float32 or bfloat16 (or raw 16-bit patterns), got {logits.dtype}")


def make_params(params: Optional[Dict[str, Optional[torch.Tensor]]], B: int) -> SipParams:
    sp = SipParams()
    for name in PARAM_FIELDS:
        t = None if params is None else params.get(name)
        if t is not None:
            if t.dtype != _PARAM_DTYPES[name] or t.numel() != B or not t.is_contiguous() or not t.is_cuda:
                raise TypeError(f"params[{name!r}] must be a contiguous device tensor of {B} x {_PARAM_DTYPES[name]}")
        setattr(sp, name, _ptr(t))
    return sp


def sip_sample(logits: torch.Tensor, params: Optional[Dict[str, Optional[torch.Tensor]]],
               hist_indptr: Optional[torch.Tensor], hist_tokens: Optional[torch.Tensor],
               seed: int, step: int, k_logprobs: int, *,
               out_ids: Optional[torch.Tensor] = None, out_lp_ids: Optional[torch.Tensor] = None,
               out_lp: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
               V: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None
               ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
    """Enqueue one sampling call on ``stream`` (default: torch's current stream).

    ``logits`` is a 2-D device tensor whose rows are contiguous; ``V`` (default: its width)
    may be smaller than the row stride.  Outputs and workspace are allocated with torch when
    not supplied.  Returns (ids [B], logprob ids [B,1+k] or None, logprobs [B,1+k] or None)."""
    lib = load()
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise TypeError("logits must be a 2-D device tensor with contiguous rows")
    B = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    dt = dtype_code(logits)
    dev = logits.device
    nnz = 0
    if hist_indptr is not None and hist_tokens is not None:
        if hist_indptr.dtype != torch.int64 or hist_tokens.dtype != torch.int32:
            raise TypeError("hist_indptr must be int64 and hist_tokens int32")
        if hist_indptr.numel() != B + 1:
            raise TypeError("hist_indptr must have B + 1 entries")
        nnz = hist_tokens.numel()
    if out_ids is None:
        out_ids = torch.empty(B, dtype=torch.int32, device=dev)
    if k_logprobs >= 0:
        if out_lp_ids is None:
            out_lp_ids = torch.empty(B, 1 + k_logprobs, dtype=torch.int32, device=dev)
        if out_lp is None:
            out_lp = torch.empty(B, 1 + k_logprobs, dtype=torch.float32, device=dev)
    if workspace is None:
        need = sip_workspace_bytes(B, V, dt, nnz, k_logprobs)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    sp = make_params(params, B)
    s = torch.cuda.current_stream(dev) if stream is None else stream
    status = lib.sip_sample(_ptr(logits), B, V, logits.stride(0), dt, ctypes.byref(sp),
                            _ptr(hist_indptr) if nnz else None, _ptr(hist_tokens) if nnz else None, nnz,
                            seed, step, _ptr(out_ids), _ptr(out_lp_ids), _ptr(out_lp), k_logprobs,
                            _ptr(workspace), workspace.numel() * workspace.element_size(), s.cuda_stream)
    if status != SIP_OK:
        raise SipError(status)
    return out_ids, out_lp_ids, out_lp


def sip_init() -> None:
    """One-time set-up of the library on torch's current device (see include/sip.h)."""
    status = load().sip_init()
    if status != SIP_OK:
        raise SipError(status)


def sip_noalloc_scratch_bytes() -> int:
    return int(load().sip_noalloc_scratch_bytes())


def sip_sample_noalloc(logits: torch.Tensor, params: Optional[Dict[str, Optional[torch.Tensor]]],
                       hist_indptr: Optional[torch.Tensor], hist_tokens: Optional[torch.Tensor],
                       seed: int, step: int, k_logprobs: int, *, out_ids: torch.Tensor,
                       out_lp_ids: Optional[torch.Tensor] = None, out_lp: Optional[torch.Tensor] = None,
                       V: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """sip_sample_noalloc of include/sip.h: the caller supplies every output; nothing is allocated
    here either (no tensor is created)."""
    lib = load()
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise TypeError("logits must be a 2-D device tensor with contiguous rows")
    B = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    nnz = 0
    if hist_indptr is not None and hist_tokens is not None:
        if hist_indptr.dtype != torch.int64 or hist_tokens.dtype != torch.int32 or hist_indptr.numel() != B + 1:
            raise TypeError("hist_indptr must be int64 with B + 1 entries and hist_tokens int32")
        nnz = hist_tokens.numel()
    sp = make_params(params, B)
    status = lib.sip_sample_noalloc(_ptr(logits), B, V, logits.stride(0), dtype_code(logits), ctypes.byref(sp),
                                    _ptr(hist_indptr) if nnz else None, _ptr(hist_tokens) if nnz else None, nnz,
                                    seed, step, _ptr(out_ids), _ptr(out_lp_ids), _ptr(out_lp), k_logprobs,
                                    _stream_handle(logits.device, stream))
    if status != SIP_OK:
        raise SipError(status)


# ---- device-resident sampler state

def sip_state_bytes(slots: int, L_max: int) -> int:
    return int(load().sip_state_bytes(slots, L_max))


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def _stream_handle(dev, stream):
    return (torch.cuda.current_stream(dev) if stream is None else stream).cuda_stream


def sip_state_init(state: torch.Tensor, slots: int, L_max: int,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    """Enqueue the initialisation of ``state`` (a device byte buffer of sip_state_bytes())."""
    if not state.is_cuda:
        raise TypeError("state must be a device tensor")
    status = load().sip_state_init(_ptr(state), _nbytes(state), slots, L_max, _stream_handle(state.device, stream))
    if status != SIP_OK:
        raise SipError(status)


def sip_state_assign(state: torch.Tensor, slots: int, L_max: int, slot_ids: torch.Tensor,
                     indptr: Optional[torch.Tensor], tokens: Optional[torch.Tensor],
                     stream: Optional[torch.cuda.Stream] = None) -> None:
    """Enqueue: slot ``slot_ids[i]`` restarts with ``tokens[indptr[i]:indptr[i+1]]`` as its history."""
    if not state.is_cuda or not slot_ids.is_cuda or slot_ids.dtype != torch.int32:
        raise TypeError("state and slot_ids (int32) must be device tensors")
    n = slot_ids.numel()
    nnz = 0
    if indptr is not None and tokens is not None:
        if indptr.dtype != torch.int64 or tokens.dtype != torch.int32 or indptr.numel() != n + 1:
            raise TypeError("indptr must be int64 with n + 1 entries and tokens int32")
        nnz = tokens.numel()
    status = load().sip_state_assign(_ptr(state), _nbytes(state), slots, L_max, n, _ptr(slot_ids),
                                     _ptr(indptr) if nnz else None, _ptr(tokens) if nnz else None, nnz,
                                     _stream_handle(state.device, stream))
    if status != SIP_OK:
        raise SipError(status)


def sip_sample_state(logits: torch.Tensor, params: Optional[Dict[str, Optional[torch.Tensor]]],
                     state: torch.Tensor, slots: int, L_max: int, slot_of_row: torch.Tensor,
                     seed: int, step: int, k_logprobs: int, *,
                     out_ids: Optional[torch.Tensor] = None, out_lp_ids: Optional[torch.Tensor] = None,
                     out_lp: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     V: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None
                     ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
    """sip_sample with the histories read from, and the sampled ids appended to, ``state``."""
    lib = load()
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise TypeError("logits must be a 2-D device tensor with contiguous rows")
    B = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    dt = dtype_code(logits)
    dev = logits.device
    if not slot_of_row.is_cuda or slot_of_row.dtype != torch.int32 or slot_of_row.numel() != B:
        raise TypeError("slot_of_row must be a device tensor of B x int32")
    if out_ids is None:
        out_ids = torch.empty(B, dtype=torch.int32, device=dev)
    if k_logprobs >= 0:
        if out_lp_ids is None:
            out_lp_ids = torch.empty(B, 1 + k_logprobs, dtype=torch.int32, device=dev)
        if out_lp is None:
            out_lp = torch.empty(B, 1 + k_logprobs, dtype=torch.float32, device=dev)
    if workspace is None:
        need = sip_workspace_bytes(B, V, dt, B * L_max, k_logprobs)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    sp = make_params(params, B)
    status = lib.sip_sample_state(_ptr(logits), B, V, logits.stride(0), dt, ctypes.byref(sp), _ptr(state),
                                  _nbytes(state), slots, L_max, _ptr(slot_of_row), seed, step, _ptr(out_ids),
                                  _ptr(out_lp_ids), _ptr(out_lp), k_logprobs, _ptr(workspace), _nbytes(workspace),
                                  _stream_handle(dev, stream))
    if status != SIP_OK:
        raise SipError(status)
    return out_ids, out_lp_ids, out_lp


STATE_TABLE_SLOTS = 4096     # slots of a state's per-sequence table of multiplicities


def state_views(state: torch.Tensor, slots: int, L_max: int):
    """(tick, overflow, len [slots], tokens [slots, L_max]) as views of a state buffer, per the
    layout that include/sip.h documents."""
    len_bytes = (4 * slots + 255) // 256 * 256
    tick = state[0:8].view(torch.int64)
    overflow = state[8:12].view(torch.int32)
    length = state[256:256 + 4 * slots].view(torch.int32)
    base = 256 + 2 * len_bytes
    tokens = state[base:base + 4 * slots * L_max].view(torch.int32).view(slots, L_max)
    return tick, overflow, length, tokens


def state_table_views(state: torch.Tensor, slots: int, L_max: int):
    """(distinct [slots], keys [slots, 4096], multiplicities [slots, 4096]) of a state buffer:
    each slot's table token -> occurrences (key -1 = free slot; distinct -1 = table given up)."""
    len_bytes = (4 * slots + 255) // 256 * 256
    distinct = state[256 + len_bytes:256 + len_bytes + 4 * slots].view(torch.int32)
    base = 256 + 2 * len_bytes + (4 * slots * L_max + 255) // 256 * 256
    tab = state[base:base + slots * 2 * STATE_TABLE_SLOTS * 4].view(torch.int32).view(slots, 2, STATE_TABLE_SLOTS)
    return distinct, tab[:, 0], tab[:, 1]


# ---- vocabulary-sharded logits

def sip_workspace_bytes_sharded(B: int, V_shard: int, t: int, dtype: int, hist_nnz: int, k_logprobs: int) -> int:
    return int(load().sip_workspace_bytes_sharded(B, V_shard, t, dtype, hist_nnz, k_logprobs))


class ShardTable:
    """The host array of piece pointers that sip_sample_sharded takes, checked and built once for
    pieces that are used call after call.  Keeps the tensors alive."""

    def __init__(self, shards, V_shard: Optional[int] = None):
        first = shards[0]
        for x in shards:
            if (not x.is_cuda or x.dim() != 2 or x.stride(1) != 1 or x.dtype != first.dtype
                    or x.shape[0] != first.shape[0] or x.stride(0) != first.stride(0)):
                raise TypeError("shards must be 2-D device tensors with contiguous rows, one dtype, one shape")
        self.tensors = list(shards)
        self.t = len(shards)
        self.B = first.shape[0]
        self.V_shard = first.shape[1] if V_shard is None else int(V_shard)
        self.stride = first.stride(0)
        self.dtype = dtype_code(first)
        self.device = first.device
        self.table = (ctypes.c_void_p * self.t)(*[x.data_ptr() for x in shards])


def sip_sample_sharded(shards, params: Optional[Dict[str, Optional[torch.Tensor]]],
                       hist_indptr: Optional[torch.Tensor], hist_tokens: Optional[torch.Tensor],
                       seed: int, step: int, k_logprobs: int, *,
                       out_ids: Optional[torch.Tensor] = None, out_lp_ids: Optional[torch.Tensor] = None,
                       out_lp: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                       V_shard: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None
                       ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
    """sip_sample on logits that come as ``t`` vocabulary pieces: ``shards`` is a sequence of 2-D
    device tensors [B, >= V_shard] of one dtype and one row stride, or a ShardTable made of them."""
    lib = load()
    st = shards if isinstance(shards, ShardTable) else ShardTable(shards, V_shard)
    t, B, V_shard, dt, dev = st.t, st.B, st.V_shard, st.dtype, st.device
    nnz = 0
    if hist_indptr is not None and hist_tokens is not None:
        if hist_indptr.dtype != torch.int64 or hist_tokens.dtype != torch.int32 or hist_indptr.numel() != B + 1:
            raise TypeError("hist_indptr must be int64 with B + 1 entries and hist_tokens int32")
        nnz = hist_tokens.numel()
    if out_ids is None:
        out_ids = torch.empty(B, dtype=torch.int32, device=dev)
    if k_logprobs >= 0:
        if out_lp_ids is None:
            out_lp_ids = torch.empty(B, 1 + k_logprobs, dtype=torch.int32, device=dev)
        if out_lp is None:
            out_lp = torch.empty(B, 1 + k_logprobs, dtype=torch.float32, device=dev)
    if workspace is None:
        need = sip_workspace_bytes_sharded(B, V_shard, t, dt, nnz, k_logprobs)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    sp = make_params(params, B)
    status = lib.sip_sample_sharded(st.table, t, B, V_shard, st.stride, dt, ctypes.byref(sp),
                                    _ptr(hist_indptr) if nnz else None, _ptr(hist_tokens) if nnz else None, nnz,
                                    seed, step, _ptr(out_ids), _ptr(out_lp_ids), _ptr(out_lp), k_logprobs,
                                    _ptr(workspace), _nbytes(workspace), _stream_handle(dev, stream))
    if status != SIP_OK:
        raise SipError(status)
    return out_ids, out_lp_ids, out_lp


# ---- hand-off of the ids to the host

def sip_publish_ids(ids: torch.Tensor, host_ids: torch.Tensor, host_flag: torch.Tensor, ticket: int,
                    stream: Optional[torch.cuda.Stream] = None) -> None:
    """Enqueue the copy of ``ids`` (device int32 [B]) into ``host_ids`` (pinned int32 [>= B]) followed
    by the store of ``ticket`` into ``host_flag`` (pinned, one 64-bit word)."""
    if not ids.is_cuda or ids.dtype != torch.int32:
        raise TypeError("ids must be a device int32 tensor")
    if (host_ids.is_cuda or not host_ids.is_pinned() or host_ids.dtype != torch.int32 or host_ids.numel() < ids.numel()
            or host_flag.is_cuda or not host_flag.is_pinned() or host_flag.element_size() != 8):
        raise TypeError("host_ids (int32) and host_flag (one 64-bit word) must be pinned host tensors")
    status = load().sip_publish_ids(_ptr(ids), ids.numel(), _ptr(host_ids), _ptr(host_flag), ticket,
                                    _stream_handle(ids.device, stream))
    if status != SIP_OK:
        raise SipError(status)


def sip_wait_ids(host_flag: torch.Tensor, ticket: int, timeout_ns: int = 2 ** 64 - 1) -> bool:
    """Spin on the host until the flag reaches ``ticket``; False on time-out.  No HIP call."""
    status = load().sip_wait_ids(_ptr(host_flag), ticket, timeout_ns)
    if status == SIP_OK:
        return True
    if status == SIP_ERR_TIMEOUT:
        return False
    raise SipError(status)


def sip_probe_read(src: torch.Tensor, workgroups: int, workspace: torch.Tensor, start_event: Optional[int] = None,
                   stop_event: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Enqueue the bare streaming read of ``src`` (see include/sip.h)."""
    if not src.is_cuda or not src.is_contiguous() or not workspace.is_cuda:
        raise TypeError("src must be a contiguous device tensor and workspace a device tensor")
    status = load().sip_probe_read(_ptr(src), _nbytes(src), workgroups, _ptr(workspace), _nbytes(workspace),
                                   start_event, stop_event, _stream_handle(src.device, stream))
    if status != SIP_OK:
        raise SipError(status)


# ---- everything in one call

def sip_sample_call(*, logits: Optional[torch.Tensor] = None, shards=None, V: Optional[int] = None,
                    params: Optional[Dict[str, Optional[torch.Tensor]]] = None,
                    hist_indptr: Optional[torch.Tensor] = None, hist_tokens: Optional[torch.Tensor] = None,
                    state: Optional[torch.Tensor] = None, slots: int = 0, L_max: int = 0,
                    slot_of_row: Optional[torch.Tensor] = None, seed: int = 0, step: int = 0, k_logprobs: int = 0,
                    out_ids: Optional[torch.Tensor] = None, out_lp_ids: Optional[torch.Tensor] = None,
                    out_lp: Optional[torch.Tensor] = None, host_ids: Optional[torch.Tensor] = None,
                    host_flag: Optional[torch.Tensor] = None, ticket: int = 0,
                    prompt_indptr: Optional[torch.Tensor] = None, prompt_tokens: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None
                    ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
    """sip_sample_call of include/sip.h: logits as one matrix (``logits``, ``V``) or as pieces
    (``shards``: a ShardTable or a sequence of tensors), histories as a CSR or in a ``state``,
    and the hand-off to ``host_ids`` / ``host_flag`` behind it if both are given."""
    lib = load()
    c = SipCall()
    keep = []
    if shards is not None:
        st = shards if isinstance(shards, ShardTable) else ShardTable(shards, V)
        keep.append(st)
        c.shard_logits = ctypes.cast(st.table, ctypes.POINTER(ctypes.c_void_p))
        c.t_shards, c.V_shard, c.shard_stride = st.t, st.V_shard, st.stride
        B, dt, dev = st.B, st.dtype, st.device
    else:
        if logits is None or not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
            raise TypeError("logits must be a 2-D device tensor with contiguous rows")
        B, dt, dev = logits.shape[0], dtype_code(logits), logits.device
        c.logits, c.row_stride, c.V = _ptr(logits), logits.stride(0), logits.shape[1] if V is None else int(V)
    c.B, c.dtype = B, dt
    sp = make_params(params, B)
    c.params = ctypes.pointer(sp)
    if state is not None:
        c.state, c.state_bytes, c.slots, c.L_max, c.slot_of_row = _ptr(state), _nbytes(state), slots, L_max, _ptr(slot_of_row)
    elif hist_indptr is not None and hist_tokens is not None and hist_tokens.numel():
        if hist_indptr.dtype != torch.int64 or hist_tokens.dtype != torch.int32 or hist_indptr.numel() != B + 1:
            raise TypeError("hist_indptr must be int64 with B + 1 entries and hist_tokens int32")
        c.hist_indptr, c.hist_tokens, c.hist_nnz = _ptr(hist_indptr), _ptr(hist_tokens), hist_tokens.numel()
    if prompt_indptr is not None and prompt_tokens is not None and prompt_tokens.numel():
        if prompt_indptr.dtype != torch.int64 or prompt_tokens.dtype != torch.int32 or prompt_indptr.numel() != B + 1:
            raise TypeError("prompt_indptr must be int64 with B + 1 entries and prompt_tokens int32")
        c.prompt_indptr, c.prompt_tokens, c.prompt_nnz = _ptr(prompt_indptr), _ptr(prompt_tokens), prompt_tokens.numel()
    c.seed, c.step, c.k_logprobs = seed, step, k_logprobs
    if out_ids is None:
        out_ids = torch.empty(B, dtype=torch.int32, device=dev)
    if k_logprobs >= 0:
        if out_lp_ids is None:
            out_lp_ids = torch.empty(B, 1 + k_logprobs, dtype=torch.int32, device=dev)
        if out_lp is None:
            out_lp = torch.empty(B, 1 + k_logprobs, dtype=torch.float32, device=dev)
    c.out_ids, c.out_lp_ids, c.out_lp = _ptr(out_ids), _ptr(out_lp_ids), _ptr(out_lp)
    if host_ids is not None or host_flag is not None:
        if host_ids is None or host_flag is None or not host_ids.is_pinned() or not host_flag.is_pinned():
            raise TypeError("host_ids and host_flag must both be given, as pinned host tensors")
        c.host_ids, c.host_flag, c.ticket = _ptr(host_ids), _ptr(host_flag), ticket
    if workspace is None:
        need = int(lib.sip_call_workspace_bytes(ctypes.byref(c)))
        if need == 0:
            raise SipError(SIP_ERR_INVALID_ARG)
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    c.workspace, c.workspace_bytes = _ptr(workspace), _nbytes(workspace)
    c.hip_stream = _stream_handle(dev, stream)
    status = lib.sip_sample_call(ctypes.byref(c))
    if status != SIP_OK:
        raise SipError(status)
    return out_ids, out_lp_ids, out_lp
