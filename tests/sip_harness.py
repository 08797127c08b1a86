"""Shared plumbing of the GPU parity tests: move a workload to the device, run the library
through its C boundary, run the oracle on the same inputs and compare.

Comparison rules (stated once here, used by every parity test):
  * greedy rows: token ids bit-exact;
  * stochastic rows: ids exact unless the oracle flags the row as near-boundary (its
    uniform within 1e-6 of a CDF edge, or the top-p cut within 1e-6 relative mass of a group
    edge that survives min-p); a flagged row may instead return one of the oracle's
    alternatives for it (the draw under the neighbouring decision: cut one value group earlier
    or later, CDF entry before or after) and nothing else; flagged rows and those among them
    that returned an alternative are counted and reported;
  * best-n token ids exact, in order;
  * logprobs: |gpu - oracle| <= 1e-5 + 2^-22 * |oracle|  (the relative term is one fp32
    half-ulp of the value: s_v - s_max itself is an fp32 number on both sides).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np
import torch

import paper_2506_22033_amd as sip
from oracle import sip_oracle as O

last_row_path = None        # per-row code path of the most recent run_gpu() call (see include/sip.h)
last_row_why = None         # per-row code of the finishing kernel (1, or why the row went to the rescue kernel)
LP_ABS = 1e-5
LP_REL = 2.0 ** -22
DEV = "cuda:0"


def have_gpu() -> bool:
    return torch.cuda.is_available()


@dataclass
class DeviceWorkload:
    logits: torch.Tensor
    V: int
    params: Dict[str, Optional[torch.Tensor]]
    indptr: Optional[torch.Tensor]
    tokens: Optional[torch.Tensor]
    k_logprobs: int


def logits_to_device(logits: np.ndarray, pad_to: int = 8) -> torch.Tensor:
    """Upload [B, V] logits into a buffer whose row stride is a multiple of ``pad_to``
    elements (16-byte rows); returns the [B, stride] tensor (caller passes V)."""
    B, V = logits.shape
    stride = (V + pad_to - 1) // pad_to * pad_to
    if logits.dtype == np.uint16:
        host = torch.from_numpy(logits.view(np.int16)).view(torch.bfloat16)
        buf = torch.full((B, stride), float("nan"), dtype=torch.bfloat16, device=DEV)
    else:
        host = torch.from_numpy(logits)
        buf = torch.full((B, stride), float("nan"), dtype=torch.float32, device=DEV)
    buf[:, :V] = host.to(DEV)
    return buf


def to_device(w, pad_to: int = 8) -> DeviceWorkload:
    params = {}
    for k, v in w.params.items():
        params[k] = None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(DEV)
    indptr = tokens = None
    if w.hist_indptr is not None:
        indptr = torch.from_numpy(w.hist_indptr).to(DEV)
        tokens = torch.from_numpy(w.hist_tokens).to(DEV)
    return DeviceWorkload(logits_to_device(w.logits, pad_to), w.V, params, indptr, tokens, w.k_logprobs)


def run_gpu(d: DeviceWorkload, seed: int, step: int, k_logprobs: Optional[int] = None, row_ids=None):
    params = dict(d.params)
    if row_ids is not None:
        params["row_id"] = row_ids
    k = d.k_logprobs if k_logprobs is None else k_logprobs
    B = d.logits.shape[0]
    nnz = 0 if d.tokens is None else d.tokens.numel()
    need = sip.sip_workspace_bytes(B, d.V, sip.binding.dtype_code(d.logits), nnz, k)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
    ids, lp_ids, lp = sip.sip_sample(d.logits, params, d.indptr, d.tokens, seed, step, k, V=d.V, workspace=ws)
    torch.cuda.synchronize()
    global last_row_path, last_row_why
    last_row_path = ws[:4 * B].view(torch.int32).cpu().numpy().copy()
    last_row_why = ws[4 * B:8 * B].view(torch.int32).cpu().numpy().copy()
    return (ids.cpu().numpy(), None if lp_ids is None else lp_ids.cpu().numpy(),
            None if lp is None else lp.cpu().numpy())


@dataclass
class ParityStats:
    rows: int = 0
    greedy_rows: int = 0
    flagged: int = 0
    flagged_mismatch: int = 0
    max_lp_err: float = 0.0
    lp_needed_rel: int = 0

    def merge(self, o: "ParityStats"):
        self.rows += o.rows; self.greedy_rows += o.greedy_rows; self.flagged += o.flagged
        self.flagged_mismatch += o.flagged_mismatch
        self.max_lp_err = max(self.max_lp_err, o.max_lp_err); self.lp_needed_rel += o.lp_needed_rel


def check_lp(got: np.ndarray, want: np.ndarray, st: ParityStats, ctx: str):
    got = got.astype(np.float64)
    err = np.abs(got - want)
    finite = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), finite), ctx
    if finite.any():
        e = err[finite]
        st.max_lp_err = max(st.max_lp_err, float(e.max()))
        st.lp_needed_rel += int((e > LP_ABS).sum())
        bound = LP_ABS + LP_REL * np.abs(want[finite])
        assert (e <= bound).all(), f"{ctx}: logprob error {e.max():.3e} (bound {bound[e.argmax()]:.3e})"


ORACLE_THREADS = 16         # the GPU machine's share of host cores


def oracle_rows(w, seed: int, step: int, k: int, rows: Sequence[int], row_ids: Optional[np.ndarray] = None):
    """The oracle's RowResults for ``rows``; large jobs are spread over host threads (numpy's
    sort / exp / cumsum release the GIL)."""
    rows = list(rows)
    def one(b):
        return O.sample_batch(w.logits, w.params, w.hist_indptr, w.hist_tokens, seed, step, max(k, 0),
                              row_ids=row_ids, rows=[b])[0]
    if len(rows) * w.V < 4_000_000:
        return [one(b) for b in rows]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(ORACLE_THREADS) as ex:
        return list(ex.map(one, rows))


def compare(w, gpu_out, seed: int, step: int, rows: Optional[Sequence[int]] = None,
            k_logprobs: Optional[int] = None, row_ids: Optional[np.ndarray] = None) -> ParityStats:
    k = w.k_logprobs if k_logprobs is None else k_logprobs
    rows = list(range(w.B)) if rows is None else list(rows)
    ref = oracle_rows(w, seed, step, k, rows, row_ids)
    return check_rows(f"{w.name} step {step}", rows, ref, gpu_out, k)


def check_rows(name: str, rows: Sequence[int], ref, gpu_out, k: int) -> ParityStats:
    """Apply the comparison rules to the oracle's RowResults ``ref`` of the rows ``rows``."""
    ids, lp_ids, lp = gpu_out
    st = ParityStats()
    for b, r in zip(rows, ref):
        ctx = f"{name} row {b}"
        st.rows += 1
        if r.greedy:
            st.greedy_rows += 1
            assert ids[b] == r.token, f"{ctx}: greedy id {ids[b]} != {r.token}"
        elif r.flagged():
            st.flagged += 1
            st.flagged_mismatch += int(ids[b] != r.token)
            assert ids[b] == r.token or int(ids[b]) in r.alt_tokens, (
                f"{ctx}: near-boundary row returned {ids[b]}, neither the oracle's {r.token} nor one of its "
                f"alternatives {r.alt_tokens} (draw margin {r.draw_margin:.3e}, top-p margin {r.topp_margin:.3e})")
        else:
            assert ids[b] == r.token, (f"{ctx}: id {ids[b]} != {r.token} (u={r.u!r}, draw margin "
                                       f"{r.draw_margin:.3e}, top-p margin {r.topp_margin:.3e})")
        if k >= 0:
            assert lp_ids[b, 0] == ids[b], ctx
            if ids[b] == r.token:
                check_lp(lp[b, :1], np.array([r.logprob]), st, ctx + " sampled logprob")
            n = len(r.top_ids)
            assert np.array_equal(lp_ids[b, 1:1 + n], r.top_ids), f"{ctx}: best-{k} ids differ"
            check_lp(lp[b, 1:1 + n], r.top_logprobs, st, ctx + " best-n logprobs")
            if n < k:
                assert (lp_ids[b, 1 + n:] == -1).all() and np.isneginf(lp[b, 1 + n:]).all(), ctx
    return st


def custom(name, logits: np.ndarray, params: Optional[dict] = None, histories=None, k_logprobs: int = 0):
    """A hand-made workload: ``histories`` is a list of per-row token lists (or None)."""
    import workloads
    B, V = logits.shape
    full = {k: None for k in ("temperature", "top_k", "top_p", "min_p", "repetition_penalty",
                              "frequency_penalty", "presence_penalty")}
    for k, v in (params or {}).items():
        dt = np.int32 if k == "top_k" else np.float32
        full[k] = np.broadcast_to(np.asarray(v, dtype=dt), (B,)).copy()
    indptr = tokens = None
    if histories is not None:
        indptr = np.concatenate(([0], np.cumsum([len(h) for h in histories]))).astype(np.int64)
        tokens = (np.concatenate([np.asarray(h, dtype=np.int32) for h in histories]).astype(np.int32)
                  if indptr[-1] > 0 else np.zeros(0, np.int32))
    dtype = "bf16" if logits.dtype == np.uint16 else "f32"
    return workloads.Workload(name, B, V, dtype, logits, full, indptr, tokens, k_logprobs)
