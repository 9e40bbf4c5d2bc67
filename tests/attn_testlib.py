"""Shared helpers for the GPU parity tests: upload a Workload, run the HIP path, compare."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W

# Tolerances.  bf16 inputs: the bound the benchmark contract states.  fp32: true fp32 FMA with
# exact inputs; the error is a few ulp of the largest partial sums.
# fp16: weights and outputs carry 11 significant bits instead of 8, so the rounding errors that make
# up the bf16 figure shrink eightfold; a fifth of the bf16 bound leaves the same margin.
TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-4, 1e-5), "f16": (4e-3, 1e-3)}


def to_device(arr: np.ndarray) -> torch.Tensor:
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(arr).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


class DeviceWorkload:
    def __init__(self, wl: W.Workload):
        self.wl = wl
        self.q, self.k, self.v = to_device(wl.q), to_device(wl.k), to_device(wl.v)
        self.out = torch.full_like(self.q, float("nan"))
        self.qsl = torch.from_numpy(wl.query_start_loc.astype(np.int32)).cuda()
        self.seq_lens = torch.from_numpy(wl.seq_lens.astype(np.int32)).cuda()
        self.kvsl = None if wl.kv_start_loc is None else torch.from_numpy(wl.kv_start_loc.astype(np.int32)).cuda()
        self.bt = None if wl.block_table is None else torch.from_numpy(wl.block_table.astype(np.int32)).cuda()
        self.max_q = int(wl.q_lens().max()) if wl.num_seqs else 0
        self.max_kv = int(wl.seq_lens.max()) if wl.num_seqs else 0
        self.ws = None

    def args(self, is_decode: bool) -> A.AttnArgs:
        a = A.make_args(self.q, self.k, self.v, self.out, self.seq_lens, self.wl.scale, max_q_len=1 if is_decode else self.max_q,
                        max_kv_len=self.max_kv, query_start_loc=None if is_decode else self.qsl, kv_start_loc=self.kvsl,
                        block_table=self.bt, causal=self.wl.causal, is_decode=is_decode)
        if is_decode:
            need = A.attn_workspace_bytes(a, True)
            if self.ws is None or self.ws.numel() * 4 < need:
                self.ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device="cuda")
            a.workspace = self.ws.data_ptr()
            a.workspace_bytes = self.ws.numel() * 4
        return a

    def run(self, is_decode=None, poison_out=True) -> torch.Tensor:
        if is_decode is None:
            is_decode = self.wl.kind == "decode"
        if poison_out:
            self.out.fill_(float("nan"))
        a = self.args(is_decode)
        if is_decode:
            A.attn_decode_paged(None, None, None, None, None, None, None, max_kv_len=0, args=a)
        else:
            A.attn_prefill_varlen(None, None, None, None, None, None, None, max_q_len=0, max_kv_len=0, args=a)
        torch.cuda.synchronize()
        return self.out


def oracle_problem(wl: W.Workload) -> oracle.OracleProblem:
    if wl.dtype == "f16":  # widened exactly; the oracle has no fp16 reader of its own
        return oracle.OracleProblem(wl.q.astype(np.float32), wl.k.astype(np.float32), wl.v.astype(np.float32), wl.query_start_loc,
                                    wl.seq_lens, wl.scale, wl.causal, block_table=wl.block_table, kv_start_loc=wl.kv_start_loc)
    return oracle.OracleProblem(wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, wl.causal,
                                block_table=wl.block_table, kv_start_loc=wl.kv_start_loc)


def errors(got: np.ndarray, ref: np.ndarray):
    """max-abs error and relative RMS error sqrt(sum (got-ref)^2 / sum ref^2)."""
    d = got - ref
    max_abs = float(np.max(np.abs(d))) if d.size else 0.0
    den = float(np.sum(ref * ref))
    rel_rms = float(np.sqrt(np.sum(d * d) / den)) if den > 0 else float(np.sqrt(np.sum(d * d)))
    return max_abs, rel_rms


def assert_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "%s: non-finite output" % what
    max_abs, rel_rms = errors(got, ref)
    tol_abs, tol_rms = TOL[dtype]
    assert max_abs <= tol_abs and rel_rms <= tol_rms, "%s: max-abs %.3e (<= %.1e), rel-RMS %.3e (<= %.1e)" % (
        what, max_abs, tol_abs, rel_rms, tol_rms)
    return max_abs, rel_rms


def check_full(wl: W.Workload, is_decode=None, what=""):
    dw = DeviceWorkload(wl)
    got = to_host_f64(dw.run(is_decode))
    ref = oracle.attention(oracle_problem(wl))
    # per-sequence relative RMS as well as the whole output
    qsl = wl.query_start_loc
    for s in range(wl.num_seqs):
        if qsl[s + 1] > qsl[s]:
            assert_close(got[qsl[s]:qsl[s + 1]], ref[qsl[s]:qsl[s + 1]], wl.dtype, "%s seq %d" % (what or wl.name, s))
    return assert_close(got, ref, wl.dtype, what or wl.name)


def sample_rows(wl: W.Workload, n: int, seed: int = 0):
    """Up to n distinct random (sequence, token, head) triples (drawn without replacement), always
    including each sequence's first and last token."""
    rng = np.random.default_rng(seed)
    nq = wl.q_lens()
    H = wl.num_q_heads
    qsl = wl.query_start_loc.astype(np.int64)
    total = int(qsl[-1]) * H
    picked = []
    for s in range(wl.num_seqs):
        if nq[s] == 0:
            continue
        for t in {0, int(nq[s]) - 1}:
            picked.append((int(qsl[s]) + t) * H + int(rng.integers(H)))
    rest = rng.permutation(total)[: max(0, min(n, total) - len(picked))]
    flat = np.unique(np.concatenate([np.asarray(picked, np.int64), rest.astype(np.int64)]))
    row, heads = flat // H, flat % H
    seqs = np.searchsorted(qsl, row, side="right") - 1
    return seqs.astype(np.int32), (row - qsl[seqs]).astype(np.int32), heads.astype(np.int32)


def check_sampled(wl: W.Workload, n_rows: int, is_decode=None, what="", seed=0, dw=None):
    dw = dw or DeviceWorkload(wl)
    out = dw.run(is_decode)
    seqs, toks, heads = sample_rows(wl, n_rows, seed)
    ref = oracle.attention_rows(oracle_problem(wl), seqs, toks, heads)
    rows = torch.from_numpy(wl.query_start_loc[seqs].astype(np.int64) + toks).cuda()
    got = to_host_f64(out[rows, torch.from_numpy(heads.astype(np.int64)).cuda()])
    # nothing outside the sample may be left unwritten
    assert bool(torch.isfinite(out.float()).all()), "%s: unwritten or non-finite output rows" % (what or wl.name)
    return assert_close(got, ref, wl.dtype, what or wl.name)
