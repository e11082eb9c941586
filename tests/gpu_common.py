"""Set-up shared by the GPU parity tests: draw a workload, build the oracle's index,
hand the identical stored index to the HIP library, keep both sides' handles."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

import lc_workloads as wl
from oracle import lychee_oracle as orc


def oracle_index_to_levels(idx: orc.Index) -> List[Dict]:
    out = []
    for l in range(idx.L):
        out.append(dict(center=idx.center[l].astype(np.float32),
                        radius=idx.radius[l].astype(np.float32),
                        parent=idx.parent[l].astype(np.int32),
                        ntok=idx.ntok[l].astype(np.int32),
                        nchunk=idx.nchunk[l].astype(np.int32)))
    return out


def levels_to_oracle_index(levels: List[Dict], bounds: np.ndarray, T: int, F: int, geometry: int) -> orc.Index:
    L = len(levels)
    return orc.Index(d=levels[0]["center"].shape[1], L=L, F=F, geometry=geometry,
                     bounds=np.asarray(bounds, dtype=np.int64).copy(), T=int(T),
                     center=[lv["center"].astype(np.float64) for lv in levels],
                     radius=[lv["radius"].astype(np.float64) for lv in levels],
                     parent=[lv["parent"].astype(np.int64) for lv in levels],
                     ntok=[lv["ntok"].astype(np.int64) for lv in levels],
                     nchunk=[lv["nchunk"].astype(np.int64) for lv in levels])


def to_bf16_tensor(bits: np.ndarray, device="cuda"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


@dataclass
class Case:
    w: wl.Workload
    seqs: List[wl.SeqInputs]
    oidx: List[List[orc.Index]]            # [b][h]
    cfg: object
    idx: object                            # binding.Index
    K: object                              # torch bf16 [B][H_kv][Tcap][d]
    V: object
    ws: object
    index_buf: object
    cap: int
    Tcap: int

    def Kf(self, b: int, h: int) -> np.ndarray:
        return wl.bf16_bits_to_f64(self.seqs[b].K[h])

    def Vf(self, b: int, h: int) -> np.ndarray:
        return wl.bf16_bits_to_f64(self.seqs[b].V[h])


def make_case(w: wl.Workload, tails: Optional[Sequence[int]] = None, extra_tokens: int = 0,
              extra_chunks: int = 0, geometry: int = orc.TOKEN_BALL, build_on: str = "oracle",
              offset_std: float = 0.5, noise_std: float = 1.0, cap: Optional[int] = None,
              decode_splits: int = 0, prune: int = 1, mutate=None, center_dtype: int = 0,
              fanouts: Optional[Sequence[int]] = None) -> Case:
    """build_on = "oracle": the oracle builds the index and the GPU imports it (identical
    stored values on both sides); "gpu": lc_build_index builds it (the oracle index is still
    built for comparison).  `mutate(seqs)` may edit the drawn sequences in place before anything
    is built from them."""
    import torch
    from paper_2603_08453_amd import binding as lc

    lens = wl.seq_lengths(w)
    seqs = []
    for b in range(w.B):
        s = wl.make_sequence(w, b, lens[b], offset_std=offset_std, noise_std=noise_std)
        if tails is not None and tails[b] > 0:
            # turn the last chunks into an open tail of about `tails[b]` tokens
            keep = np.searchsorted(s.bounds, s.T - tails[b], side="right")
            keep = max(1, min(keep, len(s.bounds) - 1))
            s.bounds = s.bounds[: keep + 1].copy()
        seqs.append(s)
    if mutate is not None:
        mutate(seqs)
    Tmax = max(s.T for s in seqs)
    Mmax = max(len(s.bounds) - 1 for s in seqs)
    Tcap = Tmax + extra_tokens
    cfg = lc.lc_config_default(levels=w.levels, fanout=w.fanout, geometry=geometry,
                               max_chunks=Mmax + extra_chunks, max_tokens=Tcap, decode_splits=decode_splits,
                               prune=prune, center_dtype=center_dtype,
                               **({} if fanouts is None else {"fanouts": list(fanouts)}))      # default 1 = always walk the levels, so the pruning path is what is tested
    F_or = w.fanout if fanouts is None else [f if f > 0 else w.fanout for f in fanouts]
    oidx = [[orc.build_index(wl.bf16_bits_to_f64(s.K[h]), s.bounds, s.T, w.levels, F_or, geometry=geometry,
                             center_dtype=center_dtype)
             for h in range(w.H_kv)] for s in seqs]

    Kt = torch.zeros((w.B, w.H_kv, Tcap, w.d), dtype=torch.bfloat16, device="cuda")
    Vt = torch.zeros_like(Kt)
    for b, s in enumerate(seqs):
        Kt[b, :, : s.T] = to_bf16_tensor(s.K)
        Vt[b, :, : s.T] = to_bf16_tensor(s.V)
    index_buf = torch.zeros(lc.lc_index_bytes(cfg, w.B, w.H_kv), dtype=torch.uint8, device="cuda")
    ws = torch.zeros(lc.lc_workspace_bytes(cfg, w.B, w.H_q, w.H_kv), dtype=torch.uint8, device="cuda")
    if build_on == "oracle":
        blob = lc.pack_blob(w.B, w.H_kv, w.d, w.levels, w.fanout, geometry,
                            [dict(T=s.T, bounds=s.bounds, heads=[oracle_index_to_levels(oidx[b][h])
                                                                 for h in range(w.H_kv)])
                             for b, s in enumerate(seqs)], center_dtype=center_dtype, fanouts=fanouts)
        idx = lc.lc_index_import(cfg, blob, index_buf)
    else:
        idx = lc.lc_build_index(cfg, Kt, [s.T for s in seqs], [s.bounds for s in seqs], index_buf, ws)
    torch.cuda.synchronize()
    if cap is None:
        cap = max(1, Mmax + extra_chunks)
    return Case(w, seqs, oidx, cfg, idx, Kt, Vt, ws, index_buf, cap, Tcap)


def gpu_retrieve(case: Case, q_bits: np.ndarray, budget: int, want_scores: bool = True):
    """q_bits uint16 [B][H_q][d].  Returns (ids list [b][h] -> np.ndarray, scores or None)."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = case.w
    q = to_bf16_tensor(q_bits)
    ids = torch.full((w.B, w.H_kv, case.cap), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((w.B, w.H_kv), -1, dtype=torch.int32, device="cuda")
    scores = None
    if want_scores:
        scores = torch.full((w.B, w.H_kv, case.cfg.max_chunks), float("nan"), dtype=torch.float32, device="cuda")
    lc.lc_retrieve(case.idx, q, budget, ids, counts, case.ws, scores=scores)
    torch.cuda.synchronize()
    ids_h, counts_h = ids.cpu().numpy(), counts.cpu().numpy()
    out = [[ids_h[b, h, : counts_h[b, h]].copy() for h in range(w.H_kv)] for b in range(w.B)]
    return out, (scores.cpu().numpy() if scores is not None else None), (ids, counts, q)


def gpu_decode(case: Case, q_bits: np.ndarray, ids_per_bh):
    """ids_per_bh[b][h] = ascending chunk ids.  Returns (out [B][H_q][d], lse [B][H_q])."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = case.w
    q = to_bf16_tensor(q_bits)
    ids = torch.zeros((w.B, w.H_kv, case.cap), dtype=torch.int32, device="cuda")
    counts = torch.zeros((w.B, w.H_kv), dtype=torch.int32, device="cuda")
    ids_h = np.zeros((w.B, w.H_kv, case.cap), dtype=np.int32)
    counts_h = np.zeros((w.B, w.H_kv), dtype=np.int32)
    for b in range(w.B):
        for h in range(w.H_kv):
            a = np.asarray(ids_per_bh[b][h], dtype=np.int32)
            ids_h[b, h, : len(a)] = a
            counts_h[b, h] = len(a)
    ids.copy_(torch.from_numpy(ids_h))
    counts.copy_(torch.from_numpy(counts_h))
    out = torch.full((w.B, w.H_q, w.d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.B, w.H_q), float("nan"), dtype=torch.float32, device="cuda")
    lc.lc_sparse_decode(case.idx, q, case.K, case.V, ids, counts, out, case.ws, lse=lse)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def gpu_step(case: Case, q_bits: np.ndarray, budget: int, with_ids: bool = True):
    """The fused entry point.  Returns (ids_per_bh or None, out, lse)."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = case.w
    q = to_bf16_tensor(q_bits)
    ids = counts = None
    if with_ids:
        ids = torch.full((w.B, w.H_kv, case.cap), -1, dtype=torch.int32, device="cuda")
        counts = torch.full((w.B, w.H_kv), -1, dtype=torch.int32, device="cuda")
    out = torch.full((w.B, w.H_q, w.d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.B, w.H_q), float("nan"), dtype=torch.float32, device="cuda")
    lc.lc_decode_step(case.idx, q, case.K, case.V, budget, out, case.ws, lse=lse, chunk_ids=ids, counts=counts)
    torch.cuda.synchronize()
    got = None
    if with_ids:
        ids_h, counts_h = ids.cpu().numpy(), counts.cpu().numpy()
        got = [[ids_h[b, h, : counts_h[b, h]].copy() for h in range(w.H_kv)] for b in range(w.B)]
    return got, out.cpu().numpy(), lse.cpu().numpy()


def attention_errors(got: np.ndarray, ref: np.ndarray):
    """(max abs error, relative L2 error) over the whole output."""
    got = got.astype(np.float64)
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
