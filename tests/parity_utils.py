"""Helpers shared by the GPU parity tests: build inputs for a workload, run the CPU oracle
on the host copy of the same bits, and the comparison rules.

Tolerances (stated once here, used by every parity test):
  psi      |gpu - oracle| <= 1e-3 * |oracle| + 1e-7 * G*W/L        (fp32 accumulation)
  w_m      1e-3 relative (free-running), 2e-6 relative when both sides read the same psi
  k_m      equal, or the oracle's sorted cumulative mass shows a crossing within 1e-4 relative
  budgets  bit-exact when both sides read the same statistics
  kept     bit-exact when both sides read the same scores and budgets; free-running: every index
           in the symmetric difference has an oracle score within 1e-4 relative of the threshold
  decode   2e-3 absolute on the fp32 output; bf16 output within 1 bf16 ulp of the rounded oracle
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import madakv_oracle as O
from paper_2506_15724_amd import workloads as WL

PSI_RTOL = 1e-3
DECODE_ATOL = 2e-3
TIE_RTOL = 1e-4


def oracle_params(wl: WL.Workload, **kw) -> O.Params:
    base = dict(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                ctx_len=wl.ctx_len, window=wl.window, budget=wl.budget, pool_k=wl.pool_k)
    base.update(kw)
    return O.Params(**base)


def make_inputs(wl: WL.Workload, device):
    """Device tensors q_win[NL,B,Hq,W,d], k, v [NL,B,H,L,d], mask[B,L] and the host masks."""
    masks = [WL.modality_mask(wl, b) for b in range(wl.batch)]
    qs, ks, vs = [], [], []
    for l in range(wl.n_layers):
        ql, kl, vl = [], [], []
        for b in range(wl.batch):
            q, k, v = WL.layer_inputs(wl, l, b, masks[b], device)
            ql.append(q); kl.append(k); vl.append(v)
        qs.append(torch.stack(ql)); ks.append(torch.stack(kl)); vs.append(torch.stack(vl))
    q, k, v = torch.stack(qs).contiguous(), torch.stack(ks).contiguous(), torch.stack(vs).contiguous()
    mask = torch.from_numpy(np.stack(masks)).to(device)
    return q, k, v, mask, masks


def psi_close(gpu: np.ndarray, ref: np.ndarray, G: int, W: int, L: int):
    eps = 1e-7 * G * W / L
    err = np.abs(gpu.astype(np.float64) - ref)
    bad = err > PSI_RTOL * np.abs(ref) + eps
    return int(bad.sum()), float((err / (np.abs(ref) + eps)).max())


def k_count_ok(k_gpu: int, values: np.ndarray, theta: float) -> bool:
    """values: the oracle's candidate scores of one modality.  Accept k_gpu when the sorted
    cumulative mass crosses theta*w within 1e-4 relative at k_gpu."""
    if values.size == 0 or values.sum() <= 0:
        return k_gpu == 0
    c = np.cumsum(np.sort(values)[::-1])
    tgt = theta * values.sum()
    if k_gpu < 1 or k_gpu > values.size:
        return False
    hi_ok = c[k_gpu - 1] >= tgt * (1 - TIE_RTOL)
    lo_ok = (k_gpu == 1) or (c[k_gpu - 2] < tgt * (1 + TIE_RTOL))
    return bool(hi_ok and lo_ok)


def kept_diff_excused(kept_gpu: np.ndarray, kept_ref: np.ndarray, score: np.ndarray, mask: np.ndarray,
                      b_t: int, b_v: int, nc: int) -> tuple[int, int]:
    """(excused, unexcused) count of indices in the symmetric difference of the candidate parts."""
    a, r = set(kept_gpu.tolist()), set(kept_ref.tolist())
    diff = [i for i in (a ^ r) if i < nc]
    if not diff:
        return 0, 0
    exc = unexc = 0
    for i in diff:
        m = int(mask[i])
        sel = mask[:nc] == m
        b = b_t if m == 0 else b_v
        srt = np.sort(score[:nc][sel])[::-1]
        thr = srt[b - 1] if 0 < b <= srt.size else (srt[-1] if srt.size else 0.0)
        if abs(score[i] - thr) <= TIE_RTOL * abs(thr):
            exc += 1
        else:
            unexc += 1
    return exc, unexc


def bf16_round(x: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
