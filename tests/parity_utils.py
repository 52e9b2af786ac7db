"""Helpers shared by the GPU parity tests: build inputs for a workload, run the CPU oracle
on the host copy of the same bits, and the comparison rules.

Tolerances (stated once here, used by every parity test):
  psi      |gpu - oracle| <= 1e-3 * |oracle| + 1e-7 * G*W/L        (fp32 accumulation)
  w_m      1e-3 relative (free-running), 2e-6 relative when both sides read the same psi
  k_m      equal, or the oracle's sorted cumulative mass shows a crossing within 1e-4 relative
  budgets  bit-exact when both sides read the same statistics; free-running: a head whose budgets
           differ from the oracle's must be explained (see free_running_check), anything else fails
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
W_RTOL = 2e-6                  # masses when both sides read the same psi bits: the fp32 rounding of the result ...
W_QUANTUM = 2.0 ** -44         # ... plus the fixed point the GPU sums in: every addend is rounded to a multiple of this


def assert_masses_close(w_gpu, w_ref, n_candidates):
    """Eq. 6 on the same psi bits.  The GPU adds the scores in 2^-44 fixed point (integer adds commute, so the sum is
    the same on every run) and rounds the total to fp32 once: |gpu - exact| <= n * 2^-45 + 2^-24 * |exact|."""
    np.testing.assert_allclose(w_gpu, w_ref, rtol=W_RTOL, atol=n_candidates * W_QUANTUM / 2)


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


def split_on_rounding_boundary(w_t: float, w_v: float, n_t: int, n_v: int, a: int) -> bool:
    """Eq. 8 rounds share_t * a half up: true when that product lies within 1e-4 * a of a .5
    boundary, so that a 1e-3-relative difference in the masses may move one token."""
    x = O.text_share(w_t, w_v, n_t, n_v) * a + 0.5
    return abs(x - round(x)) < TIE_RTOL * max(a, 1)


def free_running_check(p: O.Params, res: dict, mask: np.ndarray, w_g, k_g, n_mod_g, bud_g, kept_of, say=None):
    """Whole-path comparison of one batch item: the GPU's free-running results against the
    oracle's (`res` = oracle.evict of the same inputs).
      w_g[NL,H,M], k_g[NL,H,M], n_mod_g[M], bud_g[NL,H,M]: the GPU's statistics and budgets;
      kept_of(l, h) -> the GPU's kept positions of that head.
    Rules: masses within 1e-3 relative; a theta-mass count that differs must sit on a crossing of
    the oracle's cumulative mass (k_count_ok); the oracle's allocation run on the GPU's own
    statistics must give the GPU's budgets bit for bit; a head whose budgets differ from the
    free-running oracle's is excused only by a (checked) count difference in its own or an earlier
    layer - the layer totals of Eq. 10-11 couple all heads from there on - or by an Eq. 8 product on
    a rounding boundary; kept positions are compared with the GPU's budgets on both sides and may
    differ only in near-ties of the oracle's pooled scores.  Returns a dict of counts."""
    NL, H, M = k_g.shape
    L, W = p.ctx_len, p.window
    nc = L - W
    assert tuple(int(x) for x in n_mod_g) == tuple(int(x) for x in res["n_mod"])
    np.testing.assert_allclose(w_g, res["w"], rtol=1e-3, atol=1e-30)
    replay = O.allocate(w_g, k_g.astype(np.int64), n_mod_g, p)
    np.testing.assert_array_equal(bud_g, replay, err_msg="allocation differs from the oracle's on the same statistics")
    out = dict(k_excused=0, budget_excused=0, budget_unexcused=0, kept_excused=0, kept_unexcused=0, heads=NL * H)
    k_diff_upto = np.zeros(NL, dtype=bool)
    for l in range(NL):
        for h in range(H):
            for m in range(M):
                if k_g[l, h, m] != res["kcnt"][l, h, m]:
                    vals = res["psi"][l, h, :nc][mask[:nc] == m]
                    assert k_count_ok(int(k_g[l, h, m]), vals, p.theta), ("theta-mass count", l, h, m, int(k_g[l, h, m]), int(res["kcnt"][l, h, m]))
                    out["k_excused"] += 1
                    k_diff_upto[l:] = True
    for l in range(NL):
        for h in range(H):
            bg = [int(x) for x in bud_g[l, h]]
            bo = [int(x) for x in res["budgets"][l, h]]
            if bg != bo:
                ok = bool(k_diff_upto[l])
                if not ok and M == 2 and sum(bg) == sum(bo) and p.mpa_mode == 1:
                    ok = split_on_rounding_boundary(float(res["w"][l, h, 0]), float(res["w"][l, h, 1]),
                                                    int(n_mod_g[0]), int(n_mod_g[1]), sum(bo))
                out["budget_excused" if ok else "budget_unexcused"] += 1
                if not ok and say:
                    say(f"unexcused budget difference at layer {l} head {h}: gpu {bg} oracle {bo}")
            if p.keep_all or p.select_mode == 1:
                ref = res["kept"][l][h]
            else:
                ref = O.select_n(res["psi_pool"][l, h], mask, bg, L, W, p.mpa_mode)
            kept = np.asarray(kept_of(l, h))
            assert len(kept) == sum(bg) + W or p.keep_all
            if M == 2:
                e, u = kept_diff_excused(kept, ref, res["psi_pool"][l, h], mask, bg[0], bg[1], nc)
            else:
                u = 0 if np.array_equal(kept, ref) else 1
                e = 0
            out["kept_excused"] += e
            out["kept_unexcused"] += u
    return out
