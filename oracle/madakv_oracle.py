"""MadaKV eviction + decode, written out plainly in NumPy float64.

TEST INFRASTRUCTURE ONLY.  This module is the checker for the HIP library: it is
imported by the tests, by the smoke check and by the benchmark's CPU-baseline
leg, and by nothing on the product path.  It imports nothing from the HIP
package and shares no code with it.

Everything here follows the MadaKV paper (arxiv 2506.15724), Section 3:

  * Sec. 3.1, Eq. 3-5   decode: append K_t, V_t, softmax(q K^T / sqrt(d_k)) V
  * Sec. 3.3, Eq. 7     proxy-token score  psi(i) = sum_{j in P} alpha_{j->i}
  * Sec. 3.3, Eq. 6     modality mass      w_v, w_t
  * Sec. 3.3, Eq. 8     per-head, per-modality budget split (MPA)
  * Sec. 3.3, Eq. 9     theta-mass sparsity counts k_v, k_t
  * Sec. 3.3, Eq. 10-11 layer compensation K^l and the budget recurrence (HCC)

The paper leaves several things open (size of the proxy set, theta, how Eq. 10-11
turn into integers, tie-breaks, pooling).  Each function states the reading it
takes.  The HCC allocation reading (clamps, apportionment) has no worked example
in the paper to pin it against: it is "parity unpinned" with respect to the paper
and is pinned only by its own invariants (exact conservation, Eq. 11 identity,
sign behaviour, brute-force apportionment).

Conventions
-----------
modality id 0 = text, 1 = image (the mask array holds these ids).
L = context length, W = number of proxy (observation-window) tokens = the last W
prompt positions, H = KV heads, Hq = query heads, G = Hq / H, d = head_dim.
Candidates for eviction are positions [0, L-W); the window is always kept and is
counted inside the per-head budget.
All arrays are float64 / int64 unless stated.  One call handles one batch item.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

TEXT, IMAGE = 0, 1


@dataclasses.dataclass
class Params:
    """Hyper-parameters of the method (paper Sec. 3.3 names theta, |P| and the
    layer budget but prints no values; the defaults are this build's reading)."""
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_len: int
    window: int            # |P|
    budget: int            # tokens kept per KV head per layer, window included
    pool_k: int = 1        # odd; 1 = Eq. 7 scores used as they are
    mpa_mode: int = 1      # 1 = Eq. 8 split, 0 = modality-agnostic, 2 = text first, 3 = image first (fixed priority)
    hcc_mode: int = 1      # 1 = Eq. 9-11 with demand-driven head totals, 0 = every head gets the same budget,
                           # 2 = Eq. 9-11 layer totals shared equally by the heads of the layer (Eq. 8 as printed)
    pool_mode: int = 0     # 0 = max-pool, 1 = average-pool
    share_mode: int = 0    # Eq. 6 sums over 0 = the candidates, 1 = all L columns (window included)
    select_mode: int = 0   # 0 = top scores, 1 = first `sink_tokens` + most recent candidates (score-free baseline)
    sink_tokens: int = 4
    n_modalities: int = 2  # the paper has text and image; more (audio, video: its Sec. 6) make Eq. 6, 8, 9 M-way
    cache_fp8: int = 0     # 1 = the reduced cache holds K, V as 8-bit floats (E4M3), not part of the paper
    hcc_rho: int = 2       # clamp ratio around the running nominal budget
    theta: float = 0.9     # Eq. 9 threshold
    softmax_scale: float = 0.0  # 0 -> 1/sqrt(head_dim)

    @property
    def scale(self) -> float:
        return self.softmax_scale if self.softmax_scale > 0 else 1.0 / math.sqrt(self.head_dim)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_cand(self) -> int:
        return self.ctx_len - self.window

    @property
    def keep_all(self) -> bool:
        return self.budget >= self.ctx_len


# --------------------------------------------------------------------------- #
# Eq. 7: proxy-token scores
# --------------------------------------------------------------------------- #
def window_scores(q_win: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """psi[h, i] = sum over the proxy rows of the attention they pay to key i.

    q_win : [Hq, W, d]  queries of the last W prompt positions
    k     : [H, L, d]   keys of the whole prompt
    Proxy row r sits at absolute position L-W+r and, the prefill being causal,
    sees keys 0..L-W+r only.  With grouped queries the G query heads that share
    KV head h (query head j uses KV head j // G) all add into psi[h].
    Returns psi [H, L].   (Sec. 3.3 Eq. 7; logits scaled as in Eq. 5.)
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    Hq, W, d = q_win.shape
    H, L, _ = k.shape
    G = Hq // H
    psi = np.zeros((H, L), dtype=np.float64)
    pos = np.arange(L)
    for h in range(H):
        for g in range(G):
            logits = scale * (q_win[h * G + g] @ k[h].T)          # [W, L]
            for r in range(W):
                p = L - W + r
                row = np.where(pos <= p, logits[r], -np.inf)
                row = row - row.max()
                e = np.exp(row)
                psi[h] += e / e.sum()
    return psi


def proxy_row_lse(q_win: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """lse[j, r] = log sum_i exp(scale * q_win[j, r] . k[j // G, i]) over the keys proxy row r sees:
    the softmax normaliser a prefill attention kernel has for these rows anyway."""
    q_win = np.asarray(q_win, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    Hq, W, d = q_win.shape
    H, L, _ = k.shape
    G = Hq // H
    out = np.zeros((Hq, W), dtype=np.float64)
    for j in range(Hq):
        logits = scale * (q_win[j] @ k[j // G].T)
        for r in range(W):
            row = logits[r, :L - W + r + 1]
            mx = row.max()
            out[j, r] = mx + math.log(np.exp(row - mx).sum())
    return out


def window_scores_from_lse(q_win: np.ndarray, k: np.ndarray, lse: np.ndarray, scale: float) -> np.ndarray:
    """Eq. 7 when the row normalisers are given: psi[h, i] = sum over proxy rows of exp(logit - lse)."""
    q_win = np.asarray(q_win, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    Hq, W, d = q_win.shape
    H, L, _ = k.shape
    G = Hq // H
    psi = np.zeros((H, L), dtype=np.float64)
    for j in range(Hq):
        logits = scale * (q_win[j] @ k[j // G].T)
        for r in range(W):
            n = L - W + r + 1
            psi[j // G, :n] += np.exp(logits[r, :n] - lse[j, r])
    return psi


def window_attention(q_win: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """The prefill attention of the last W prompt positions (Eq. 5 applied to the proxy rows of
    Sec. 3.3): out[j, r] = softmax(scale * q_win[j, r] . K^T) V over the keys row r sees (causal:
    keys 0 .. L-W+r), and the natural log-sum-exp of each row.  Query head j reads KV head j // G.
    This is the step before the eviction path: the softmax rows it forms are the alpha of Eq. 7.
    Returns (out [Hq, W, d], lse [Hq, W])."""
    q_win = np.asarray(q_win, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    Hq, W, d = q_win.shape
    H, L, _ = k.shape
    G = Hq // H
    out = np.zeros((Hq, W, d), dtype=np.float64)
    lse = np.zeros((Hq, W), dtype=np.float64)
    for j in range(Hq):
        for r in range(W):
            n = L - W + r + 1
            s = scale * (k[j // G, :n] @ q_win[j, r])
            mx = s.max()
            e = np.exp(s - mx)
            out[j, r] = (e / e.sum()) @ v[j // G, :n]
            lse[j, r] = mx + math.log(e.sum())
    return out, lse


# --------------------------------------------------------------------------- #
# Eq. 6 and Eq. 9: modality mass and theta-mass counts
# --------------------------------------------------------------------------- #
def modality_mass(psi_h: np.ndarray, mask: np.ndarray, window: int, n_modalities: int = 2):
    """(w[M], n[M]) over the candidates [0, L-W) of one head (Eq. 6, one sum per modality)."""
    L = psi_h.shape[0]
    c = L - window
    w = np.zeros(n_modalities, dtype=np.float64)
    n = np.zeros(n_modalities, dtype=np.int64)
    for m in range(n_modalities):
        sel = mask[:c] == m
        n[m] = int(sel.sum())
        w[m] = float(psi_h[:c][sel].sum())
    return w, n


def theta_mass_count(values: np.ndarray, theta: float) -> int:
    """Smallest number of entries of `values` whose sum reaches theta * sum(values)
    (Eq. 9): the entries are taken from the largest down.  0 if there is nothing
    to cover (no entries or zero mass)."""
    n = values.shape[0]
    if n == 0:
        return 0
    total = float(values.sum())
    if total <= 0.0:
        return 0
    srt = np.sort(values)[::-1]
    c = np.cumsum(srt)
    target = theta * total
    hit = np.nonzero(c >= target)[0]
    return int(hit[0]) + 1 if hit.size else n


def modality_stats(psi: np.ndarray, mask: np.ndarray, window: int, theta: float, share_mode: int = 0,
                   n_modalities: int = 2):
    """Per head: w[H,M] (Eq. 6), kcnt[H,M] (Eq. 9), and n_mod[M] candidate counts.
    Uses the raw Eq. 7 scores (never the pooled ones).  share_mode = 1 is the other reading
    of Eq. 6: X_v, X_t are all prompt positions, so the window columns add to w (the counts
    of Eq. 9 and n_mod stay on the candidates, the only tokens that can be evicted)."""
    H, L = psi.shape
    c = L - window
    M = n_modalities
    w = np.zeros((H, M), dtype=np.float64)
    kcnt = np.zeros((H, M), dtype=np.int64)
    n_mod = np.zeros(M, dtype=np.int64)
    for h in range(H):
        w[h], n_mod = modality_mass(psi[h], mask, window, M)
        if share_mode == 1:
            for m in range(M):
                w[h, m] += float(psi[h, c:][mask[c:] == m].sum())
        for m in range(M):
            kcnt[h, m] = theta_mass_count(psi[h, :c][mask[:c] == m], theta)
    return w, kcnt, n_mod


def text_share(w_t: float, w_v: float, n_t: int, n_v: int) -> float:
    """Share of the head's attention mass that goes to text (the weight in Eq. 8).
    If the head put no mass on any candidate, fall back to the token share."""
    tot = float(w_t) + float(w_v)
    if tot > 0.0:
        return float(w_t) / tot
    return n_t / (n_t + n_v) if (n_t + n_v) > 0 else 0.0


# --------------------------------------------------------------------------- #
# Score pooling (not in the paper; ranking only)
# --------------------------------------------------------------------------- #
def pool_scores(psi: np.ndarray, window: int, pool_k: int, pool_mode: int = 0) -> np.ndarray:
    """psi_pool[h, i] = max of psi[h, j] over candidates j with |j-i| <= (pool_k-1)/2,
    for i in [0, L-W).  Position-based, clipped at both ends of the candidate range,
    blind to modality boundaries.  pool_k = 1 returns the candidate scores as is.
    pool_mode = 1 takes the mean of the same (clipped) neighbourhood instead of the max."""
    H, L = psi.shape
    c = L - window
    r = (pool_k - 1) // 2
    out = np.empty((H, c), dtype=np.float64)
    for i in range(c):
        lo, hi = max(0, i - r), min(c, i + r + 1)
        out[:, i] = psi[:, lo:hi].max(axis=1) if pool_mode == 0 else psi[:, lo:hi].mean(axis=1)
    return out


# --------------------------------------------------------------------------- #
# Eq. 9-11: hierarchical compression compensation, in integers
# --------------------------------------------------------------------------- #
def _largest_remainder(base: np.ndarray, rem: np.ndarray, extra: int) -> np.ndarray:
    """Add 1 to the `extra` entries with the largest remainder, ties to the lower index."""
    out = base.copy()
    order = sorted(range(len(base)), key=lambda h: (-int(rem[h]), h))
    for h in order[:extra]:
        out[h] += 1
    return out


def apportion(total: int, demand: np.ndarray, n_cand: int) -> np.ndarray:
    """Integers a_h >= 0, a_h <= n_cand, sum a_h == total, proportional to `demand`
    when scaling down, and proportional to the head-room n_cand - demand when
    scaling up (Hamilton / largest remainder, ties to the lower head index)."""
    demand = np.asarray(demand, dtype=np.int64)
    D = int(demand.sum())
    if total == D:
        return demand.copy()
    if total < D:
        num = total * demand                      # exact in int64
        base = num // D
        rem = num % D
        return _largest_remainder(base, rem, total - int(base.sum()))
    room = n_cand - demand
    S = total - D
    Rm = int(room.sum())
    num = S * room
    base = num // Rm
    rem = num % Rm
    return demand + _largest_remainder(base, rem, S - int(base.sum()))


def hcc_allocate(kcnt: np.ndarray, p: Params, trace: dict | None = None) -> np.ndarray:
    """Per-head candidate totals a[N_L, H] from the theta-mass counts kcnt[N_L, H, 2].

    Reading of Eq. 9-11 taken here.  Budgets are counted in candidate tokens
    (beta = budget - W per head).  A head's demand is its Eq. 9 count k_t + k_v.
    The model holds one integer pool R = N_L * H * beta.  Layer l (0-based, rem =
    N_L - l layers left) has the nominal per-head budget phi^l = R / (H * rem);
    demands are clamped to [phi/rho, rho*phi] (and to [1, n_cand]); the layer draws
    A = sum of clamped demands, itself clamped so that the layers after it can
    still be given between beta_floor and n_cand per head; the last layer draws
    what is left.  Heads receive `apportion(A, demand)`.  Then R -= A, which is
    Eq. 11 with K^l = sum_h (a_h - phi^l) taken per head (divided by H):
        phi^{l+1} = phi^l - (K^l / H) / (rem - 1).
    hcc_mode = 0 gives every head beta.  hcc_mode = 2 keeps the layer totals A but gives every
    head of a layer the same share of it.
    """
    NL, H, _ = kcnt.shape
    beta = p.budget - p.window
    n_c = p.n_cand
    a = np.zeros((NL, H), dtype=np.int64)
    if p.hcc_mode == 0:
        a[:] = beta
        return a
    rho = p.hcc_rho
    beta_floor = max(1, beta // (rho * rho))
    R = NL * H * beta
    if trace is not None:
        trace["phi"], trace["K"], trace["R"] = [], [], []
    for l in range(NL):
        rem = NL - l
        lo = max(1, -((-R) // (rho * H * rem)))            # ceil
        hi = min(n_c, (rho * R) // (H * rem))
        dem = np.clip(kcnt[l].sum(axis=-1), lo, hi).astype(np.int64)
        D = int(dem.sum())
        if l == NL - 1:
            A = R
        else:
            A = min(max(D, R - (rem - 1) * H * n_c), R - (rem - 1) * H * beta_floor)
        if p.hcc_mode == 2:
            # Eq. 8 as printed: one budget phi^l for every head of the layer; the layer total of
            # Eq. 10-11 is shared equally, the A mod H spare tokens go to the lowest heads
            a[l] = A // H + (np.arange(H) < A % H)
        else:
            a[l] = apportion(A, dem, n_c)
        if trace is not None:
            phi = R / (H * rem)
            trace["phi"].append(phi)
            trace["K"].append(float(a[l].sum()) - H * phi)
            trace["R"].append(R)
        R -= A
    return a


def mpa_split(a: int, w_t: float, w_v: float, n_t: int, n_v: int, mpa_mode: int = 1) -> tuple[int, int]:
    """Eq. 8 in integers: b_t = round-half-up(share_t * a), b_v = a - b_t; a modality
    that has fewer candidates than its budget hands the surplus to the other.
    mpa_mode 2 / 3 are the fixed-priority baselines the paper argues against (Sec. 1, 2):
    the preferred modality (text / image) takes all it can, the other gets the rest."""
    s_t = text_share(w_t, w_v, n_t, n_v)
    if mpa_mode == 2:
        s_t = 1.0
    elif mpa_mode == 3:
        s_t = 0.0
    b_t = int(math.floor(s_t * a + 0.5))
    b_v = a - b_t
    if b_t > n_t:
        b_t, b_v = n_t, a - n_t
    if b_v > n_v:
        b_v, b_t = n_v, a - n_v
    return b_t, b_v


def mpa_split_n(a: int, w: np.ndarray, n: np.ndarray, mpa_mode: int = 1) -> list[int]:
    """Eq. 8 for M modalities, in integers.  Two modalities: exactly `mpa_split`.  More:
    quotas share_m * a are floored and the spare tokens go one each to the largest fractional
    parts (ties: lower modality id); a modality short of candidates is cut to what it has and
    the surplus goes to the others in order of decreasing share (ties: lower id), each up to its
    room.  mpa_mode 2 / 3 fill the modalities greedily in ascending / descending id order."""
    M = len(n)
    n = [int(x) for x in n]
    if M == 2:
        return list(mpa_split(a, float(w[0]), float(w[1]), n[0], n[1], mpa_mode))
    if mpa_mode in (2, 3):
        order = range(M) if mpa_mode == 2 else range(M - 1, -1, -1)
        b, left = [0] * M, a
        for m in order:
            b[m] = min(left, n[m]); left -= b[m]
        return b
    tot = 0.0
    for m in range(M):
        tot += float(w[m])
    nt = sum(n)
    share = [(float(w[m]) / tot) if tot > 0.0 else ((n[m] / nt) if nt > 0 else 0.0) for m in range(M)]
    quota = [share[m] * a for m in range(M)]
    b = [int(math.floor(x)) for x in quota]
    frac = [quota[m] - b[m] for m in range(M)]
    spare = a - sum(b)
    for m in sorted(range(M), key=lambda m: (-frac[m], m))[:max(spare, 0)]:
        b[m] += 1
    surplus = 0
    for m in range(M):
        if b[m] > n[m]:
            surplus += b[m] - n[m]; b[m] = n[m]
    for m in sorted(range(M), key=lambda m: (-share[m], m)):
        give = min(surplus, n[m] - b[m])
        b[m] += give; surplus -= give
    return b


def allocate(w: np.ndarray, kcnt: np.ndarray, n_mod: np.ndarray, p: Params,
             trace: dict | None = None) -> np.ndarray:
    """budgets[N_L, H, M] for one batch item.
    w[N_L,H,M] are the Eq. 6 masses as they cross the interface (float32 values),
    kcnt[N_L,H,M] the Eq. 9 counts, n_mod[M] the candidate counts per modality.
    mpa_mode = 0 puts the whole total in slot 0: selection then ignores modality."""
    NL, H, M = kcnt.shape
    out = np.zeros((NL, H, M), dtype=np.int64)
    if p.keep_all:
        out[:, :, :] = np.asarray(n_mod, dtype=np.int64)[None, None, :]
        return out
    a = hcc_allocate(kcnt, p, trace)
    for l in range(NL):
        for h in range(H):
            if p.mpa_mode == 0:
                out[l, h, 0] = a[l, h]
            else:
                w32 = np.asarray(w[l, h], dtype=np.float32).astype(np.float64)
                out[l, h] = mpa_split_n(int(a[l, h]), w32, n_mod, p.mpa_mode)
    return out


# --------------------------------------------------------------------------- #
# Eviction: top-k per head per modality, then gather
# --------------------------------------------------------------------------- #
def top_indices(scores: np.ndarray, idx: np.ndarray, b: int) -> np.ndarray:
    """The b entries of idx with the largest scores; equal scores: lower index first."""
    if b <= 0:
        return np.zeros(0, dtype=np.int64)
    order = sorted(range(len(idx)), key=lambda j: (-scores[j], idx[j]))
    return idx[np.asarray(order[:b], dtype=np.int64)]


def select_sink_recent(total: int, L: int, window: int, sink_tokens: int) -> np.ndarray:
    """Score-free baseline (attention sinks + recency): the first min(sink, total) candidates and
    the most recent total - that many candidates, then the window."""
    c = L - window
    total = min(total, c)
    s = min(sink_tokens, total)
    keep = np.concatenate([np.arange(s, dtype=np.int64), np.arange(c - (total - s), c, dtype=np.int64)])
    return np.concatenate([keep, np.arange(c, L, dtype=np.int64)])


def select(psi_pool_h: np.ndarray, mask: np.ndarray, b_t: int, b_v: int,
           L: int, window: int, mpa_mode: int = 1) -> np.ndarray:
    """Kept positions of one head: per modality the b_m best-scored candidates, all in
    ascending position, then the window positions L-W..L-1 (Sec. 3.3, last line of
    the MPA paragraph: eviction is per head and per modality)."""
    c = L - window
    cand = np.arange(c, dtype=np.int64)
    if mpa_mode == 0:
        keep = top_indices(psi_pool_h, cand, b_t + b_v)
    else:
        parts = []
        for m, b in ((TEXT, b_t), (IMAGE, b_v)):
            sel = mask[:c] == m
            parts.append(top_indices(psi_pool_h[sel], cand[sel], b))
        keep = np.concatenate(parts)
    keep = np.sort(keep)
    return np.concatenate([keep, np.arange(c, L, dtype=np.int64)])


def select_n(psi_pool_h: np.ndarray, mask: np.ndarray, budgets, L: int, window: int, mpa_mode: int = 1) -> np.ndarray:
    """`select` for any number of modalities: budgets[m] best-scored candidates of modality m."""
    c = L - window
    cand = np.arange(c, dtype=np.int64)
    if mpa_mode == 0:
        keep = top_indices(psi_pool_h, cand, int(sum(budgets)))
    else:
        parts = []
        for m, b in enumerate(budgets):
            sel = mask[:c] == m
            parts.append(top_indices(psi_pool_h[sel], cand[sel], int(b)))
        keep = np.concatenate(parts)
    keep = np.sort(keep)
    return np.concatenate([keep, np.arange(c, L, dtype=np.int64)])


def gather(x_h: np.ndarray, kept: np.ndarray) -> np.ndarray:
    """Rows `kept` of x_h[L, d], copied."""
    return x_h[kept].copy()


# --------------------------------------------------------------------------- #
# 8-bit reduced cache (an encoding, not part of the paper): OCP FP8 E4M3
# --------------------------------------------------------------------------- #
def e4m3_decode_table() -> np.ndarray:
    """The 256 values of the E4M3 format: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits;
    exponent 0 is subnormal (m * 2^-9); there are no infinities; S.1111.111 is NaN."""
    t = np.zeros(256, dtype=np.float64)
    for code in range(256):
        sgn = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sgn * m * 2.0 ** -9
        else:
            t[code] = sgn * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


def quantize_e4m3(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each value, ties to the even mantissa, magnitudes that round above
    the largest finite value (448) saturate to it."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    code = np.zeros(x.shape, dtype=np.int64)
    small = a < 2.0 ** -6
    code[small] = np.rint(a[small] * 512.0).astype(np.int64)          # subnormal grid 2^-9; 8 is the first normal code
    big = ~small
    mant, ex = np.frexp(a[big])                                        # a = mant * 2^ex, mant in [0.5, 1)
    e = ex - 1
    q = np.rint((mant * 2.0 - 1.0) * 8.0).astype(np.int64)             # 0..8
    e = e + (q == 8); q = np.where(q == 8, 0, q)
    code[big] = ((e + 7) << 3) | q
    code = np.where(a >= 448.0, 0x7E, np.minimum(code, 0x7E))
    return (code | np.where(np.signbit(x), 0x80, 0)).astype(np.uint8)


def dequantize_e4m3(codes: np.ndarray) -> np.ndarray:
    return e4m3_decode_table()[np.asarray(codes, dtype=np.uint8)]


# --------------------------------------------------------------------------- #
# Eq. 3-5: decode over a (reduced) cache
# --------------------------------------------------------------------------- #
def attend(q: np.ndarray, k_c: np.ndarray, v_c: np.ndarray, scale: float) -> np.ndarray:
    """softmax(scale * q k_c^T) v_c for one query vector q[d] (Eq. 5)."""
    s = scale * (k_c.astype(np.float64) @ q.astype(np.float64))
    s = s - s.max()
    e = np.exp(s)
    return (e / e.sum()) @ v_c.astype(np.float64)


def decode_step(q: np.ndarray, k_new, v_new, k_cache: list, v_cache: list, scale: float):
    """One decode step for one layer of one batch item.
    q[Hq,d]; k_new, v_new [H,d] or None; k_cache/v_cache: lists of H arrays [len_h, d]
    which are extended in place by the new row (Eq. 4) before attention (Eq. 5).
    Returns out[Hq, d]."""
    Hq, d = q.shape
    H = len(k_cache)
    G = Hq // H
    out = np.zeros((Hq, d), dtype=np.float64)
    for h in range(H):
        if k_new is not None:
            k_cache[h] = np.concatenate([k_cache[h], np.asarray(k_new[h], dtype=np.float64)[None]], 0)
            v_cache[h] = np.concatenate([v_cache[h], np.asarray(v_new[h], dtype=np.float64)[None]], 0)
        for g in range(G):
            out[h * G + g] = attend(q[h * G + g], k_cache[h], v_cache[h], scale)
    return out


# --------------------------------------------------------------------------- #
# Re-eviction during generation (not in the paper, which evicts once after the prefill; its
# Sec. 6 leaves long generation open)
# --------------------------------------------------------------------------- #
def reevict_head(q_recent_h: np.ndarray, k_rows: np.ndarray, v_rows: np.ndarray, origin: np.ndarray, mask: np.ndarray,
                 total: int, p: Params):
    """One KV head whose cache has grown by appended rows is brought back to `total` + W rows.
    q_recent_h [G, W, d]: queries of the tokens in the last W rows; k_rows, v_rows [len, d]: the
    head's cache; origin [len]: original position of every row (< ctx_len: a prompt position whose
    modality the mask gives; >= ctx_len: a generated token, which is text).
    The steps are those of the prompt eviction applied to the rows of the cache, per head: Eq. 7
    with the last W rows as proxies (proxy r sees rows up to its own), Eq. 6 masses and candidate
    counts over the rows before them, pooling over neighbouring rows, the Eq. 8 split of the
    unchanged total, the best candidates per modality (ties: lower row), then the proxies.
    Returns (sel rows, budgets, w, n_mod, psi, psi_pool)."""
    n, W = k_rows.shape[0], p.window
    rowmod = np.where(origin < p.ctx_len, mask[np.minimum(origin, p.ctx_len - 1)], TEXT).astype(mask.dtype)
    rowmod = np.minimum(rowmod, p.n_modalities - 1)
    psi = window_scores(q_recent_h, k_rows[None], p.scale)[0]
    psi = psi.astype(np.float32).astype(np.float64)                       # the scores cross an fp32 interface
    w, n_mod = modality_mass(psi, rowmod, 0 if p.share_mode else W, p.n_modalities)
    if p.share_mode:                                                      # masses over all rows, counts over the candidates
        n_mod = modality_mass(psi, rowmod, W, p.n_modalities)[1]
    pool = pool_scores(psi[None], W, p.pool_k, p.pool_mode)[0]
    w32 = np.asarray(w, dtype=np.float32).astype(np.float64)
    bud = [min(total, n - W), 0] + [0] * (p.n_modalities - 2) if p.mpa_mode == 0 else mpa_split_n(min(total, n - W), w32, n_mod, p.mpa_mode)
    if p.select_mode == 1:
        sel = select_sink_recent(sum(bud), n, W, p.sink_tokens)
    else:
        sel = select_n(pool, rowmod, bud, n, W, p.mpa_mode)
    return sel, bud, w, n_mod, psi, pool


# --------------------------------------------------------------------------- #
# The whole eviction for one batch item
# --------------------------------------------------------------------------- #
def score_layer(q_win: np.ndarray, k: np.ndarray, mask: np.ndarray, p: Params,
                interface_fp32: bool = True):
    """Eq. 7, Eq. 6, Eq. 9 and pooling for one layer: (psi, psi_pool, w, kcnt, n_mod).
    With interface_fp32 the scores are rounded to float32 once, as they are when
    they cross the library boundary, before the statistics are taken from them."""
    psi = window_scores(q_win, k, p.scale)
    if interface_fp32:
        psi = psi.astype(np.float32).astype(np.float64)
    w, kcnt, n_mod = modality_stats(psi, mask, p.window, p.theta, p.share_mode, p.n_modalities)
    psi_pool = pool_scores(psi, p.window, p.pool_k, p.pool_mode)
    return psi, psi_pool, w, kcnt, n_mod


def evict(q_win: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray, p: Params):
    """Full eviction of one batch item.
    q_win[N_L,Hq,W,d], k,v[N_L,H,L,d], mask[L].
    Returns dict with psi, psi_pool, w, kcnt, n_mod, budgets, kept (list of lists of
    index arrays), k_c / v_c (lists of lists of arrays [len, d])."""
    NL, H, L = k.shape[0], k.shape[1], k.shape[2]
    res = {"psi": [], "psi_pool": [], "w": [], "kcnt": []}
    n_mod = None
    for l in range(NL):
        psi, psi_pool, w, kcnt, n_mod = score_layer(q_win[l], k[l], mask, p)
        res["psi"].append(psi); res["psi_pool"].append(psi_pool)
        res["w"].append(w); res["kcnt"].append(kcnt)
    for key in ("psi", "psi_pool", "w", "kcnt"):
        res[key] = np.stack(res[key])
    res["n_mod"] = n_mod
    res["budgets"] = allocate(res["w"], res["kcnt"], n_mod, p)
    res["kept"], res["k_c"], res["v_c"] = [], [], []
    for l in range(NL):
        kl, kc, vc = [], [], []
        for h in range(H):
            if p.keep_all:
                kept = np.arange(L, dtype=np.int64)
            else:
                bud = [int(x) for x in res["budgets"][l, h]]
                if p.select_mode == 1:
                    kept = select_sink_recent(sum(bud), L, p.window, p.sink_tokens)
                else:
                    kept = select_n(res["psi_pool"][l, h], mask, bud, L, p.window, p.mpa_mode)
            kl.append(kept); kc.append(gather(k[l, h], kept)); vc.append(gather(v[l, h], kept))
        res["kept"].append(kl); res["k_c"].append(kc); res["v_c"].append(vc)
    return res
