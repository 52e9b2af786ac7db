"""Pins for the CPU oracle: closed forms, invariants, brute force on tiny inputs and
special cases that reduce to a textbook routine.  None of these re-type the oracle's
own formula; each is chosen so that a dropped term, a wrong sign or index or a
transposed operand in the oracle fails at least one of them.  (No GPU needed.)"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import madakv_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ Eq. 7 scores
def test_psi_hand_example_single_row():
    # One proxy row (W=1) looking at 3 keys along e1: psi is softmax(scale * a_i).
    scale = 0.5
    q = np.array([[[1.0, 0.0]]])                       # [Hq=1, W=1, d=2]
    k = np.array([[[2.0, 7.0], [-1.0, 3.0], [0.5, -4.0]]])
    z = [math.exp(scale * a) for a in (2.0, -1.0, 0.5)]
    want = np.array(z) / sum(z)
    got = O.window_scores(q, k, scale)
    assert got.shape == (1, 3)
    np.testing.assert_allclose(got[0], want, rtol=1e-14)


def test_psi_hand_example_causal_two_rows():
    # W=2, L=3: row 0 sits at position 1 and must not see key 2.
    scale = 1.0
    q = np.array([[[1.0], [2.0]]])                     # [1, 2, 1]
    k = np.array([[[0.3], [-0.2], [0.9]]])             # [1, 3, 1]
    r0 = [math.exp(0.3), math.exp(-0.2)]
    r1 = [math.exp(0.6), math.exp(-0.4), math.exp(1.8)]
    want = [r0[0] / sum(r0) + r1[0] / sum(r1), r0[1] / sum(r0) + r1[1] / sum(r1), r1[2] / sum(r1)]
    got = O.window_scores(q, k, scale)[0]
    np.testing.assert_allclose(got, want, rtol=1e-14)


@pytest.mark.parametrize("Hq,H", [(4, 4), (6, 2)])
def test_psi_rows_sum_to_one(Hq, H):
    r = rng(1)
    W, L, d = 5, 37, 8
    psi = O.window_scores(r.normal(size=(Hq, W, d)), r.normal(size=(H, L, d)), 0.3)
    np.testing.assert_allclose(psi.sum(axis=1), (Hq // H) * W, rtol=1e-12)
    assert (psi >= 0).all()


def test_psi_identical_keys_closed_form():
    r = rng(2)
    W, L, d = 4, 19, 6
    k = np.tile(r.normal(size=(1, 1, d)), (2, L, 1))
    psi = O.window_scores(r.normal(size=(2, W, d)), k, 0.7)
    want = np.array([sum(1.0 / (L - W + rr + 1) for rr in range(W) if L - W + rr >= i) for i in range(L)])
    np.testing.assert_allclose(psi[0], want, rtol=1e-12)
    np.testing.assert_allclose(psi[1], want, rtol=1e-12)


def test_psi_last_column_only_from_last_row():
    r = rng(3)
    W, L, d = 3, 11, 4
    q, k = r.normal(size=(1, W, d)), r.normal(size=(1, L, d))
    psi = O.window_scores(q, k, 0.5)[0]
    logits = 0.5 * k[0] @ q[0, W - 1]
    want = math.exp(logits[L - 1]) / sum(math.exp(x) for x in logits)
    assert psi[L - 1] == pytest.approx(want, rel=1e-12)


def test_psi_matches_textbook_masked_softmax():
    r = rng(4)
    Hq, H, W, L, d = 6, 3, 4, 29, 8
    q, k = r.normal(size=(Hq, W, d)), r.normal(size=(H, L, d))
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    kk = tk.repeat_interleave(Hq // H, dim=0)                           # query head j -> kv head j // G
    att = torch.einsum("hwd,hld->hwl", tq, kk) * 0.41
    pos = torch.arange(L)[None, :]
    row = (L - W + torch.arange(W))[:, None]
    att = att.masked_fill(pos > row, float("-inf")).softmax(dim=-1)
    want = att.sum(dim=1).reshape(H, Hq // H, L).sum(dim=1).numpy()
    np.testing.assert_allclose(O.window_scores(q, k, 0.41), want, rtol=1e-12, atol=1e-300)


def test_psi_duplicated_query_heads_scale_by_group():
    r = rng(5)
    W, L, d = 3, 17, 4
    q1, k = r.normal(size=(2, W, d)), r.normal(size=(2, L, d))
    q3 = np.repeat(q1, 3, axis=0)
    np.testing.assert_allclose(O.window_scores(q3, k, 0.5), 3 * O.window_scores(q1, k, 0.5), rtol=1e-12)


# ------------------------------------------------------------------ Eq. 6 shares
def test_share_closed_form_constant_logit_per_modality():
    # logit a on text keys, b on image keys: share_t = n_t e^a / (n_t e^a + n_v e^b),
    # whatever mass the window columns take.
    W, L, d = 4, 40, 2
    a, b, scale = 0.8, -0.3, 0.5
    mask = np.zeros(L, dtype=np.uint8); mask[5:21] = 1
    k = np.zeros((1, L, d)); k[0, :, 0] = np.where(mask == 1, b, a) / scale
    k[0, L - W:, 0] = 0.123
    q = np.zeros((1, W, d)); q[0, :, 0] = 1.0
    psi = O.window_scores(q, k, scale)
    w, kc, n = O.modality_stats(psi, mask, W, 0.9)
    n_t, n_v = L - W - 16, 16
    assert tuple(n) == (n_t, n_v)
    want = n_t * math.exp(a) / (n_t * math.exp(a) + n_v * math.exp(b))
    assert O.text_share(w[0, 0], w[0, 1], n_t, n_v) == pytest.approx(want, rel=1e-12)


def test_share_bounds_and_single_modality():
    r = rng(6)
    W, L = 4, 50
    psi = r.random((3, L))
    mask = (r.random(L) < 0.5).astype(np.uint8)
    w, _, n = O.modality_stats(psi, mask, W, 0.9)
    for h in range(3):
        s = O.text_share(w[h, 0], w[h, 1], n[0], n[1])
        assert 0.0 <= s <= 1.0
        assert s + w[h, 1] / (w[h, 0] + w[h, 1]) == pytest.approx(1.0, abs=1e-15)
    w1, _, n1 = O.modality_stats(psi, np.zeros(L, np.uint8), W, 0.9)
    assert O.text_share(w1[0, 0], w1[0, 1], n1[0], n1[1]) == 1.0
    w2, _, n2 = O.modality_stats(psi, np.ones(L, np.uint8), W, 0.9)
    assert O.text_share(w2[0, 0], w2[0, 1], n2[0], n2[1]) == 0.0
    assert O.text_share(0.0, 0.0, 3, 9) == 0.25
    # window columns are excluded from the masses
    np.testing.assert_allclose(w[:, 0] + w[:, 1], psi[:, :L - W].sum(axis=1), rtol=1e-13)


# ------------------------------------------------------------------ Eq. 9 counts
def test_theta_count_brute_force_over_subsets():
    r = rng(7)
    for trial in range(40):
        n = int(r.integers(1, 9))
        v = r.random(n) ** 3
        theta = float(r.uniform(0.05, 0.99))
        tot = v.sum()
        best = None
        for size in range(1, n + 1):
            if any(sum(c) >= theta * tot for c in itertools.combinations(v, size)):
                best = size
                break
        assert O.theta_mass_count(v, theta) == best


def test_theta_count_special_cases():
    assert O.theta_mass_count(np.ones(10), 0.5) == 5
    assert O.theta_mass_count(np.ones(8), 0.75) == 6
    assert O.theta_mass_count(np.ones(8), 0.70) == 6          # ceil(5.6)
    onehot = np.zeros(9); onehot[4] = 2.5
    assert O.theta_mass_count(onehot, 0.9) == 1
    assert O.theta_mass_count(rng(8).random(20), 1e-9) == 1
    assert O.theta_mass_count(np.zeros(5), 0.9) == 0
    assert O.theta_mass_count(np.zeros(0), 0.9) == 0
    v = rng(9).random(30)
    ks = [O.theta_mass_count(v, t) for t in np.linspace(0.01, 1.0, 34)]
    assert all(x <= y for x, y in zip(ks, ks[1:])) and ks[-1] <= 30


def test_stats_count_uses_modality_subsets():
    psi = np.array([[8.0, 1.0, 1.0, 4.0, 4.0, 1.0, 99.0]])      # last column is the window
    mask = np.array([0, 0, 0, 1, 1, 1, 0], dtype=np.uint8)
    w, kc, n = O.modality_stats(psi, mask, 1, 0.8)
    assert tuple(w[0]) == (10.0, 9.0) and tuple(n) == (3, 3)
    assert tuple(kc[0]) == (1, 2)                               # 8 >= 8 ; 4+4 >= 7.2


# ------------------------------------------------------------------ pooling
def test_pool_brute_force_and_identity():
    r = rng(10)
    psi = r.random((2, 23))
    W = 3
    np.testing.assert_array_equal(O.pool_scores(psi, W, 1), psi[:, :20])
    for pk in (3, 5, 7):
        got = O.pool_scores(psi, W, pk)
        rad = (pk - 1) // 2
        for h in range(2):
            for i in range(20):
                js = [j for j in range(20) if abs(j - i) <= rad]
                assert got[h, i] == max(psi[h, j] for j in js)
        assert (got >= psi[:, :20]).all()


# ------------------------------------------------------------------ Eq. 10-11 HCC
def _params(NL, H, L, W, budget, **kw):
    return O.Params(n_layers=NL, n_q_heads=H, n_kv_heads=H, head_dim=8, ctx_len=L, window=W, budget=budget, **kw)


def test_apportion_hamilton_properties_small():
    r = rng(11)
    for trial in range(300):
        H = int(r.integers(1, 5))
        n_c = int(r.integers(4, 30))
        dem = r.integers(1, n_c + 1, size=H)
        total = int(r.integers(0, H * n_c + 1))
        a = O.apportion(total, dem, n_c)
        assert a.sum() == total and (a >= 0).all() and (a <= n_c).all()
        D = int(dem.sum())
        if total == D:
            assert (a == dem).all(); continue
        if total < D:
            quota = [Fraction(total * int(x), D) for x in dem]
            part = a
        else:
            room = n_c - dem
            quota = [Fraction((total - D) * int(x), int(room.sum())) for x in room]
            part = a - dem
        fl = [q.numerator // q.denominator for q in quota]
        fr = [q - f for q, f in zip(quota, fl)]
        assert all(p in (f, f + 1) for p, f in zip(part, fl))
        ups = [h for h in range(H) if part[h] == fl[h] + 1]
        downs = [h for h in range(H) if part[h] == fl[h]]
        for u in ups:
            for dn in downs:       # nobody with a strictly larger remainder (or equal and lower index) was skipped
                assert fr[u] > fr[dn] or (fr[u] == fr[dn] and u < dn)


def test_hcc_conservation_bounds_and_split():
    r = rng(12)
    for trial in range(60):
        NL, H = int(r.integers(1, 7)), int(r.integers(1, 6))
        W = int(r.integers(1, 5)); L = int(r.integers(W + 8, 80))
        budget = int(r.integers(W + 1, L))
        p = _params(NL, H, L, W, budget, theta=0.9)
        n_c = L - W
        n_t = int(r.integers(0, n_c + 1)); n_v = n_c - n_t
        kc = np.stack([r.integers(0, n_t + 1, size=(NL, H)), r.integers(0, n_v + 1, size=(NL, H))], -1)
        w = r.random((NL, H, 2)).astype(np.float32)
        b = O.allocate(w, kc, np.array([n_t, n_v]), p)
        assert b.sum() == NL * H * (budget - W)
        assert (b >= 0).all() and (b[..., 0] <= n_t).all() and (b[..., 1] <= n_v).all()
        a = O.hcc_allocate(kc, p)
        assert (b.sum(-1) == a).all()


def test_hcc_fixed_point_and_uniform_mode():
    NL, H, L, W, budget = 5, 4, 100, 4, 24
    p = _params(NL, H, L, W, budget)
    kc = np.zeros((NL, H, 2), dtype=np.int64); kc[..., 0] = 12; kc[..., 1] = 8      # demand == beta everywhere
    assert (O.hcc_allocate(kc, p) == 20).all()
    kc2 = rng(13).integers(0, 40, size=(NL, H, 2))
    assert (O.hcc_allocate(kc2, _params(NL, H, L, W, budget, hcc_mode=0)) == 20).all()
    one = O.hcc_allocate(kc2[:1], _params(1, H, L, W, budget))
    assert one.sum() == H * 20


def test_hcc_sign_of_compensation_and_eq11_replay():
    NL, H, L, W, budget = 6, 4, 200, 8, 48
    beta = budget - W
    p = _params(NL, H, L, W, budget)
    base = np.zeros((NL, H, 2), dtype=np.int64); base[..., 0] = beta
    for first, sign in ((beta + 20, +1), (beta - 20, -1)):
        kc = base.copy(); kc[0, :, 0] = first
        tr = {}
        a = O.hcc_allocate(kc, p, tr)
        assert np.sign(tr["K"][0]) == sign                       # overdraft positive, saving negative
        later = a[1:].mean()
        assert (later < beta) if sign > 0 else (later > beta)    # overdraft -> later layers get less
        # Eq. 11 with K^l taken per head: phi^{l+1} = phi^l - (K^l / H) / (layers left after l)
        for l in range(NL - 1):
            want = tr["phi"][l] - (tr["K"][l] / H) / (NL - l - 1)
            assert tr["phi"][l + 1] == pytest.approx(want, rel=1e-9)
        # Eq. 10: K^l = sum_h (realised - phi^l)
        for l in range(NL):
            assert tr["K"][l] == pytest.approx(sum(float(x) - tr["phi"][l] for x in a[l]), abs=1e-9)
        assert tr["phi"][0] == beta


def test_mpa_split_rounding_and_spill():
    assert O.mpa_split(7, 1.0, 1.0, 100, 100) == (4, 3)          # 3.5 rounds half up on text
    assert O.mpa_split(10, 3.0, 1.0, 100, 100) == (8, 2)         # 7.5 -> 8
    assert O.mpa_split(10, 1.0, 3.0, 100, 100) == (3, 7)         # 2.5 -> 3
    assert O.mpa_split(10, 9.0, 1.0, 4, 100) == (4, 6)           # text short: surplus to image
    assert O.mpa_split(10, 1.0, 9.0, 100, 5) == (5, 5)           # image short: surplus to text
    assert O.mpa_split(10, 0.0, 0.0, 30, 10) == (8, 2)           # no mass: token share 0.75 -> 7.5 -> 8
    assert O.mpa_split(6, 5.0, 0.0, 10, 10) == (6, 0)
    # Eq. 8 proportionality on exact numbers
    assert O.mpa_split(100, 0.25, 0.75, 1000, 1000) == (25, 75)


# ------------------------------------------------------------------ selection
def _brute_select(score, mask, b, L, W):
    c = L - W
    keep = []
    for i in range(c):
        m = mask[i]
        ahead = sum(1 for j in range(c) if mask[j] == m and (score[j] > score[i] or (score[j] == score[i] and j < i)))
        if ahead < b[m]:
            keep.append(i)
    return keep + list(range(c, L))


def test_select_brute_force_with_ties():
    r = rng(14)
    for trial in range(60):
        W = int(r.integers(1, 4)); L = int(r.integers(W + 3, 40)); c = L - W
        mask = (r.random(L) < 0.5).astype(np.uint8)
        score = r.integers(0, 5, size=c).astype(np.float64)       # many exact ties
        n = [int((mask[:c] == m).sum()) for m in (0, 1)]
        b = [int(r.integers(0, n[0] + 1)), int(r.integers(0, n[1] + 1))]
        got = O.select(score, mask, b[0], b[1], L, W)
        assert list(got) == _brute_select(score, mask, b, L, W)
        assert (np.diff(got) > 0).all() and list(got[-W:]) == list(range(c, L))


def test_select_single_modality_is_plain_topk_and_full():
    r = rng(15)
    L, W = 33, 3; c = L - W
    score = r.random(c)
    mask = np.zeros(L, np.uint8)
    got = O.select(score, mask, 7, 0, L, W)
    want = sorted(np.argsort(-score, kind="stable")[:7].tolist()) + list(range(c, L))
    assert list(got) == want
    mask2 = (r.random(L) < 0.4).astype(np.uint8)
    got_all = O.select(score, mask2, int((mask2[:c] == 0).sum()), int((mask2[:c] == 1).sum()), L, W)
    assert list(got_all) == list(range(L))
    # modality-agnostic mode ignores the mask
    got0 = O.select(score, mask2, 5, 4, L, W, mpa_mode=0)
    assert list(got0) == sorted(np.argsort(-score, kind="stable")[:9].tolist()) + list(range(c, L))


def test_top_indices_vs_lexsort_tiny():
    r = rng(16)
    for _ in range(30):
        n = int(r.integers(1, 25))
        s = r.integers(0, 4, size=n).astype(np.float64)
        idx = np.sort(r.choice(100, size=n, replace=False))
        b = int(r.integers(0, n + 1))
        want = idx[np.lexsort((idx, -s))[:b]]
        assert list(O.top_indices(s, idx, b)) == list(want)


# ------------------------------------------------------------------ Eq. 3-5 decode
def _full_attention(q, k, v, scale):
    tq, tk, tv = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (q, k, v))
    return (torch.softmax(scale * tk @ tq, dim=0) @ tv).numpy()


def test_attend_textbook_and_degenerate_cases():
    r = rng(17)
    q, k, v = r.normal(size=8), r.normal(size=(21, 8)), r.normal(size=(21, 8))
    np.testing.assert_allclose(O.attend(q, k, v, 0.35), _full_attention(q, k, v, 0.35), rtol=1e-12)
    np.testing.assert_allclose(O.attend(q, k[:1], v[:1], 0.35), v[0], rtol=1e-15)
    same = np.tile(k[:1], (21, 1))
    np.testing.assert_allclose(O.attend(q, same, v, 0.35), v.mean(axis=0), rtol=1e-12)
    perm = r.permutation(21)
    np.testing.assert_allclose(O.attend(q, k[perm], v[perm], 0.35), O.attend(q, k, v, 0.35), rtol=1e-12, atol=1e-14)


def test_decode_append_then_attend_equals_concat_and_gqa_mapping():
    r = rng(18)
    Hq, H, d = 4, 2, 8
    kc = [r.normal(size=(5, d)), r.normal(size=(9, d))]
    vc = [r.normal(size=(5, d)), r.normal(size=(9, d))]
    q, kn, vn = r.normal(size=(Hq, d)), r.normal(size=(H, d)), r.normal(size=(H, d))
    k2, v2 = [x.copy() for x in kc], [x.copy() for x in vc]
    out = O.decode_step(q, kn, vn, k2, v2, 0.4)
    assert k2[0].shape == (6, d) and v2[1].shape == (10, d)
    for j in range(Hq):
        h = j // 2
        want = _full_attention(q[j], np.vstack([kc[h], kn[h]]), np.vstack([vc[h], vn[h]]), 0.4)
        np.testing.assert_allclose(out[j], want, rtol=1e-12)
    out2 = O.decode_step(q, None, None, k2, v2, 0.4)            # attend only: nothing appended
    assert k2[0].shape == (6, d)
    np.testing.assert_allclose(out2, out, rtol=1e-15)


# ------------------------------------------------------------------ whole eviction
def _tiny_problem(seed, NL=3, H=2, G=2, L=48, W=4, d=8):
    r = rng(seed)
    mask = np.zeros(L, np.uint8); mask[6:20] = 1; mask[26:38] = 1
    q = r.normal(size=(NL, H * G, W, d)); k = r.normal(size=(NL, H, L, d)); v = r.normal(size=(NL, H, L, d))
    return q, k, v, mask


def test_budget_at_or_above_context_keeps_everything_and_is_full_attention():
    q, k, v, mask = _tiny_problem(19)
    NL, H, L, d = k.shape
    for budget in (L, L + 7):
        p = O.Params(n_layers=NL, n_q_heads=4, n_kv_heads=H, head_dim=d, ctx_len=L, window=4, budget=budget)
        res = O.evict(q, k, v, mask, p)
        qd = rng(20).normal(size=(4, d))
        for l in range(NL):
            for h in range(H):
                assert list(res["kept"][l][h]) == list(range(L))
                np.testing.assert_array_equal(res["k_c"][l][h], k[l, h])
            out = O.decode_step(qd, None, None, res["k_c"][l], res["v_c"][l], p.scale)
            for j in range(4):
                np.testing.assert_allclose(out[j], _full_attention(qd[j], k[l, j // 2], v[l, j // 2], p.scale), rtol=1e-12)


def test_evict_end_to_end_invariants():
    q, k, v, mask = _tiny_problem(21)
    NL, H, L, d = k.shape
    p = O.Params(n_layers=NL, n_q_heads=4, n_kv_heads=H, head_dim=d, ctx_len=L, window=4, budget=16, pool_k=3)
    res = O.evict(q, k, v, mask, p)
    assert res["budgets"].sum() == NL * H * 12
    for l in range(NL):
        for h in range(H):
            kept = res["kept"][l][h]
            b_t, b_v = res["budgets"][l, h]
            assert len(kept) == b_t + b_v + 4
            assert (np.diff(kept) > 0).all()
            assert int((mask[kept[:-4]] == 0).sum()) == b_t and int((mask[kept[:-4]] == 1).sum()) == b_v
            np.testing.assert_array_equal(res["k_c"][l][h], k[l, h][kept])
            np.testing.assert_array_equal(res["v_c"][l][h], v[l, h][kept])
    # modality-agnostic + uniform mode = plain top-(budget-W) of the pooled window scores
    p0 = O.Params(n_layers=NL, n_q_heads=4, n_kv_heads=H, head_dim=d, ctx_len=L, window=4, budget=16,
                  pool_k=3, mpa_mode=0, hcc_mode=0)
    res0 = O.evict(q, k, v, mask, p0)
    for l in range(NL):
        for h in range(H):
            sp = res0["psi_pool"][l, h]
            want = sorted(np.argsort(-sp, kind="stable")[:12].tolist()) + list(range(L - 4, L))
            assert list(res0["kept"][l][h]) == want


def test_hcc_hand_worked_examples():
    """Three allocations carried out by hand (pencil arithmetic, rho = 2) from the
    reading stated in the oracle: pool R, nominal phi = R/(H*rem), demand clamp
    [ceil(phi/rho), floor(rho*phi)], layer total clamped so later layers stay
    feasible, Hamilton apportionment."""
    def run(NL, H, n_c, beta, dem):
        W = 2
        p = _params(NL, H, n_c + W, W, beta + W)
        kc = np.zeros((NL, H, 2), dtype=np.int64); kc[..., 0] = np.asarray(dem)
        return O.hcc_allocate(kc, p).tolist()
    # (1) nobody clamps the layer total.  R=48: l0 lo=4 hi=16, demands (20,18)->(16,16), A=32;
    #     R=16: l1 lo=2 hi=8, (1,20)->(2,8), A=10; R=6: last layer lo=ceil(6/4)=2,
    #     (1,5)->(2,5), D=7 > 6: floors (1,4), remainders (5,2) -> (2,4).
    assert run(3, 2, 20, 8, [[20, 18], [1, 20], [1, 5]]) == [[16, 16], [2, 8], [2, 4]]
    # (2) upper clamp of the layer total.  R=32, beta_floor=2: l0 D=32 > 32-1*2*2=28 -> A=28 -> (14,14);
    #     R=4: last layer lo=1 hi=4, (3,9)->(3,4), D=7: floors (1,2), remainders (5,2) -> (2,2).
    assert run(2, 2, 20, 8, [[20, 18], [3, 9]]) == [[14, 14], [2, 2]]
    # (3) lower clamp of the layer total.  n_c=10, R=32: l0 (1,1)->(4,4), D=8 < 32-1*2*10=12 -> A=12,
    #     head-room (6,6) -> (6,6); R=20: last layer lo=5 hi=10, (7,2)->(7,5), D=12, room (3,5) -> (10,10).
    assert run(2, 2, 10, 8, [[1, 1], [7, 2]]) == [[6, 6], [10, 10]]


# ------------------------------------------------------------------ alternative readings and baseline policies
def test_uniform_within_layer_totals():
    r = rng(30)
    NL, H, L, W, budget = 6, 5, 120, 4, 30
    kc = np.stack([r.integers(0, 60, size=(NL, H)), r.integers(0, 50, size=(NL, H))], -1)
    a1 = O.hcc_allocate(kc, _params(NL, H, L, W, budget))
    a2 = O.hcc_allocate(kc, _params(NL, H, L, W, budget, hcc_mode=2))
    assert (a1.sum(axis=1) == a2.sum(axis=1)).all()                     # same layer totals (Eq. 10-11)
    assert a2.sum() == NL * H * (budget - W)
    assert ((a2.max(axis=1) - a2.min(axis=1)) <= 1).all()               # one budget per layer (Eq. 8), spare tokens to the low heads
    assert (np.diff(a2, axis=1) <= 0).all()


def test_fixed_priority_splits():
    assert O.mpa_split(10, 1.0, 9.0, 100, 100, mpa_mode=2) == (10, 0)
    assert O.mpa_split(10, 1.0, 9.0, 4, 100, mpa_mode=2) == (4, 6)       # text first, the rest to image
    assert O.mpa_split(10, 9.0, 1.0, 100, 100, mpa_mode=3) == (0, 10)
    assert O.mpa_split(10, 9.0, 1.0, 100, 7, mpa_mode=3) == (3, 7)       # image first


def test_average_pool_brute_force():
    r = rng(31)
    psi = r.random((2, 19)); W = 3
    np.testing.assert_array_equal(O.pool_scores(psi, W, 1, pool_mode=1), psi[:, :16])
    got = O.pool_scores(psi, W, 5, pool_mode=1)
    for h in range(2):
        for i in range(16):
            js = [j for j in range(16) if abs(j - i) <= 2]
            assert got[h, i] == pytest.approx(sum(psi[h, j] for j in js) / len(js), rel=1e-14)
    np.testing.assert_allclose(O.pool_scores(np.full((1, 12), 0.25), 2, 7, pool_mode=1), 0.25, rtol=1e-15)


def test_shares_over_all_columns():
    r = rng(32)
    Hq, H, W, L, d = 4, 2, 5, 33, 8
    psi = O.window_scores(r.normal(size=(Hq, W, d)), r.normal(size=(H, L, d)), 0.4)
    mask = (r.random(L) < 0.5).astype(np.uint8); mask[L - W:] = 0
    w0, k0, n0 = O.modality_stats(psi, mask, W, 0.9, share_mode=0)
    w1, k1, n1 = O.modality_stats(psi, mask, W, 0.9, share_mode=1)
    np.testing.assert_allclose(w1.sum(axis=1), (Hq // H) * W, rtol=1e-12)   # all the mass of the proxy rows
    np.testing.assert_allclose(w1[:, 1], w0[:, 1], rtol=1e-15)             # the window is text: image mass unchanged
    np.testing.assert_allclose(w1[:, 0] - w0[:, 0], psi[:, L - W:].sum(axis=1), rtol=1e-12)
    assert (k0 == k1).all() and (n0 == n1).all()


def test_sink_recent_baseline():
    assert list(O.select_sink_recent(7, 20, 3, 4)) == [0, 1, 2, 3, 14, 15, 16, 17, 18, 19]
    assert list(O.select_sink_recent(2, 20, 3, 4)) == [0, 1, 17, 18, 19]
    assert list(O.select_sink_recent(99, 10, 2, 4)) == list(range(10))
    q, k, v, mask = _tiny_problem(33)
    NL, H, L, d = k.shape
    p = O.Params(n_layers=NL, n_q_heads=4, n_kv_heads=H, head_dim=d, ctx_len=L, window=4, budget=16, select_mode=1,
                 hcc_mode=0, sink_tokens=2)
    res = O.evict(q, k, v, mask, p)
    for l in range(NL):
        for h in range(H):
            assert list(res["kept"][l][h]) == [0, 1] + list(range(34, 48))


# ------------------------------------------------------------------ more than two modalities (Eq. 6, 8, 9 M-way)
def test_three_modality_split_hand_examples():
    assert O.mpa_split_n(10, np.array([1.0, 1.0, 2.0]), [100, 100, 100]) == [3, 2, 5]      # quotas 2.5 2.5 5: the spare token to the lower id
    assert O.mpa_split_n(10, np.array([8.0, 1.0, 1.0]), [3, 100, 100]) == [3, 6, 1]        # modality 0 short: surplus by share, ties to the lower id
    assert O.mpa_split_n(7, np.array([0.0, 0.0, 0.0]), [10, 30, 60]) == [1, 2, 4]          # no mass: token shares .1 .3 .6 -> .7 2.1 4.2, spare to 0.7
    assert O.mpa_split_n(10, np.array([1.0, 5.0, 1.0]), [4, 3, 100], mpa_mode=2) == [4, 3, 3]
    assert O.mpa_split_n(10, np.array([1.0, 5.0, 1.0]), [4, 3, 100], mpa_mode=3) == [0, 0, 10]
    assert O.mpa_split_n(9, np.array([2.0, 1.0]), [100, 100]) == list(O.mpa_split(9, 2.0, 1.0, 100, 100))


def test_m_way_split_properties():
    r = rng(40)
    for _ in range(300):
        M = int(r.integers(3, 5))
        n = r.integers(0, 40, size=M)
        a = int(r.integers(0, n.sum() + 1))
        w = r.random(M) ** 2
        if r.random() < 0.1:
            w[:] = 0.0
        b = O.mpa_split_n(a, w, n)
        assert sum(b) == a and all(0 <= b[m] <= n[m] for m in range(M))
        tot = w.sum()
        share = w / tot if tot > 0 else n / max(1, n.sum())
        if all(math.ceil(share[m] * a) <= n[m] for m in range(M)):      # nobody short of candidates: quota rule
            assert all(math.floor(share[m] * a) <= b[m] <= math.ceil(share[m] * a) for m in range(M))


def test_three_modality_stats_and_selection():
    psi = np.array([[8.0, 1.0, 6.0, 4.0, 4.0, 1.0, 3.0, 3.0, 3.0, 99.0]])          # last column is the window
    mask = np.array([0, 0, 2, 1, 1, 1, 2, 2, 2, 0], dtype=np.uint8)
    w, kc, n = O.modality_stats(psi, mask, 1, 0.8, n_modalities=3)
    assert tuple(w[0]) == (9.0, 9.0, 15.0) and tuple(n) == (2, 3, 4)
    assert tuple(kc[0]) == (1, 2, 3)                                               # 8 >= 7.2 ; 4+4 >= 7.2 ; 6+3+3 >= 12
    got = O.select_n(psi[0, :9], mask, [1, 2, 2], 10, 1)
    assert list(got) == [0, 2, 3, 4, 6, 9]
    r = rng(41)
    for _ in range(30):
        W = 2; L = int(r.integers(8, 30)); c = L - W
        m3 = r.integers(0, 3, size=L).astype(np.uint8)
        sc = r.integers(0, 4, size=c).astype(np.float64)
        nm = [int((m3[:c] == m).sum()) for m in range(3)]
        bud = [int(r.integers(0, nm[m] + 1)) for m in range(3)]
        want = [i for i in range(c) if sum(1 for j in range(c) if m3[j] == m3[i] and (sc[j] > sc[i] or (sc[j] == sc[i] and j < i))) < bud[m3[i]]]
        assert list(O.select_n(sc, m3, bud, L, W)) == want + list(range(c, L))


def test_three_modality_eviction_invariants():
    r = rng(42)
    NL, H, G, L, W, d = 3, 2, 2, 60, 4, 8
    mask = np.zeros(L, np.uint8); mask[5:20] = 1; mask[25:45] = 2
    q = r.normal(size=(NL, H * G, W, d)); k = r.normal(size=(NL, H, L, d)); v = r.normal(size=(NL, H, L, d))
    p = O.Params(n_layers=NL, n_q_heads=H * G, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=20, n_modalities=3)
    res = O.evict(q, k, v, mask, p)
    assert res["budgets"].shape == (NL, H, 3) and res["budgets"].sum() == NL * H * 16
    for l in range(NL):
        for h in range(H):
            kept = res["kept"][l][h]
            for m in range(3):
                assert int((mask[kept[:-W]] == m).sum()) == res["budgets"][l, h, m]
            sh = res["w"][l, h] / res["w"][l, h].sum()
            assert abs(sh.sum() - 1.0) < 1e-12 and (sh >= 0).all()


def test_row_lse_and_scores_from_it():
    r = rng(50)
    Hq, H, W, L, d = 4, 2, 3, 21, 8
    q, k = r.normal(size=(Hq, W, d)), r.normal(size=(H, L, d))
    lse = O.proxy_row_lse(q, k, 0.37)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k).repeat_interleave(2, dim=0)
    att = torch.einsum("hwd,hld->hwl", tq, tk) * 0.37
    pos = torch.arange(L)[None, :]; row = (L - W + torch.arange(W))[:, None]
    want = torch.logsumexp(att.masked_fill(pos > row, float("-inf")), dim=-1).numpy()
    np.testing.assert_allclose(lse, want, rtol=1e-13)
    np.testing.assert_allclose(O.window_scores_from_lse(q, k, lse, 0.37), O.window_scores(q, k, 0.37), rtol=1e-12)
    # a normaliser that is off by log 2 halves that row's contribution
    lse2 = lse.copy(); lse2[:, :] += math.log(2.0)
    np.testing.assert_allclose(O.window_scores_from_lse(q, k, lse2, 0.37), 0.5 * O.window_scores(q, k, 0.37), rtol=1e-12)


# ------------------------------------------------------------------ 8-bit reduced cache encoding
def test_e4m3_table_and_quantiser():
    t = O.e4m3_decode_table()
    assert t[0x38] == 1.0 and t[0x7E] == 448.0 and t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6 and np.isnan(t[0x7F])
    fin = np.array([c for c in range(256) if (c & 0x7F) != 0x7F])
    assert (np.diff(t[fin[fin < 0x80]]) > 0).all()                                   # codes order like values
    np.testing.assert_array_equal(O.quantize_e4m3(t[fin]) & 0x7F, fin & 0x7F)        # every code is its own nearest
    # the library format of the same name, wherever it does not overflow to NaN
    allbf = torch.arange(0, 65536, dtype=torch.int32).to(torch.int16).view(torch.bfloat16).float()
    ok = torch.isfinite(allbf) & (allbf.abs() <= 448.0)
    want = allbf[ok].to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = O.quantize_e4m3(allbf[ok].numpy())
    nz = (want & 0x7F) != 0                                                          # sign of zero results aside
    np.testing.assert_array_equal(got[nz], want[nz])
    assert ((got[~nz] & 0x7F) == 0).all()
    # ties to even, subnormals, saturation
    assert O.quantize_e4m3(np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 464.0, 1e9, -1e9])).tolist() == \
        [0x38, 0x3A, 0x00, 0x02, 0x7E, 0x7E, 0xFE]
    np.testing.assert_array_equal(O.dequantize_e4m3(np.array([0x38, 0xB8, 0x7E], dtype=np.uint8)), [1.0, -1.0, 448.0])


def test_split_products_on_a_half_go_up_to_text():
    """Eq. 8 in integers, hand-worked: share_t * a exactly on x.5 rounds up (to text)."""
    for wt, wv, a, bt in [(1.0, 1.0, 7, 4), (3.0, 1.0, 6, 5), (1.0, 3.0, 6, 2), (0.25, 0.75, 1002, 251), (5.0, 3.0, 4, 3)]:
        assert O.mpa_split(a, wt, wv, a, a) == (bt, a - bt)


# ---- re-eviction during generation (an extension: the paper evicts once) -------------------------
def test_reevict_head_reduces_to_the_prompt_eviction_and_to_the_identity():
    """On a cache that still holds the whole prompt, with the prompt's own proxy queries and uniform head
    totals, re-eviction is the prompt eviction (whose pieces are pinned above); with nothing appended
    and the total it already has, a head keeps every row."""
    r = rng(21)
    NL, H, G, L, W, d = 1, 3, 2, 60, 4, 8
    q = r.standard_normal((NL, H * G, W, d)); k = r.standard_normal((NL, H, L, d)); v = r.standard_normal((NL, H, L, d))
    mask = (r.random(L) < 0.5).astype(np.uint8); mask[-W:] = 0
    p = O.Params(n_layers=NL, n_q_heads=H * G, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=20, pool_k=3, hcc_mode=0)
    res = O.evict(q, k, v, mask, p)
    for h in range(H):
        sel, bud, w, n_mod, psi, pool = O.reevict_head(q[0, h * G:(h + 1) * G], k[0, h], v[0, h], np.arange(L), mask, 20 - W, p)
        np.testing.assert_array_equal(sel, res["kept"][0][h])
        assert list(bud) == list(res["budgets"][0, h])
        np.testing.assert_allclose(psi, res["psi"][0, h], rtol=0, atol=0)
        # the reduced cache itself, nothing appended: all of it stays
        kept = res["kept"][0][h]
        sel2, bud2, *_ = O.reevict_head(q[0, h * G:(h + 1) * G], k[0, h][kept], v[0, h][kept], kept, mask, len(kept) - W, p)
        np.testing.assert_array_equal(sel2, np.arange(len(kept)))
        assert sum(bud2) == len(kept) - W


def test_reevict_head_hand_example_generated_tokens_are_text():
    """Identical keys: every proxy row spreads its attention evenly over the rows it sees, so all
    candidates score alike, masses are proportional to counts and ties go to the lower rows."""
    L, W, d = 100, 2, 4
    mask = np.zeros(L, dtype=np.uint8); mask[10:60] = 1
    p = O.Params(n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=d, ctx_len=L, window=W, budget=8)
    # cache: prompt positions 0 (text), 12, 13, 20 (image), 70 (text), then the old window 98, 99, then 3 generated tokens
    origin = np.array([0, 12, 13, 20, 70, 98, 99, L + 0, L + 1, L + 2])
    n = len(origin)
    kr = np.ones((n, d)); vr = np.arange(n * d, dtype=np.float64).reshape(n, d)
    qr = np.ones((1, W, d))
    sel, bud, w, n_mod, psi, pool = O.reevict_head(qr, kr, vr, origin, mask, 5, p)
    # candidates: rows 0..7 = text {0, 4, 5, 6, 7} (the generated row 7 is text), image {1, 2, 3}
    assert list(n_mod) == [5, 3]
    np.testing.assert_allclose(psi[:8], 1.0 / 9 + 1.0 / 10)                # both proxy rows see rows 0..7
    np.testing.assert_allclose(w, [5 * psi[0], 3 * psi[0]])
    assert bud == [3, 2]                                                   # floor(5/8 * 5 + 0.5) = 3
    np.testing.assert_array_equal(sel, [0, 1, 2, 4, 5, 8, 9])              # lowest rows of each modality, then the proxies


def test_window_attention_textbook_and_consistency_with_the_scores():
    """The last-window prefill attention against a library masked softmax attention in fp64, its last
    row against plain Eq. 5 over the whole prompt, its log-sum-exp against proxy_row_lse, and its
    softmax rows against Eq. 7: psi is their column sum."""
    r = rng(31)
    Hq, H, L, W, d = 6, 3, 40, 5, 8
    q = r.standard_normal((Hq, W, d)); k = r.standard_normal((H, L, d)); v = r.standard_normal((H, L, d))
    scale = 0.3
    out, lse = O.window_attention(q, k, v, scale)
    G = Hq // H
    qt, kt, vt = torch.from_numpy(q), torch.from_numpy(k).repeat_interleave(G, 0), torch.from_numpy(v).repeat_interleave(G, 0)
    logits = scale * torch.einsum("jwd,jld->jwl", qt, kt)
    pos = torch.arange(L)[None, None, :]; rowpos = (L - W + torch.arange(W))[None, :, None]
    logits = logits.masked_fill(pos > rowpos, float("-inf"))
    ref = torch.softmax(logits, -1) @ vt
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(logits, -1).numpy(), rtol=1e-12)
    np.testing.assert_allclose(lse, O.proxy_row_lse(q, k, scale), rtol=1e-12)
    for j in range(Hq):
        np.testing.assert_allclose(out[j, W - 1], O.attend(q[j, W - 1], k[j // G], v[j // G], scale), rtol=1e-12, atol=1e-13)
    psi = torch.softmax(logits, -1).reshape(H, G * W, L).sum(1).numpy()
    np.testing.assert_allclose(O.window_scores(q, k, scale), psi, rtol=1e-12, atol=1e-15)
    # identical keys: every row is the mean of the values it sees
    out1, _ = O.window_attention(q, np.ones((H, L, d)), v, scale)
    for rr in range(W):
        np.testing.assert_allclose(out1[0, rr], v[0, :L - W + rr + 1].mean(0), rtol=1e-12)
