"""The rules of the free-running GPU-vs-oracle comparison, exercised on the CPU: the oracle's own
results must pass with nothing to excuse, and mistakes planted in a copy of them must be caught."""
import numpy as np
import pytest

from oracle import madakv_oracle as O
from tests import parity_utils as PU


def problem(seed=3, NL=3, H=3, G=2, L=96, W=4, d=8, budget=24):
    r = np.random.default_rng(seed)
    q = r.standard_normal((NL, H * G, W, d)); k = r.standard_normal((NL, H, L, d)); v = r.standard_normal((NL, H, L, d))
    mask = (r.random(L) < 0.6).astype(np.uint8); mask[-W:] = 0
    p = O.Params(n_layers=NL, n_q_heads=H * G, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=budget, pool_k=3)
    return p, mask, O.evict(q, k, v, mask, p)


def run(p, mask, res, w=None, kc=None, bud=None, kept=None):
    w = res["w"].astype(np.float32) if w is None else w
    kc = res["kcnt"] if kc is None else kc
    bud = res["budgets"] if bud is None else bud
    kept = res["kept"] if kept is None else kept
    return PU.free_running_check(p, res, mask, w, kc, res["n_mod"], bud, lambda l, h: kept[l][h])


def test_oracle_against_itself_has_nothing_to_excuse():
    p, mask, res = problem()
    cnt = run(p, mask, res)
    assert cnt == dict(k_excused=0, budget_excused=0, budget_unexcused=0, kept_excused=0, kept_unexcused=0, heads=9)


def test_a_moved_token_between_modalities_is_caught():
    p, mask, res = problem()
    bud = res["budgets"].copy()
    l, h = 1, 2
    assert bud[l, h, 0] > 0
    bud[l, h, 0] -= 1; bud[l, h, 1] += 1
    # the allocation replayed on the same statistics no longer gives these budgets
    with pytest.raises(AssertionError):
        run(p, mask, res, bud=bud)


def test_a_wrong_kept_position_is_caught():
    p, mask, res = problem()
    kept = [[x.copy() for x in row] for row in res["kept"]]
    nc = p.ctx_len - p.window
    psi = res["psi_pool"][0, 0]
    dropped = [i for i in range(nc) if i not in set(kept[0][0].tolist())]
    worst = min(dropped, key=lambda i: psi[i])                 # a clearly worse candidate of the same modality
    m = mask[worst]
    best_kept = max((i for i in kept[0][0][:-p.window] if mask[i] == m), key=lambda i: psi[i])
    kept[0][0] = np.sort(np.array([worst if i == best_kept else i for i in kept[0][0]]))
    cnt = run(p, mask, res, kept=kept)
    assert cnt["kept_unexcused"] >= 1


def test_a_count_off_a_crossing_is_caught_and_one_on_a_crossing_is_excused():
    p, mask, res = problem()
    kc = res["kcnt"].copy()
    kc[0, 0, 1] += 3                                           # nowhere near the theta crossing
    with pytest.raises(AssertionError):
        run(p, mask, res, kc=kc, bud=O.allocate(res["w"], kc, res["n_mod"], p))
    # a count on the crossing: make the (k+1)-th value of a modality negligible, so that k and k+1
    # both reach theta * w within 1e-4
    vals = np.array([0.5, 0.3, 0.1, 1e-9, 0.1])
    k0 = O.theta_mass_count(vals, 0.9)
    assert PU.k_count_ok(k0, vals, 0.9) and not PU.k_count_ok(k0 + 2, vals, 0.9)
    assert PU.k_count_ok(4, np.array([0.5, 0.3, 0.1, 1e-9, 0.1 - 1e-9]), 0.9)   # 0.9 reached at 3 up to 1e-9


def test_split_boundary_rule():
    assert PU.split_on_rounding_boundary(1.0, 1.0, 100, 100, 7)          # 3.5 + 0.5 is an integer
    assert not PU.split_on_rounding_boundary(1.0, 2.0, 100, 100, 7)      # 2.33 + 0.5
