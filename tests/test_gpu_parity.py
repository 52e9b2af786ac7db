"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Sizes span several tiles and ragged tails but stay small enough for the
oracle to finish in seconds.  Stage-isolated checks feed both sides the same upstream
values; the free-running check runs the whole path and applies the near-tie rules."""
import sys

import numpy as np
import pytest
import torch

from oracle import madakv_oracle as O
from paper_2506_15724_amd import binding as MB
from paper_2506_15724_amd import workloads as WL
from tests import parity_utils as PU

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _four_layer_groups(monkeypatch):
    """The library pipelines a call over several layers in as many layer groups as leave a group 256 heads: one for
    the small shapes here.  The tests of this file ask for four, so that the pipelined path (two streams, events,
    per-group workspaces) is what they run; test_fused_eviction_call_matches_the_three_calls also runs the default."""
    monkeypatch.setenv("MADAKV_LAYER_GROUPS", "4")


def say(msg):
    print(f"[parity] {msg}", flush=True)
    sys.stdout.flush()


def small_workloads():
    C = WL.CONFIGS
    return {
        "tiny_fp32": C["tiny"],
        "bf16_mha": C["llava_layer"].scaled(name="bf16_mha", n_layers=3, batch=2, n_q_heads=4, n_kv_heads=4,
                                            ctx_len=2000, budget=300, n_images=2, decode_steps=3),
        "bf16_gqa7": C["qwen_gqa"].scaled(name="bf16_gqa7", n_layers=2, batch=1, n_q_heads=14, n_kv_heads=2,
                                          ctx_len=1500, budget=200, image_tokens=(64, 300), text_tokens=(16, 128),
                                          decode_steps=2),
        "bf16_w64": C["long_128k"].scaled(name="bf16_w64", n_layers=1, batch=1, n_q_heads=3, n_kv_heads=3,
                                          ctx_len=3000, budget=256, n_images=3, decode_steps=2),
        "bf16_d64_gqa2": C["llava_layer"].scaled(name="bf16_d64_gqa2", n_layers=2, batch=1, n_q_heads=4, n_kv_heads=2,
                                                 head_dim=64, ctx_len=1200, budget=150, n_images=1, window=16,
                                                 decode_steps=2),
        # odd lengths: candidate rows start at unaligned addresses (scalar load paths, ragged tiles)
        "bf16_odd": C["llava_layer"].scaled(name="bf16_odd", n_layers=2, batch=2, n_q_heads=6, n_kv_heads=3,
                                            ctx_len=1501, window=17, budget=211, n_images=1, pool_k=5, decode_steps=2),
        "fp32_d128": C["tiny"].scaled(name="fp32_d128", n_layers=2, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128,
                                      ctx_len=700, window=8, budget=100, pool_k=3, fixed_layout=(), n_images=2,
                                      image_tokens=(100, 100), text_tokens=(20, 200), decode_steps=2),
    }


def engine(wl, **kw):
    args = dict(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                head_dim=wl.head_dim, ctx_len=wl.ctx_len, window=wl.window, budget=wl.budget, dtype=wl.dtype,
                pool_k=wl.pool_k, max_new_tokens=wl.decode_steps, out_fp32=1, device=DEV)
    args.update(kw)
    return MB.MadaKV(**args)


def stats_struct(w, k, device):
    """[..., 4] int32 tensor holding {f32 w_t, f32 w_v, i32 k_t, i32 k_v}."""
    wf = torch.from_numpy(np.asarray(w, dtype=np.float32)).view(torch.int32)
    ki = torch.from_numpy(np.asarray(k, dtype=np.int32))
    return torch.cat([wf, ki], dim=-1).contiguous().to(device)


@pytest.mark.parametrize("name", list(small_workloads().keys()))
def test_stagewise_parity(name):
    wl = small_workloads()[name]
    NL, B, H, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window, wl.head_dim
    G, nc = wl.n_q_heads // H, L - W
    p = PU.oracle_params(wl)
    say(f"{name}: inputs")
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    say(f"{name}: madakv_score")
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    psi_g = eng.psi.cpu().numpy()
    pool_g = eng.psi_pool.cpu().numpy()
    w_g, k_g = eng.stats_host()
    nmod_g = eng.n_mod.cpu().numpy()

    # ---- S1: psi against the oracle
    qh, kh, vh = WL.to_f64(q), WL.to_f64(k), WL.to_f64(v)
    psi_o = np.stack([np.stack([O.window_scores(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    nbad, worst = PU.psi_close(psi_g, psi_o, G, W, L)
    say(f"{name}: psi worst scaled error {worst:.2e}")
    assert nbad == 0, f"psi: {nbad} entries outside tolerance (worst {worst})"
    np.testing.assert_allclose(psi_g.sum(-1), G * W, rtol=2e-4)

    # ---- S2: statistics and pooling, both sides reading the GPU's psi bits
    for l in range(NL):
        for b in range(B):
            psi_in = psi_g[l, b].astype(np.float64)
            w_o, k_o, n_o = O.modality_stats(psi_in, masks[b], W, p.theta)
            assert tuple(nmod_g[b]) == tuple(n_o)
            PU.assert_masses_close(w_g[l, b], w_o, L)
            np.testing.assert_array_equal(pool_g[l, b], O.pool_scores(psi_in, W, p.pool_k).astype(np.float32))
            for h in range(H):
                for m in (0, 1):
                    if k_g[l, b, h, m] != k_o[h, m]:
                        vals = psi_in[h, :nc][masks[b][:nc] == m]
                        assert PU.k_count_ok(int(k_g[l, b, h, m]), vals, p.theta), (l, b, h, m, k_g[l, b, h, m], k_o[h, m])

    # ---- S3: allocation, fed the GPU's own statistics on both sides: bit-exact
    say(f"{name}: madakv_allocate")
    eng.allocate(0, NL)
    torch.cuda.synchronize()
    bud_g = eng.budgets.cpu().numpy()
    for b in range(B):
        bud_o = O.allocate(w_g[:, b], k_g[:, b].astype(np.int64), nmod_g[b], p)
        np.testing.assert_array_equal(bud_g[:, b], bud_o)
    assert bud_g.sum() == NL * B * H * (wl.budget - W)

    # ---- S4 + S5: selection and gather, both sides reading the GPU's pooled scores and budgets
    say(f"{name}: madakv_select_gather")
    eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    kv_off, kv_len = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    kept_all = eng.kept_idx.cpu().numpy()
    kc_all, vc_all = eng.k_c.cpu(), eng.v_c.cpu()
    cap_b = eng.capacity // B
    for b in range(B):
        cursor = b * cap_b
        for l in range(NL):
            for h in range(H):
                bt, bv = (int(x) for x in bud_g[l, b, h])
                assert kv_len[l, b, h] == bt + bv + W
                assert kv_off[l, b, h] == cursor, "segments must tile the batch item's region"
                cursor += kv_len[l, b, h] + wl.decode_steps
                kept_o = O.select(pool_g[l, b, h].astype(np.float64), masks[b], bt, bv, L, W)
                o = kv_off[l, b, h]
                kept = kept_all[o:o + kv_len[l, b, h]]
                np.testing.assert_array_equal(kept, kept_o)
                assert torch.equal(kc_all[o:o + len(kept)], k[l, b, h].cpu()[kept_o])
                assert torch.equal(vc_all[o:o + len(kept)], v[l, b, h].cpu()[kept_o])

    # ---- S6: decode steps (append + attend), fp32 output against the fp64 oracle
    k_cache = [[[WL.to_f64(kc_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]]) for h in range(H)]
                for b in range(B)] for l in range(NL)]
    v_cache = [[[WL.to_f64(vc_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]]) for h in range(H)]
                for b in range(B)] for l in range(NL)]
    out = torch.empty(NL, B, wl.n_q_heads, d, dtype=torch.float32, device=DEV)
    for step in range(wl.decode_steps):
        dq, dk, dv = [], [], []
        for l in range(NL):
            row = [WL.decode_inputs(wl, l, b, step, DEV) for b in range(B)]
            dq.append(torch.stack([r[0] for r in row])); dk.append(torch.stack([r[1] for r in row]))
            dv.append(torch.stack([r[2] for r in row]))
        dq, dk, dv = torch.stack(dq).contiguous(), torch.stack(dk).contiguous(), torch.stack(dv).contiguous()
        say(f"{name}: madakv_decode_attn step {step}")
        if step % 2 == 0:
            eng.decode_attn(0, NL, dq, dk, dv, out)              # all layers in one call
        else:
            for l in range(NL):                                  # one call per layer (split-KV path)
                eng.decode_attn(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out[l:l + 1])
        torch.cuda.synchronize()
        out_g = out.cpu().numpy()
        for l in range(NL):
            for b in range(B):
                ref = O.decode_step(WL.to_f64(dq[l, b]), WL.to_f64(dk[l, b]), WL.to_f64(dv[l, b]),
                                    k_cache[l][b], v_cache[l][b], p.scale)
                err = np.abs(out_g[l, b] - ref).max()
                assert err <= PU.DECODE_ATOL, (step, l, b, err)
        assert (eng.kv_len.cpu().numpy() == kv_len + step + 1).all()
    # the appended rows are in the cache
    kc2 = eng.k_c.cpu()
    for l in range(NL):
        for b in range(B):
            for h in range(H):
                o = kv_off[l, b, h]
                got = WL.to_f64(kc2[o:o + kv_len[l, b, h] + wl.decode_steps])
                np.testing.assert_array_equal(got, k_cache[l][b][h])
    # beyond the slack the library refuses
    with pytest.raises(MB.MadaKVError) as ei:
        eng.decode_attn(0, NL, dq, dk, dv, out)
    assert ei.value.status == -1
    eng.decode_attn(0, NL, dq, None, None, out)                 # attend-only is still fine
    torch.cuda.synchronize()
    eng.close()


@pytest.mark.parametrize("name", ["tiny_fp32", "bf16_mha", "bf16_gqa7"])
def test_free_running_end_to_end(name):
    """Whole path on the GPU against the whole oracle, with the near-tie rules."""
    wl = small_workloads()[name]
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    nc = L - W
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    say(f"{name}: full eviction")
    eng.score(0, NL, q, k, mask)
    eng.allocate(0, NL)
    eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    bud_g = eng.budgets.cpu().numpy()
    kv_off, kv_len = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    kept_all = eng.kept_idx.cpu().numpy()
    w_g, k_g = eng.stats_host()
    nmod_g = eng.n_mod.cpu().numpy()
    qh, kh, vh = WL.to_f64(q), WL.to_f64(k), WL.to_f64(v)
    tot = {}
    for b in range(B):
        res = O.evict(qh[:, b], kh[:, b], vh[:, b], masks[b], p)
        cnt = PU.free_running_check(p, res, masks[b], w_g[:, b], k_g[:, b], nmod_g[b], bud_g[:, b],
                                    lambda l, h: kept_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]], say)
        for key, val in cnt.items():
            tot[key] = tot.get(key, 0) + val
    say(f"{name}: {tot}")
    assert tot["budget_unexcused"] == 0 and tot["kept_unexcused"] == 0, tot
    assert bud_g.sum() == NL * B * H * (wl.budget - W)
    eng.close()


def test_budget_at_or_above_context_is_full_attention():
    wl = small_workloads()["bf16_mha"].scaled(budget=2000, n_layers=1, batch=1, decode_steps=1)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    say("keep-all: select_gather without scores")
    MB.madakv_select_gather(eng.h, 0, 1, None, mask, None, k, v, eng.kept_idx, eng.kv_off, eng.kv_len, eng.k_c,
                            eng.v_c, eng.select_ws)
    torch.cuda.synchronize()
    H, L, d = wl.n_kv_heads, wl.ctx_len, wl.head_dim
    assert (eng.kv_len.cpu().numpy() == L).all()
    kept = eng.kept_idx.cpu().numpy()
    off = eng.kv_off.cpu().numpy()
    for h in range(H):
        np.testing.assert_array_equal(kept[off[0, 0, h]:off[0, 0, h] + L], np.arange(L))
        assert torch.equal(eng.k_c[off[0, 0, h]:off[0, 0, h] + L], k[0, 0, h])
    dq, _, _ = WL.decode_inputs(wl, 0, 0, 0, DEV)
    out = torch.empty(1, 1, wl.n_q_heads, d, dtype=torch.float32, device=DEV)
    eng.decode_attn(0, 1, dq[None, None].contiguous(), None, None, out)
    torch.cuda.synchronize()
    p = PU.oracle_params(wl)
    kh, vh = WL.to_f64(k), WL.to_f64(v)
    for j in range(wl.n_q_heads):
        ref = O.attend(WL.to_f64(dq[j]), kh[0, 0, j], vh[0, 0, j], p.scale)     # Eq. 5 over the whole prompt
        assert np.abs(out[0, 0, j].cpu().numpy() - ref).max() <= PU.DECODE_ATOL
    eng.close()


def test_layer_by_layer_calls_match_one_call_and_runs_repeat_bitwise():
    wl = small_workloads()["bf16_mha"]
    NL = wl.n_layers
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    outs = []
    for mode in ("all", "per_layer", "all"):
        eng = engine(wl, layers_per_call=NL if mode == "all" else 1)
        if mode == "all":
            eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
        else:
            for l in range(NL):
                eng.score(l, 1, q[l:l + 1], k[l:l + 1], mask)
                eng.allocate(l, 1)
                eng.select_gather(l, 1, k[l:l + 1], v[l:l + 1], mask)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (eng.psi, eng.psi_pool, eng.stats, eng.budgets, eng.kv_off, eng.kv_len)]
                    + [eng.kept_idx.clone(), eng.k_c.clone()])
        eng.close()
    lens, offs = outs[0][5].cpu().numpy(), outs[0][4].cpu().numpy()
    for other in outs[1:]:
        for a, b in zip(outs[0][:6], other[:6]):
            assert torch.equal(a, b)
        for l in range(NL):
            for b in range(wl.batch):
                for h in range(wl.n_kv_heads):
                    o, n = offs[l, b, h], lens[l, b, h]
                    assert torch.equal(outs[0][6][o:o + n], other[6][o:o + n])
                    assert torch.equal(outs[0][7][o:o + n], other[7][o:o + n])


def test_ablation_modes_match_oracle():
    wl = small_workloads()["bf16_mha"]
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    for mpa, hcc in ((0, 1), (1, 0), (0, 0)):
        p = PU.oracle_params(wl, mpa_mode=mpa, hcc_mode=hcc)
        eng = engine(wl, mpa_mode=mpa, hcc_mode=hcc)
        say(f"ablation mpa={mpa} hcc={hcc}")
        eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
        torch.cuda.synchronize()
        w_g, k_g = eng.stats_host()
        bud_g, pool_g = eng.budgets.cpu().numpy(), eng.psi_pool.cpu().numpy()
        kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
        for b in range(B):
            np.testing.assert_array_equal(bud_g[:, b], O.allocate(w_g[:, b], k_g[:, b].astype(np.int64),
                                                                 eng.n_mod.cpu().numpy()[b], p))
            for l in range(NL):
                for h in range(H):
                    bt, bv = (int(x) for x in bud_g[l, b, h])
                    ref = O.select(pool_g[l, b, h].astype(np.float64), masks[b], bt, bv, L, W, mpa)
                    np.testing.assert_array_equal(kept_all[off[l, b, h]:off[l, b, h] + ln[l, b, h]], ref)
        if hcc == 0:
            assert (bud_g.sum(-1) == wl.budget - W).all()
        eng.close()


def test_allocate_random_statistics_bit_exact():
    """madakv_allocate alone on random statistics (forces every clamp branch), vs the oracle."""
    r = np.random.default_rng(5)
    for trial in range(12):
        NL, B, H = int(r.integers(1, 9)), int(r.integers(1, 4)), int(r.integers(1, 33))
        W = int(r.integers(1, 9)); L = int(r.integers(W + 40, 600))
        budget = int(r.integers(W + 1, L))
        nc = L - W
        theta = 0.9
        eng = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=H, n_kv_heads=H, head_dim=64, ctx_len=L, window=W,
                        budget=budget, dtype="bf16", pool_k=1, hcc_rho=int(r.integers(1, 4)), device=DEV)
        p = O.Params(n_layers=NL, n_q_heads=H, n_kv_heads=H, head_dim=64, ctx_len=L, window=W, budget=budget,
                     hcc_rho=eng.cfg.hcc_rho, theta=theta)
        n_t = r.integers(0, nc + 1, size=B); n_v = nc - n_t
        skew = r.choice([0.05, 1.0, 3.0])
        kt = (r.random((NL, B, H)) ** skew * (n_t[None, :, None] + 1)).astype(np.int64).clip(0, n_t[None, :, None])
        kv_ = (r.random((NL, B, H)) ** skew * (n_v[None, :, None] + 1)).astype(np.int64).clip(0, n_v[None, :, None])
        kc = np.stack([kt, kv_], -1)
        w = r.random((NL, B, H, 2)).astype(np.float32)
        w[r.random((NL, B, H)) < 0.1] = 0.0
        n_mod = np.stack([n_t, n_v], -1).astype(np.int32)
        st = stats_struct(w, kc, DEV)
        nm = torch.from_numpy(n_mod).to(DEV)
        # in two calls when there are enough layers: the pool is carried in the handle
        cut = NL // 2
        if cut:
            eng.allocate(0, cut, st[:cut], nm, eng.budgets[:cut])
            eng.allocate(cut, NL - cut, st[cut:], nm, eng.budgets[cut:])
        else:
            eng.allocate(0, NL, st, nm, eng.budgets)
        torch.cuda.synchronize()
        got = eng.budgets.cpu().numpy()
        for b in range(B):
            np.testing.assert_array_equal(got[:, b], O.allocate(w[:, b], kc[:, b], n_mod[b], p))
        eng.close()


def test_select_with_heavy_ties_and_extreme_budgets():
    """Scores with few distinct values (pooling makes exact ties), budgets 0 and n_m."""
    r = np.random.default_rng(9)
    # budget 1600 per head: the six hand-made budgets below add up to less than the 6 * 1603 rows
    # the reduced cache holds (the library lays segments out in that space)
    wl = small_workloads()["bf16_mha"].scaled(n_layers=1, batch=1, n_q_heads=6, n_kv_heads=6, ctx_len=5000,
                                              n_images=3, budget=1600)
    H, L, W = wl.n_kv_heads, wl.ctx_len, wl.window
    nc = L - W
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    m = masks[0]
    n_t, n_v = int((m[:nc] == 0).sum()), int((m[:nc] == 1).sum())
    pool = r.integers(0, 6, size=(1, 1, H, nc)).astype(np.float32) * 0.25
    pool[0, 0, 1] = 1.0                                            # one value only
    pool[0, 0, 2] = -pool[0, 0, 2]                                 # negative scores order correctly too
    bud = np.array([[[[0, 0], [n_t, n_v], [7, 0], [0, 9], [n_t - 1, 1], [123, 456]]]], dtype=np.int32)
    bud[0, 0, 5] = [min(123, n_t), min(456, n_v)]
    assert int(bud.sum()) + H * (W + wl.decode_steps) <= eng.capacity
    pool_t, bud_t = torch.from_numpy(pool).to(DEV), torch.from_numpy(bud).to(DEV)
    say("select: ties and extreme budgets")
    eng.select_gather(0, 1, k, v, mask, psi_pool=pool_t, budgets=bud_t)
    torch.cuda.synchronize()
    kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    for h in range(H):
        ref = O.select(pool[0, 0, h].astype(np.float64), m, int(bud[0, 0, h, 0]), int(bud[0, 0, h, 1]), L, W)
        np.testing.assert_array_equal(kept_all[off[0, 0, h]:off[0, 0, h] + ln[0, 0, h]], ref)
    eng.close()


def test_bf16_output_rounding():
    wl = small_workloads()["bf16_mha"].scaled(n_layers=1, batch=1, decode_steps=1)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    res = {}
    for of in (1, 0):
        eng = engine(wl, out_fp32=of)
        eng.score(0, 1, q, k, mask); eng.allocate(0, 1); eng.select_gather(0, 1, k, v, mask)
        dq, dk, dv = WL.decode_inputs(wl, 0, 0, 0, DEV)
        out = torch.empty(1, 1, wl.n_q_heads, wl.head_dim, dtype=torch.float32 if of else torch.bfloat16, device=DEV)
        eng.decode_attn(0, 1, dq[None, None].contiguous(), dk[None, None].contiguous(), dv[None, None].contiguous(), out)
        torch.cuda.synchronize()
        res[of] = out.float().cpu()
        eng.close()
    assert torch.equal(res[0], res[1].to(torch.bfloat16).float())   # the bf16 output is the RNE of the fp32 one


def test_budgets_beyond_the_cache_leave_heads_empty():
    """Budgets that add up to more than the reduced cache holds: the library lays out what
    fits and gives the remaining heads empty segments; nothing is written out of bounds."""
    wl = small_workloads()["bf16_mha"].scaled(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=4, ctx_len=2000, budget=300,
                                              decode_steps=1)
    H, L, W = wl.n_kv_heads, wl.ctx_len, wl.window
    nc = L - W
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    m = masks[0]
    n_t, n_v = int((m[:nc] == 0).sum()), int((m[:nc] == 1).sum())
    cap = eng.capacity                                             # 4 * 301 rows
    guard_i = torch.full_like(eng.kept_idx, -7)
    eng.kept_idx.copy_(guard_i)
    eng.k_c.fill_(123.0)
    bud = np.array([[[[100, 100], [min(n_t, 700), min(n_v, 700)], [5, 5], [1, 1]]]], dtype=np.int32)   # head 1 cannot fit
    pool = np.random.default_rng(3).random((1, 1, H, nc)).astype(np.float32)
    say("select: budgets larger than the cache")
    eng.select_gather(0, 1, k, v, mask, psi_pool=torch.from_numpy(pool).to(DEV), budgets=torch.from_numpy(bud).to(DEV))
    torch.cuda.synchronize()
    ln, off = eng.kv_len.cpu().numpy()[0, 0], eng.kv_off.cpu().numpy()[0, 0]
    assert list(ln) == [200 + W, 0, 0, 0]
    assert off[0] == 0 and (off[1:] == 200 + W + 1).all()
    kept = eng.kept_idx.cpu().numpy()
    np.testing.assert_array_equal(kept[:ln[0]], O.select(pool[0, 0, 0].astype(np.float64), m, 100, 100, L, W))
    assert (kept[ln[0]:] == -7).all()
    assert (eng.k_c[ln[0]:].float() == 123.0).all()
    # decode on it: the full head works, the empty heads stay empty and append nothing
    dq, dk, dv = WL.decode_inputs(wl, 0, 0, 0, DEV)
    out = torch.empty(1, 1, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device=DEV)
    eng.decode_attn(0, 1, dq[None, None].contiguous(), dk[None, None].contiguous(), dv[None, None].contiguous(), out)
    torch.cuda.synchronize()
    assert list(eng.kv_len.cpu().numpy()[0, 0]) == [200 + W + 1, 0, 0, 0]
    assert torch.isfinite(out[0, 0, 0]).all()
    assert (eng.k_c[ln[0] + 1:].float() == 123.0).all()
    eng.close()


VARIANTS = {
    "heads_share_layer_total": dict(hcc_mode=2),
    "text_first": dict(mpa_mode=2),
    "image_first": dict(mpa_mode=3),
    "average_pool": dict(pool_mode=1, pool_k=5),
    "shares_over_all_columns": dict(share_mode=1),
    "sink_recent": dict(select_mode=1, sink_tokens=4),
    "sink_recent_uniform": dict(select_mode=1, sink_tokens=9, hcc_mode=0, mpa_mode=0),
}


@pytest.mark.parametrize("variant,shape", [(v, "small") for v in VARIANTS] +
                         [(v, "long") for v in ("text_first", "average_pool", "shares_over_all_columns")])
def test_alternative_readings_and_baselines(variant, shape):
    """The switchable readings / baseline policies, stage by stage against their oracle branch.  shape "long": heads of
    four 16384-candidate chunks, where statistics and selection run chunk-parallel."""
    kw = VARIANTS[variant]
    wl = small_workloads()["bf16_mha"]
    if shape == "long":
        wl = wl.scaled(name="bf16_long_ctx", n_layers=2, batch=1, n_q_heads=2, n_kv_heads=2, ctx_len=50001, budget=3000,
                       n_images=3, decode_steps=1)
    if "pool_k" in kw:
        wl = wl.scaled(pool_k=kw["pool_k"])
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    nc = L - W
    okw = {k: v for k, v in kw.items() if k != "pool_k"}
    p = PU.oracle_params(wl, **okw)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, **okw)
    say(f"variant {variant}")
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    psi_g, pool_g = eng.psi.cpu().numpy(), eng.psi_pool.cpu().numpy()
    w_g, k_g = eng.stats_host()
    nmod = eng.n_mod.cpu().numpy()
    bud_g = eng.budgets.cpu().numpy()
    kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    for b in range(B):
        for l in range(NL):
            psi_in = psi_g[l, b].astype(np.float64)
            w_o, k_o, _ = O.modality_stats(psi_in, masks[b], W, p.theta, p.share_mode)
            PU.assert_masses_close(w_g[l, b], w_o, L)
            pool_o = O.pool_scores(psi_in, W, p.pool_k, p.pool_mode)
            if p.pool_mode == 0:
                np.testing.assert_array_equal(pool_g[l, b], pool_o.astype(np.float32))
            else:
                np.testing.assert_allclose(pool_g[l, b], pool_o, rtol=2e-6, atol=1e-30)
            for h in range(H):
                for m in (0, 1):
                    if k_g[l, b, h, m] != k_o[h, m]:
                        assert PU.k_count_ok(int(k_g[l, b, h, m]), psi_in[h, :nc][masks[b][:nc] == m], p.theta)
        np.testing.assert_array_equal(bud_g[:, b], O.allocate(w_g[:, b], k_g[:, b].astype(np.int64), nmod[b], p))
        for l in range(NL):
            for h in range(H):
                bt, bv = (int(x) for x in bud_g[l, b, h])
                if p.select_mode == 1:
                    ref = O.select_sink_recent(bt + bv, L, W, p.sink_tokens)
                else:
                    ref = O.select(pool_g[l, b, h].astype(np.float64), masks[b], bt, bv, L, W, p.mpa_mode)
                o = off[l, b, h]
                np.testing.assert_array_equal(kept_all[o:o + ln[l, b, h]], ref)
                assert torch.equal(eng.k_c[o:o + len(ref)].cpu(), k[l, b, h].cpu()[ref])
    assert bud_g.sum() == NL * B * H * (wl.budget - W)
    if variant == "heads_share_layer_total":
        tot = bud_g.sum(-1)
        assert ((tot.max(-1) - tot.min(-1)) <= 1).all()
    eng.close()


@pytest.mark.parametrize("M,mpa,long_ctx", [(3, 1, 0), (4, 1, 0), (3, 2, 0), (3, 0, 0), (4, 3, 0), (3, 1, 1), (4, 1, 1)])
def test_more_than_two_modalities(M, mpa, long_ctx):
    """Eq. 6, 8, 9 and the selection with M modalities, stage by stage against the oracle.  long_ctx: heads of four
    16384-candidate chunks (chunk-parallel statistics and selection, the 4-modality build of those kernels)."""
    wl = small_workloads()["bf16_mha"].scaled(name=f"bf16_m{M}", n_images=5, ctx_len=4100, budget=500, n_modalities=M)
    if long_ctx:
        wl = wl.scaled(name=f"bf16_m{M}_long", n_layers=1, batch=1, n_q_heads=2, n_kv_heads=2, ctx_len=50001, budget=3000,
                       n_images=6, decode_steps=1)
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    nc = L - W
    p = PU.oracle_params(wl, n_modalities=M, mpa_mode=mpa)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    assert int(mask.max()) == M - 1
    eng = engine(wl, n_modalities=M, mpa_mode=mpa)
    say(f"{M} modalities, mpa_mode {mpa}")
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    psi_g, pool_g = eng.psi.cpu().numpy(), eng.psi_pool.cpu().numpy()
    w_g, k_g = eng.stats_host()
    assert w_g.shape[-1] == M and k_g.shape[-1] == M
    nmod = eng.n_mod.cpu().numpy()
    bud_g = eng.budgets.cpu().numpy()
    kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    for b in range(B):
        for l in range(NL):
            psi_in = psi_g[l, b].astype(np.float64)
            w_o, k_o, n_o = O.modality_stats(psi_in, masks[b], W, p.theta, 0, M)
            assert tuple(nmod[b]) == tuple(n_o)
            PU.assert_masses_close(w_g[l, b], w_o, L)
            np.testing.assert_array_equal(pool_g[l, b], O.pool_scores(psi_in, W, p.pool_k).astype(np.float32))
            for h in range(H):
                for m in range(M):
                    if k_g[l, b, h, m] != k_o[h, m]:
                        assert PU.k_count_ok(int(k_g[l, b, h, m]), psi_in[h, :nc][masks[b][:nc] == m], p.theta)
        np.testing.assert_array_equal(bud_g[:, b], O.allocate(w_g[:, b], k_g[:, b].astype(np.int64), nmod[b], p))
        for l in range(NL):
            for h in range(H):
                bud = [int(x) for x in bud_g[l, b, h]]
                assert ln[l, b, h] == sum(bud) + W
                ref = O.select_n(pool_g[l, b, h].astype(np.float64), masks[b], bud, L, W, mpa)
                o = off[l, b, h]
                np.testing.assert_array_equal(kept_all[o:o + ln[l, b, h]], ref)
                assert torch.equal(eng.k_c[o:o + len(ref)].cpu(), k[l, b, h].cpu()[ref])
                assert torch.equal(eng.v_c[o:o + len(ref)].cpu(), v[l, b, h].cpu()[ref])
    assert bud_g.sum() == NL * B * H * (wl.budget - W)
    eng.close()


def test_allocate_random_statistics_three_and_four_modalities():
    """madakv_allocate alone on random M-way statistics (every branch of the split), vs the oracle."""
    r = np.random.default_rng(6)
    for trial in range(16):
        M = 3 + trial % 2
        NL, B, H = int(r.integers(1, 6)), int(r.integers(1, 3)), int(r.integers(1, 20))
        W = int(r.integers(1, 9)); L = int(r.integers(W + 60, 500))
        budget = int(r.integers(W + 1, L)); nc = L - W
        eng = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=H, n_kv_heads=H, head_dim=64, ctx_len=L, window=W,
                        budget=budget, dtype="bf16", pool_k=1, n_modalities=M, device=DEV)
        p = O.Params(n_layers=NL, n_q_heads=H, n_kv_heads=H, head_dim=64, ctx_len=L, window=W, budget=budget, n_modalities=M)
        cuts = np.sort(r.integers(0, nc + 1, size=(B, M - 1)), axis=1)
        n_mod = np.diff(np.concatenate([np.zeros((B, 1), int), cuts, np.full((B, 1), nc)], axis=1), axis=1).astype(np.int32)
        kc = (r.random((NL, B, H, M)) ** r.choice([0.2, 1.0, 3.0]) * (n_mod[None, :, None, :] + 1)).astype(np.int64)
        kc = np.minimum(kc, n_mod[None, :, None, :])
        w = r.random((NL, B, H, M)).astype(np.float32)
        w[r.random((NL, B, H)) < 0.1] = 0.0
        w[r.random((NL, B, H, M)) < 0.15] = 0.0
        st = stats_struct(w, kc, DEV)
        eng.allocate(0, NL, st, torch.from_numpy(n_mod).to(DEV), eng.budgets)
        torch.cuda.synchronize()
        got = eng.budgets.cpu().numpy()
        for b in range(B):
            np.testing.assert_array_equal(got[:, b], O.allocate(w[:, b], kc[:, b], n_mod[b], p))
        eng.close()


def _split3_with_fused_multiply_add(w, a):
    """The three-way Eq. 8 split as it comes out when share * a - floor is formed from the exact
    product (what a fused multiply-add does): used to show that a case sits on a knife edge."""
    import math
    from fractions import Fraction
    tot = 0.0
    for x in w:
        tot += float(x)
    share = [float(x) / tot for x in w]
    b = [math.floor(s_ * a) for s_ in share]
    frac = [float(Fraction(share[m]) * a - b[m]) for m in range(3)]
    for m in sorted(range(3), key=lambda m: (-frac[m], m))[:a - sum(b)]:
        b[m] += 1
    return b


def test_allocate_rounds_after_every_operation():
    """Eq. 8 on knife edges: masses whose quotas have nearly equal fractional parts, so that the
    split depends on the product share * a being rounded before the floor is subtracted (a fused
    multiply-add would hand the spare token to another modality), and two-modality products that
    land exactly on .5 (rounded half up).  Head totals are forced with hcc_mode = 0."""
    cases3 = [([2.25, 9.75, 3.0], 836), ([38.0, 18.0, 34.0], 1818), ([13.5, 12.5, 1.5], 1845), ([18.0, 15.0, 69.0], 1748),
              ([2.0, 4.0, 30.0], 171), ([20.0, 28.0, 3.0], 4530), ([10.5, 7.5, 16.0], 3488), ([7.5, 1.5, 6.0], 4985),
              ([8.5, 10.0, 14.5], 968)]
    W = 4
    for w, a in cases3:
        n_mod = np.array([[a, a, a]], dtype=np.int32)
        L = 3 * a + W
        eng = MB.MadaKV(n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, ctx_len=L, window=W, budget=a + W,
                        dtype="bf16", pool_k=1, hcc_mode=0, n_modalities=3, device=DEV)
        p = O.Params(n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=64, ctx_len=L, window=W, budget=a + W, hcc_mode=0,
                     n_modalities=3)
        wa = np.array(w, dtype=np.float32).reshape(1, 1, 1, 3)
        kc = np.ones((1, 1, 1, 3), dtype=np.int64)
        eng.allocate(0, 1, stats_struct(wa, kc, DEV), torch.from_numpy(n_mod).to(DEV), eng.budgets)
        torch.cuda.synchronize()
        want = O.allocate(wa[:, 0], kc[:, 0], n_mod[0], p)[0, 0]
        assert list(want) != _split3_with_fused_multiply_add(w, a), "not a knife edge any more"
        np.testing.assert_array_equal(eng.budgets.cpu().numpy()[0, 0, 0], want)
        eng.close()
    for wt, wv, a, bt in [(1.0, 1.0, 7, 4), (3.0, 1.0, 6, 5), (1.0, 3.0, 6, 2), (0.25, 0.75, 1002, 251), (5.0, 3.0, 4, 3)]:
        L = 2 * a + W
        eng = MB.MadaKV(n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, ctx_len=L, window=W, budget=a + W,
                        dtype="bf16", pool_k=1, hcc_mode=0, device=DEV)
        p = O.Params(n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=64, ctx_len=L, window=W, budget=a + W, hcc_mode=0)
        wa = np.array([wt, wv], dtype=np.float32).reshape(1, 1, 1, 2)
        kc = np.ones((1, 1, 1, 2), dtype=np.int64)
        n_mod = np.array([[a, a]], dtype=np.int32)
        eng.allocate(0, 1, stats_struct(wa, kc, DEV), torch.from_numpy(n_mod).to(DEV), eng.budgets)
        torch.cuda.synchronize()
        got = eng.budgets.cpu().numpy()[0, 0, 0]
        assert tuple(got) == (bt, a - bt), (wt, wv, a, got)          # the product is exactly x.5: half goes up, to text
        np.testing.assert_array_equal(got, O.allocate(wa[:, 0], kc[:, 0], n_mod[0], p)[0, 0])
        eng.close()


def _one_sweep_workloads():
    W = small_workloads()
    out = {n: W[n] for n in ("bf16_mha", "bf16_w64", "bf16_d64_gqa2", "bf16_odd")}
    # 69 chunks of 1024 keys per head: the row statistics travel in two levels (groups of 16 chunks)
    out["bf16_70k"] = W["bf16_mha"].scaled(name="bf16_70k", n_layers=1, batch=1, n_q_heads=2, n_kv_heads=2, ctx_len=70001,
                                           budget=500, n_images=3)
    # 75 chunks of 768 keys per head (64 proxy rows): six heads fit the chip's workgroup slots, one chunk per head in the
    # way of a seventh, so the last two chunks of every head run ahead, parked (their words at the group level)
    out["bf16_w64_57k"] = W["bf16_w64"].scaled(name="bf16_w64_57k", n_layers=1, batch=1, n_q_heads=2, n_kv_heads=2, ctx_len=57001,
                                               budget=600, n_images=20)
    # ... and 80 chunks of 1024 keys (32 rows): seven parked
    out["bf16_81k"] = W["bf16_mha"].scaled(name="bf16_81k", n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, ctx_len=81001,
                                           budget=500, n_images=30)
    return out


@pytest.mark.parametrize("name", list(_one_sweep_workloads().keys()))
def test_one_sweep_scoring_and_its_lone_workgroup_path(name):
    """Scoring in one sweep over K: the workgroups of a head exchange their row statistics through
    memory and wait for each other, with a bounded wait.  In a normal run nobody gives up (the
    counter in the first word of the workspace stays 0).  With the wait cut to a single poll from
    the host, workgroups that find a word missing compute the head's statistics on their own: every
    kernel still ends normally and the scores still match the oracle."""
    import os
    wl = _one_sweep_workloads()[name]
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    G = wl.n_q_heads // H
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    qh, kh = WL.to_f64(q), WL.to_f64(k)
    psi_o = np.stack([np.stack([O.window_scores(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    eng = engine(wl)
    eng.score_ws.zero_()
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    assert int(eng.score_ws[:4].view(torch.int32)[0]) == 0, "a workgroup gave up waiting in an ordinary run"
    psi_1 = eng.psi.clone()
    nbad, worst = PU.psi_close(psi_1.cpu().numpy(), psi_o, G, W, L)
    assert nbad == 0, worst
    os.environ["MADAKV_SCORE_SPIN_LIMIT"] = "1"
    try:
        say(f"{name}: scoring with the wait cut to one poll")
        eng.score(0, NL, q, k, mask)
        torch.cuda.synchronize()
    finally:
        del os.environ["MADAKV_SCORE_SPIN_LIMIT"]
    lone = int(eng.score_ws[:4].view(torch.int32)[0])
    say(f"{name}: {lone} workgroups went their own way")
    nbad, worst = PU.psi_close(eng.psi.cpu().numpy(), psi_o, G, W, L)
    assert nbad == 0, worst
    np.testing.assert_allclose(eng.psi.sum(-1).cpu().numpy(), G * W, rtol=2e-4)
    # and the ordinary run repeats bit for bit
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    assert torch.equal(eng.psi, psi_1)
    eng.close()


def _logical_rows(eng, cache, l, b, h, length, P):
    """Rows 0..length-1 of a head of the paged cache, read back through the page table."""
    tbl = eng.page_table_host()[l, b, h]
    off = int(eng.kv_off[l, b, h])
    init = int(tbl[0]) * P
    idx = [off + r if r < init else int(tbl[1 + (r - init) // P]) * P + (r - init) % P for r in range(length)]
    return cache[torch.tensor(idx, device=cache.device)]


@pytest.mark.parametrize("name,P,fp8", [("bf16_mha", 16, 0), ("bf16_gqa7", 32, 0), ("bf16_odd", 16, 0), ("bf16_mha", 64, 1),
                                        ("fp32_d128", 16, 0)])
def test_paged_reduced_cache(name, P, fp8):
    """page_rows > 0: kept rows in whole pages, appended rows in pages taken on demand.  The eviction
    gives the same kept positions and rows as with contiguous segments; many decode steps, crossing
    page boundaries in every head, give bit for bit the outputs of the contiguous cache and match the
    oracle; the rows read back through the page table are the kept rows followed by the appended ones."""
    steps = 2 * P + 5
    wl = small_workloads()[name].scaled(decode_steps=steps)
    NL, B, H, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window, wl.head_dim
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    flat, paged = engine(wl, cache_fp8=fp8), engine(wl, cache_fp8=fp8, page_rows=P)
    for eng in (flat, paged):
        eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    assert torch.equal(flat.budgets, paged.budgets) and torch.equal(flat.kv_len, paged.kv_len)
    len0 = paged.kv_len.cpu().numpy()
    off_f, off_p = flat.kv_off.cpu().numpy(), paged.kv_off.cpu().numpy()
    tbl = paged.page_table_host()
    cap_b = paged.capacity // B
    for b in range(B):
        cursor = b * cap_b
        for l in range(NL):
            for h in range(H):
                n = int(len0[l, b, h])
                assert off_p[l, b, h] == cursor and off_p[l, b, h] % P == 0 and tbl[l, b, h, 0] == -(-n // P)
                cursor += -(-n // P) * P
                assert torch.equal(paged.kept_idx[off_p[l, b, h]:off_p[l, b, h] + n], flat.kept_idx[off_f[l, b, h]:off_f[l, b, h] + n])
                assert torch.equal(paged.k_c[off_p[l, b, h]:off_p[l, b, h] + n], flat.k_c[off_f[l, b, h]:off_f[l, b, h] + n])
                assert torch.equal(paged.v_c[off_p[l, b, h]:off_p[l, b, h] + n], flat.v_c[off_f[l, b, h]:off_f[l, b, h] + n])
    # the oracle's copy of two sampled heads' caches (decoded values for the 8-bit cache)
    dec = (lambda t: O.dequantize_e4m3(t.cpu().numpy())) if fp8 else WL.to_f64
    samples = sorted({(0, 0, 0), (NL - 1, B - 1, H - 1)})
    caches = {s: [dec(flat.k_c[off_f[s]:off_f[s] + int(len0[s])]), dec(flat.v_c[off_f[s]:off_f[s] + int(len0[s])])] for s in samples}
    out_f = torch.empty(NL, B, wl.n_q_heads, d, dtype=torch.float32, device=DEV)
    out_p = torch.empty_like(out_f)
    G = wl.n_q_heads // H
    quant = (lambda x: O.dequantize_e4m3(O.quantize_e4m3(x))) if fp8 else (lambda x: x)
    for step in range(steps):
        dq, dk, dv = WL.decode_inputs_all(wl, step, DEV)
        for eng, out in ((flat, out_f), (paged, out_p)):
            if step % 3 == 0:
                eng.decode_attn(0, NL, dq, dk, dv, out)
            else:
                for l in range(NL):
                    eng.decode_attn(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out[l:l + 1])
        torch.cuda.synchronize()
        assert torch.equal(out_f, out_p), f"paged and contiguous caches differ at step {step}"
        for (l, b, h) in samples:
            kc, vc = caches[(l, b, h)]
            kc = np.concatenate([kc, quant(WL.to_f64(dk[l, b, h]))[None]]); vc = np.concatenate([vc, quant(WL.to_f64(dv[l, b, h]))[None]])
            caches[(l, b, h)] = [kc, vc]
            if step in (0, P, steps - 1):
                for g in range(G):
                    ref = O.attend(WL.to_f64(dq[l, b, h * G + g]), kc, vc, p.scale)
                    assert np.abs(out_p[l, b, h * G + g].cpu().numpy() - ref).max() <= PU.DECODE_ATOL
    assert (paged.kv_len.cpu().numpy() == len0 + steps).all()
    # every head took the pages its appended rows needed, all different, all inside its batch item's region
    tbl = paged.page_table_host()
    for b in range(B):
        taken = []
        for l in range(NL):
            for h in range(H):
                n0 = int(len0[l, b, h]); init = int(tbl[l, b, h, 0])
                extra = max(0, -(-(n0 + steps - init * P) // P))
                taken += [int(x) for x in tbl[l, b, h, 1:1 + extra]]
        assert len(set(taken)) == len(taken)
        assert all(b * cap_b // P <= x < (b + 1) * cap_b // P for x in taken)
    for (l, b, h) in samples:
        n = int(len0[l, b, h]) + steps
        np.testing.assert_array_equal(dec(_logical_rows(paged, paged.k_c, l, b, h, n, P)), caches[(l, b, h)][0])
        np.testing.assert_array_equal(dec(_logical_rows(paged, paged.v_c, l, b, h, n, P)), caches[(l, b, h)][1])
    # a new pass hands every page back
    paged.select_gather(0, NL, k, v, mask)
    dq, dk, dv = WL.decode_inputs_all(wl, 0, DEV)
    paged.decode_attn(0, NL, dq, dk, dv, out_p)
    flat.select_gather(0, NL, k, v, mask)
    flat.decode_attn(0, NL, dq, dk, dv, out_f)
    torch.cuda.synchronize()
    assert torch.equal(out_f, out_p)
    with pytest.raises(MB.MadaKVError):
        MB.MadaKV(n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, ctx_len=100, window=4, budget=20, page_rows=24, device=DEV)
    flat.close(); paged.close()


@pytest.mark.parametrize("name,fp8", [("bf16_mha", 0), ("bf16_w64", 0), ("bf16_d64_gqa2", 0), ("bf16_odd", 0), ("bf16_gqa7", 0),
                                      ("bf16_mha", 1), ("bf16_d64_gqa2", 1), ("bf16_gqa7", 1)])
def test_reeviction_during_generation(name, fp8):
    """madakv_reevict after some decode steps, twice: every head is brought back to the length the prompt
    eviction gave it.  Stage by stage against the oracle on the GPU's own upstream values (scores within
    the psi tolerance, then masses 2e-6, budgets / surviving rows / moved K, V rows / original positions
    bit for bit), and decode afterwards against Eq. 5 over the oracle's copy of the new cache.
    fp8: the reduced cache holds E4M3 rows; the oracle works on the values those bytes stand for."""
    import os
    rounds = (5, 3)
    wl = small_workloads()[name].scaled(decode_steps=max(rounds))
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    G = Hq // H
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, cache_fp8=fp8)
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    off = eng.kv_off.cpu().numpy()
    len0 = eng.kv_len.cpu().numpy().copy()
    cap = eng.capacity
    # what cached rows stand for (float64), and what a new row becomes once it is in the cache
    cached = (lambda t: O.dequantize_e4m3(t.cpu().numpy())) if fp8 else WL.to_f64
    as_cached = (lambda t: O.dequantize_e4m3(O.quantize_e4m3(WL.to_f64(t)))) if fp8 else WL.to_f64
    # the oracle's view of every head: rows (float64), original positions
    heads = [(l, b, h) for l in range(NL) for b in range(B) for h in range(H)]
    rows_k = {s: cached(eng.k_c[off[s]:off[s] + len0[s]]) for s in heads}
    rows_v = {s: cached(eng.v_c[off[s]:off[s] + len0[s]]) for s in heads}
    origin = {s: eng.kept_idx[off[s]:off[s] + len0[s]].cpu().numpy().astype(np.int64) for s in heads}
    q_hist = [q[:, :, :, r] for r in range(W)]                 # queries of the tokens in the last W rows, oldest first
    out = torch.empty(NL, B, Hq, d, dtype=torch.float32, device=DEV)
    gen = 0
    step = 0
    for T in rounds:
        for _ in range(T):
            dq, dk, dv = WL.decode_inputs_all(wl, step, DEV)
            eng.decode_attn(0, NL, dq, dk, dv, out)
            torch.cuda.synchronize()
            for s in heads:
                l, b, h = s
                rows_k[s] = np.concatenate([rows_k[s], as_cached(dk[l, b, h])[None]])
                rows_v[s] = np.concatenate([rows_v[s], as_cached(dv[l, b, h])[None]])
                origin[s] = np.concatenate([origin[s], [L + gen]])
            for (l, b, h) in heads[::5]:
                for g in range(G):
                    ref = O.attend(WL.to_f64(dq[l, b, h * G + g]), rows_k[(l, b, h)], rows_v[(l, b, h)], p.scale)
                    assert np.abs(out[l, b, h * G + g].cpu().numpy() - ref).max() <= PU.DECODE_ATOL
            q_hist.append(dq); q_hist = q_hist[-W:]
            gen += 1; step += 1
        q_recent = torch.stack(q_hist, dim=3).contiguous()     # [NL, B, Hq, W, d]
        say(f"{name}: madakv_reevict after {T} more steps")
        eng.reevict_ws = None
        lone = fp8 and T == rounds[-1]          # once with the scoring kernel's wait cut to one poll: its own-way path on E4M3 rows
        if lone:
            os.environ["MADAKV_SCORE_SPIN_LIMIT"] = "1"
        try:
            eng.reevict(0, NL, q_recent, mask)
            torch.cuda.synchronize()
        finally:
            if lone:
                del os.environ["MADAKV_SCORE_SPIN_LIMIT"]
        ws = eng.reevict_ws
        psi_g = ws[:cap * 4].view(torch.float32).cpu().numpy()
        up = lambda x: (x + 255) // 256 * 256
        stats_at = 3 * up(cap * 4) + up(cap)
        M = 2
        rec = ws[stats_at:stats_at + NL * B * H * 8 * M].view(torch.int32).reshape(NL, B, H, 2 * M).cpu()
        w_g = rec[..., :M].contiguous().view(torch.float32).numpy(); n_g = rec[..., M:].numpy()
        bud_g = eng.budgets.cpu().numpy()
        new_len = eng.kv_len.cpu().numpy()
        assert (new_len == len0).all(), "every head is back at the length the prompt eviction gave it"
        kept_all = eng.kept_idx.cpu().numpy()
        for s in heads:
            l, b, h = s
            n = rows_k[s].shape[0]
            qh = WL.to_f64(q_recent[l, b, h * G:(h + 1) * G])
            sel_o, bud_o, w_o, n_o, psi_o, pool_o = O.reevict_head(qh, rows_k[s], rows_v[s], origin[s], masks[b], int(len0[s]) - W, p)
            pg = psi_g[off[s]:off[s] + n]
            nbad, worst = PU.psi_close(pg, psi_o, G, W, n)
            assert nbad == 0, (s, worst)
            # from here on both sides read the GPU's scores
            rowmod = np.where(origin[s] < L, masks[b][np.minimum(origin[s], L - 1)], 0)
            w_r, n_r = O.modality_mass(pg.astype(np.float64), rowmod, W, M)
            assert tuple(n_g[s]) == tuple(n_r)
            PU.assert_masses_close(w_g[s], w_r, len(pg))
            bud_r = O.mpa_split_n(int(len0[s]) - W, w_g[s].astype(np.float64), n_r, p.mpa_mode)
            assert list(bud_g[s]) == list(bud_r)
            pool_r = O.pool_scores(pg.astype(np.float64)[None], W, p.pool_k)[0].astype(np.float32).astype(np.float64)
            sel_r = O.select_n(pool_r, rowmod, bud_r, n, W, p.mpa_mode)
            got_k = cached(eng.k_c[off[s]:off[s] + len0[s]]); got_v = cached(eng.v_c[off[s]:off[s] + len0[s]])
            np.testing.assert_array_equal(got_k, rows_k[s][sel_r])
            np.testing.assert_array_equal(got_v, rows_v[s][sel_r])
            np.testing.assert_array_equal(kept_all[off[s]:off[s] + len0[s]], origin[s][sel_r])
            rows_k[s], rows_v[s], origin[s] = rows_k[s][sel_r], rows_v[s][sel_r], origin[s][sel_r]
    # generation goes on over the re-evicted cache
    dq, dk, dv = WL.decode_inputs_all(wl, step, DEV)
    eng.decode_attn(0, NL, dq, dk, dv, out)
    torch.cuda.synchronize()
    for (l, b, h) in heads:
        kc = np.concatenate([rows_k[(l, b, h)], as_cached(dk[l, b, h])[None]]); vc = np.concatenate([rows_v[(l, b, h)], as_cached(dv[l, b, h])[None]])
        for g in range(G):
            ref = O.attend(WL.to_f64(dq[l, b, h * G + g]), kc, vc, p.scale)
            assert np.abs(out[l, b, h * G + g].cpu().numpy() - ref).max() <= PU.DECODE_ATOL
    eng.close()


@pytest.mark.parametrize("name,P,fp8", [("bf16_mha", 16, 0), ("bf16_gqa7", 16, 0), ("bf16_odd", 16, 1)])
def test_reeviction_on_a_paged_cache(name, P, fp8):
    """madakv_reevict with page_rows > 0, twice, next to the same steps on contiguous segments (which
    test_reeviction_during_generation checks stage by stage against the oracle): the same budgets, lengths,
    surviving rows and original positions bit for bit, the survivors back in the heads' initial pages, and the
    same decode outputs afterwards for more steps than the page pools hold without the pages handed back."""
    rounds = (21, 9)                    # (every head fills its last initial page and one or two later pages)
    wl = small_workloads()[name].scaled(decode_steps=max(rounds))
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    flat, paged = engine(wl, cache_fp8=fp8), engine(wl, cache_fp8=fp8, page_rows=P)
    for eng in (flat, paged):
        eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    len0 = flat.kv_len.cpu().numpy().copy()
    off_f, off_p = flat.kv_off.cpu().numpy(), paged.kv_off.cpu().numpy()
    q_hist = [q[:, :, :, r] for r in range(W)]
    out_f = torch.empty(NL, B, Hq, d, dtype=torch.float32, device=DEV)
    out_p = torch.empty_like(out_f)
    step = 0

    def decode_both():
        nonlocal step, q_hist
        dq, dk, dv = WL.decode_inputs_all(wl, step, DEV)
        flat.decode_attn(0, NL, dq, dk, dv, out_f)
        paged.decode_attn(0, NL, dq, dk, dv, out_p)
        torch.cuda.synchronize()
        assert torch.equal(out_f, out_p), f"paged and contiguous caches differ at step {step}"
        q_hist.append(dq); q_hist = q_hist[-W:]
        step += 1

    for T in rounds:
        for _ in range(T):
            decode_both()
        q_recent = torch.stack(q_hist, dim=3).contiguous()
        say(f"{name}: madakv_reevict on both caches after {T} more steps")
        for eng in (flat, paged):
            eng.reevict_ws = None
            eng.reevict(0, NL, q_recent, mask)
        torch.cuda.synchronize()
        assert torch.equal(flat.kv_len, paged.kv_len) and (paged.kv_len.cpu().numpy() == len0).all()
        assert torch.equal(flat.budgets, paged.budgets)
        for l in range(NL):
            for b in range(B):
                for h in range(H):
                    n, of, op = int(len0[l, b, h]), int(off_f[l, b, h]), int(off_p[l, b, h])
                    assert torch.equal(paged.k_c[op:op + n], flat.k_c[of:of + n]) and torch.equal(paged.v_c[op:op + n], flat.v_c[of:of + n])
                    assert torch.equal(paged.kept_idx[op:op + n], flat.kept_idx[of:of + n])
    # generation goes on: five more steps would not fit the pools if the pages of the rounds above were still taken
    for _ in range(max(rounds)):
        decode_both()
    tbl = paged.page_table_host()
    cap_b = paged.capacity // B
    for b in range(B):
        taken = []
        for l in range(NL):
            for h in range(H):
                n0 = int(len0[l, b, h]); init = int(tbl[l, b, h, 0])
                extra = max(0, -(-(n0 + max(rounds) - init * P) // P))
                taken += [int(x) for x in tbl[l, b, h, 1:1 + extra]]
        assert len(set(taken)) == len(taken)
        assert all(b * cap_b // P <= x < (b + 1) * cap_b // P for x in taken)
    flat.close(); paged.close()


def test_reeviction_refusals():
    wl = small_workloads()["bf16_mha"].scaled(n_layers=1, batch=1, decode_steps=2)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    qr = q.clone()
    for kw, status in ((dict(budget=wl.ctx_len), -3),):
        eng = engine(wl, **kw)
        eng.reevict_ws = torch.empty(MB.madakv_reevict_workspace_bytes(eng.h, 1), dtype=torch.uint8, device=DEV)
        with pytest.raises(MB.MadaKVError) as ei:
            eng.reevict(0, 1, qr, mask)
        assert ei.value.status == status
        eng.close()
    # a paged cache is re-evicted as a whole (the pages it hands back belong to pools that all layers share)
    wl2 = wl.scaled(n_layers=2)
    eng = engine(wl2, page_rows=16)
    eng.reevict_ws = torch.empty(MB.madakv_reevict_workspace_bytes(eng.h, 2), dtype=torch.uint8, device=DEV)
    with pytest.raises(MB.MadaKVError) as ei:
        eng.reevict(1, 1, qr, mask)
    assert ei.value.status == -1
    eng.close()
    f32 = small_workloads()["tiny_fp32"]
    eng = engine(f32)
    eng.reevict_ws = torch.empty(MB.madakv_reevict_workspace_bytes(eng.h, 1), dtype=torch.uint8, device=DEV)
    with pytest.raises(MB.MadaKVError) as ei:
        eng.reevict(0, 1, torch.zeros(1, 1, 8, 16, 64, device=DEV), torch.zeros(1, 1024, dtype=torch.uint8, device=DEV))
    assert ei.value.status == -7
    eng.close()


def _window_workloads():
    W = small_workloads()
    # (the last three: more than 32 proxy rows, taken in blocks of 32: 224 = 7 blocks, 64 = 2, 2 x 20 = a ragged second block)
    return {"bf16_mha": W["bf16_mha"], "bf16_d64_gqa2": W["bf16_d64_gqa2"],
            "bf16_w20_odd": W["bf16_mha"].scaled(name="bf16_w20_odd", ctx_len=1777, window=20, budget=222, n_layers=2, batch=1),
            "bf16_gqa7": W["bf16_gqa7"], "bf16_w64": W["bf16_w64"],
            # 79 chunks per head: the row statistics travel in two levels
            "bf16_40k": W["bf16_mha"].scaled(name="bf16_40k", ctx_len=40001, budget=600, n_layers=1, batch=1, n_q_heads=2, n_kv_heads=2, n_images=20),
            # both at once: two blocks of proxy rows, 66 chunks per head
            "bf16_w64_34k": W["bf16_w64"].scaled(name="bf16_w64_34k", ctx_len=33555, budget=500, n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, n_images=16),
            "bf16_gqa2_w20": W["bf16_mha"].scaled(name="bf16_gqa2_w20", ctx_len=1777, window=20, budget=222, n_layers=2, batch=1,
                                                  n_q_heads=4, n_kv_heads=2)}


@pytest.mark.parametrize("name", list(_window_workloads().keys()))
@pytest.mark.parametrize("fp32_out", [1, 0])
def test_window_attention_with_scores(name, fp32_out):
    """madakv_window_attn_score: the prefill attention of the last W positions (Eq. 5) and, from the same
    pass, Eq. 7 / 6 / 9 as madakv_score gives them.  out and the row log-sum-exp against the oracle's
    window_attention, psi against window_scores, statistics and pooled scores against the oracle on the
    GPU's own psi; the whole eviction that follows equals the one after madakv_score wherever the two
    psi agree to the last bit of every decision (checked through the free-running rules)."""
    import os
    wl = _window_workloads()[name]
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    G, nc = Hq // H, L - W
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, out_fp32=fp32_out)
    out = torch.full((NL, B, Hq, W, d), float("nan"), dtype=torch.float32 if fp32_out else torch.bfloat16, device=DEV)
    lse = torch.full((NL, B, Hq, W), float("nan"), dtype=torch.float32, device=DEV)
    for spin in (None, "1"):
        if spin:
            os.environ["MADAKV_SCORE_SPIN_LIMIT"] = spin          # workgroups that find a word missing go their own way
        try:
            eng.window_attn_score(0, NL, q, k, v, mask, out, lse)
            torch.cuda.synchronize()
        finally:
            os.environ.pop("MADAKV_SCORE_SPIN_LIMIT", None)
        qh, kh, vh = WL.to_f64(q), WL.to_f64(k), WL.to_f64(v)
        psi_g, pool_g = eng.psi.cpu().numpy(), eng.psi_pool.cpu().numpy()
        w_g, k_g = eng.stats_host()
        worst_o = worst_l = 0.0
        for l in range(NL):
            for b in range(B):
                o_ref, lse_ref = O.window_attention(qh[l, b], kh[l, b], vh[l, b], p.scale)
                o_g = out[l, b].float().cpu().numpy()
                tol = PU.DECODE_ATOL if fp32_out else PU.DECODE_ATOL + 2.0 ** -8 * np.abs(o_ref)     # bf16 output: half an ulp on top
                assert (np.abs(o_g - o_ref) <= tol).all(), (l, b, np.abs(o_g - o_ref).max())
                worst_o = max(worst_o, float(np.abs(o_g - o_ref).max()))
                np.testing.assert_allclose(lse[l, b].cpu().numpy(), lse_ref, atol=2e-4, rtol=0)
                worst_l = max(worst_l, float(np.abs(lse[l, b].cpu().numpy() - lse_ref).max()))
                psi_o = O.window_scores(qh[l, b], kh[l, b], p.scale)
                nbad, worst = PU.psi_close(psi_g[l, b], psi_o, G, W, L)
                assert nbad == 0, worst
                psi_in = psi_g[l, b].astype(np.float64)
                w_o, k_o, n_o = O.modality_stats(psi_in, masks[b], W, p.theta)
                PU.assert_masses_close(w_g[l, b], w_o, L)
                np.testing.assert_array_equal(pool_g[l, b], O.pool_scores(psi_in, W, p.pool_k).astype(np.float32))
                for h in range(H):
                    for m in (0, 1):
                        if k_g[l, b, h, m] != k_o[h, m]:
                            assert PU.k_count_ok(int(k_g[l, b, h, m]), psi_in[h, :nc][masks[b][:nc] == m], p.theta)
        say(f"{name} spin={spin}: out worst abs err {worst_o:.2e}, lse {worst_l:.2e}")
    # the eviction that follows, against the whole oracle
    eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    bud_g = eng.budgets.cpu().numpy(); kv_off, kv_len = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    kept_all = eng.kept_idx.cpu().numpy(); nmod_g = eng.n_mod.cpu().numpy()
    for b in range(B):
        res = O.evict(qh[:, b], kh[:, b], vh[:, b], masks[b], p)
        cnt = PU.free_running_check(p, res, masks[b], w_g[:, b], k_g[:, b], nmod_g[b], bud_g[:, b],
                                    lambda l, h: kept_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]], say)
        assert cnt["budget_unexcused"] == 0 and cnt["kept_unexcused"] == 0, cnt
    eng.close()


def test_window_attention_refusals():
    # contexts beyond what the heads' workgroups can exchange among themselves (256 chunks of 512 keys at head_dim 128)
    wl = small_workloads()["bf16_mha"].scaled(name="win_too_long", n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, ctx_len=131073,
                                              budget=300, n_images=2)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    out = torch.empty(wl.n_layers, wl.batch, wl.n_q_heads, wl.window, wl.head_dim, dtype=torch.float32, device=DEV)
    with pytest.raises(MB.MadaKVError) as ei:
        eng.window_attn_score(0, wl.n_layers, q, k, v, mask, out)
    assert ei.value.status == -7
    eng.close()
    wl = small_workloads()["tiny_fp32"]                       # fp32 inputs
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    out = torch.empty(wl.n_layers, wl.batch, wl.n_q_heads, wl.window, wl.head_dim, dtype=torch.float32, device=DEV)
    with pytest.raises(MB.MadaKVError) as ei:
        eng.window_attn_score(0, wl.n_layers, q, k, v, mask, out)
    assert ei.value.status == -7
    eng.close()


def test_error_paths_and_streams():
    """Host-side refusals on a live handle (nothing is enqueued), and calls on a non-default stream."""
    wl = small_workloads()["bf16_mha"].scaled(n_layers=2, batch=1, decode_steps=1)
    NL, H, L, W, d = wl.n_layers, wl.n_kv_heads, wl.ctx_len, wl.window, wl.head_dim
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    lib = MB.lib()
    import ctypes as C
    vp = lambda t: C.c_void_p(t.data_ptr())
    guard = eng.psi.clone().fill_(-3.0); eng.psi.copy_(guard)
    # layer range outside the model, null tensor, misaligned tensor, workspace too small
    assert lib.madakv_score(eng.h, 1, 2, vp(q), vp(k), vp(mask), vp(eng.psi), vp(eng.psi_pool), vp(eng.stats), vp(eng.n_mod),
                            vp(eng.score_ws), eng.score_ws.numel(), None) == -1
    assert lib.madakv_score(eng.h, 0, 2, None, vp(k), vp(mask), vp(eng.psi), vp(eng.psi_pool), vp(eng.stats), vp(eng.n_mod),
                            vp(eng.score_ws), eng.score_ws.numel(), None) == -1
    assert lib.madakv_score(eng.h, 0, 2, vp(q), C.c_void_p(k.data_ptr() + 2), vp(mask), vp(eng.psi), vp(eng.psi_pool), vp(eng.stats),
                            vp(eng.n_mod), vp(eng.score_ws), eng.score_ws.numel(), None) == -1
    assert lib.madakv_score(eng.h, 0, 2, vp(q), vp(k), vp(mask), vp(eng.psi), vp(eng.psi_pool), vp(eng.stats), vp(eng.n_mod),
                            vp(eng.score_ws), 8, None) == -4
    assert lib.madakv_decode_attn(eng.h, 0, 1, vp(q), vp(k), None, vp(eng.k_c), vp(eng.v_c), vp(eng.kv_off), vp(eng.kv_len),
                                  vp(eng.psi), vp(eng.decode_ws), eng.decode_ws.numel(), None) == -1      # k_new without v_new
    torch.cuda.synchronize()
    assert torch.equal(eng.psi, guard), "a refused call must leave its outputs untouched"
    assert lib.madakv_last_hip_error(eng.h) == 0
    # the same eviction on a side stream gives the same bits as on the default stream
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (eng.psi, eng.budgets, eng.kv_len, eng.kept_idx, eng.k_c)]
    eng2 = engine(wl)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        eng2.score(0, NL, q, k, mask); eng2.allocate(0, NL); eng2.select_gather(0, NL, k, v, mask)
    st.synchronize()
    n = int(eng.kv_len.sum()) + 0
    assert torch.equal(eng2.psi, ref[0]) and torch.equal(eng2.budgets, ref[1]) and torch.equal(eng2.kv_len, ref[2])
    off, ln = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    for l in range(NL):
        for h in range(H):
            o, m = off[l, 0, h], ln[l, 0, h]
            assert torch.equal(eng2.kept_idx[o:o + m], ref[3][o:o + m]) and torch.equal(eng2.k_c[o:o + m], ref[4][o:o + m])
    eng.close(); eng2.close()


def test_two_handles_and_handle_reuse():
    """Two handles of different shape interleaved, and a second prompt on the same handle."""
    wa = small_workloads()["bf16_mha"].scaled(n_layers=2, batch=1)
    wb = small_workloads()["bf16_d64_gqa2"]
    ea, eb = engine(wa), engine(wb)
    qa, ka, va, ma, _ = PU.make_inputs(wa, DEV)
    qb, kb, vb, mb, _ = PU.make_inputs(wb, DEV)
    ea.score(0, 2, qa, ka, ma); eb.score(0, 2, qb, kb, mb)
    ea.allocate(0, 2); eb.allocate(0, 2)
    ea.select_gather(0, 2, ka, va, ma); eb.select_gather(0, 2, kb, vb, mb)
    torch.cuda.synchronize()
    first = [t.clone() for t in (ea.budgets, ea.kv_off, ea.kv_len, ea.kept_idx)]
    assert int(ea.budgets.sum()) == 2 * wa.n_kv_heads * (wa.budget - wa.window)
    assert int(eb.budgets.sum()) == 2 * wb.n_kv_heads * (wb.budget - wb.window)
    # a second prompt (other seed -> other layer data), then the first again: same bits as the first time
    wa2 = wa.scaled(cfg_id=77)
    q2, k2, v2, m2, _ = PU.make_inputs(wa2, DEV)
    ea.score(0, 2, q2, k2, m2); ea.allocate(0, 2); ea.select_gather(0, 2, k2, v2, m2)
    ea.score(0, 2, qa, ka, ma); ea.allocate(0, 2); ea.select_gather(0, 2, ka, va, ma)
    torch.cuda.synchronize()
    assert torch.equal(ea.budgets, first[0]) and torch.equal(ea.kv_off, first[1]) and torch.equal(ea.kv_len, first[2])
    off, ln = ea.kv_off.cpu().numpy(), ea.kv_len.cpu().numpy()
    for l in range(2):
        for h in range(wa.n_kv_heads):
            o, m = off[l, 0, h], ln[l, 0, h]
            assert torch.equal(ea.kept_idx[o:o + m], first[3][o:o + m])
    ea.close(); eb.close()


@pytest.mark.parametrize("name", ["bf16_mha", "bf16_gqa7", "tiny_fp32"])
def test_score_with_given_row_normalisers(name):
    """madakv_score_lse: one pass over K when the caller supplies the proxy rows' log-sum-exp."""
    wl = small_workloads()[name]
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    G = wl.n_q_heads // H
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    qh, kh = WL.to_f64(q), WL.to_f64(k)
    lse_o = np.stack([np.stack([O.proxy_row_lse(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    lse = torch.from_numpy(lse_o.astype(np.float32)).to(DEV).contiguous()
    eng = engine(wl)
    say(f"{name}: madakv_score_lse")
    eng.score_lse(0, NL, q, k, mask, lse)
    torch.cuda.synchronize()
    psi_1 = eng.psi.clone(); stats_1 = eng.stats.clone(); pool_1 = eng.psi_pool.clone()
    psi_o = np.stack([np.stack([O.window_scores(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    nbad, worst = PU.psi_close(psi_1.cpu().numpy(), psi_o, G, W, L)
    assert nbad == 0, worst
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    assert torch.allclose(eng.psi, psi_1, rtol=2e-5, atol=1e-12)        # same scores either way (lse rounded to fp32)
    with pytest.raises(MB.MadaKVError):
        MB.madakv_score_lse(eng.h, 0, NL, q, k, mask, None, eng.psi, eng.psi_pool, eng.stats, eng.n_mod, eng.score_ws)
    eng.close()


@pytest.mark.parametrize("name", ["bf16_mha", "bf16_gqa7", "bf16_d64_gqa2", "bf16_odd"])
def test_fp8_reduced_cache(name):
    """cache_fp8: the reduced cache holds E4M3 bytes.  The bytes must be the oracle's encoding of the
    kept rows (and of the appended rows); decode must match Eq. 5 over the decoded values."""
    wl = small_workloads()[name]
    NL, B, H, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window, wl.head_dim
    G = wl.n_q_heads // H
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, cache_fp8=1)
    assert eng.k_c.dtype == torch.uint8
    say(f"{name}: eviction into an 8-bit cache")
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    off, ln = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    kept_all = eng.kept_idx.cpu().numpy()
    kc, vc = eng.k_c.cpu().numpy(), eng.v_c.cpu().numpy()
    kh, vh = WL.to_f64(k), WL.to_f64(v)
    caches = {}
    for l in range(NL):
        for b in range(B):
            for h in range(H):
                o, n = off[l, b, h], ln[l, b, h]
                kept = kept_all[o:o + n]
                want_k, want_v = O.quantize_e4m3(kh[l, b, h][kept]), O.quantize_e4m3(vh[l, b, h][kept])
                # the sign of an encoded zero is not compared (both are 0.0)
                assert (((kc[o:o + n] ^ want_k) & np.where((want_k & 0x7F) == 0, 0x7F, 0xFF)) == 0).all()
                assert (((vc[o:o + n] ^ want_v) & np.where((want_v & 0x7F) == 0, 0x7F, 0xFF)) == 0).all()
                caches[(l, b, h)] = [O.dequantize_e4m3(kc[o:o + n]), O.dequantize_e4m3(vc[o:o + n])]
    out = torch.empty(NL, B, wl.n_q_heads, d, dtype=torch.float32, device=DEV)
    for step in range(wl.decode_steps):
        dq, dk, dv = WL.decode_inputs_all(wl, step, DEV)
        say(f"{name}: fp8 decode step {step}")
        if step % 2 == 0:
            for l in range(NL):
                eng.decode_attn(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out[l:l + 1])
        else:
            eng.decode_attn(0, NL, dq, dk, dv, out)
        torch.cuda.synchronize()
        og = out.cpu().numpy()
        kc2, vc2 = eng.k_c.cpu().numpy(), eng.v_c.cpu().numpy()
        for (l, b, h), (ck, cv) in caches.items():
            nk = O.dequantize_e4m3(O.quantize_e4m3(WL.to_f64(dk[l, b, h])))
            nv = O.dequantize_e4m3(O.quantize_e4m3(WL.to_f64(dv[l, b, h])))
            ck = np.concatenate([ck, nk[None]]); cv = np.concatenate([cv, nv[None]])
            caches[(l, b, h)] = [ck, cv]
            o = off[l, b, h]
            np.testing.assert_array_equal(O.dequantize_e4m3(kc2[o + len(ck) - 1]), nk)      # the appended row, as stored
            np.testing.assert_array_equal(O.dequantize_e4m3(vc2[o + len(cv) - 1]), nv)
            for g in range(G):
                ref = O.attend(WL.to_f64(dq[l, b, h * G + g]), ck, cv, p.scale)
                assert np.abs(og[l, b, h * G + g] - ref).max() <= PU.DECODE_ATOL, (step, l, b, h, g)
    assert (eng.kv_len.cpu().numpy() == ln + wl.decode_steps).all()
    eng.close()


def _run_and_check_whole_path(wl, decode_steps=1):
    """Whole path on a (possibly degenerate) shape, every head against the oracle stage by stage."""
    NL, B, H, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window, wl.head_dim
    G, nc = wl.n_q_heads // H, L - W
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, max_new_tokens=decode_steps)
    eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    psi_g, pool_g = eng.psi.cpu().numpy(), eng.psi_pool.cpu().numpy()
    w_g, k_g = eng.stats_host()
    nmod, bud_g = eng.n_mod.cpu().numpy(), eng.budgets.cpu().numpy()
    off, ln, kept_all = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy(), eng.kept_idx.cpu().numpy()
    qh, kh, vh = WL.to_f64(q), WL.to_f64(k), WL.to_f64(v)
    out = torch.empty(NL, B, wl.n_q_heads, d, dtype=torch.float32, device=DEV)
    dq, dk, dv = WL.decode_inputs_all(wl, 0, DEV)
    eng.decode_attn(0, NL, dq, dk, dv, out)
    torch.cuda.synchronize()
    og = out.cpu().numpy()
    for b in range(B):
        for l in range(NL):
            psi_o = O.window_scores(qh[l, b], kh[l, b], p.scale)
            assert PU.psi_close(psi_g[l, b], psi_o, G, W, L)[0] == 0
            psi_in = psi_g[l, b].astype(np.float64)
            w_o, k_o, n_o = O.modality_stats(psi_in, masks[b], W, p.theta)
            assert tuple(nmod[b]) == tuple(n_o)
            PU.assert_masses_close(w_g[l, b], w_o, L)
            if not p.keep_all:
                np.testing.assert_array_equal(pool_g[l, b], O.pool_scores(psi_in, W, p.pool_k).astype(np.float32))
        np.testing.assert_array_equal(bud_g[:, b], O.allocate(w_g[:, b], k_g[:, b].astype(np.int64), nmod[b], p))
        for l in range(NL):
            for h in range(H):
                bt, bv = (int(x) for x in bud_g[l, b, h])
                ref = np.arange(L) if p.keep_all else O.select(pool_g[l, b, h].astype(np.float64), masks[b], bt, bv, L, W)
                o = off[l, b, h]
                np.testing.assert_array_equal(kept_all[o:o + ln[l, b, h]], ref)
                kc = np.concatenate([kh[l, b, h][ref], WL.to_f64(dk[l, b, h])[None]])
                vc = np.concatenate([vh[l, b, h][ref], WL.to_f64(dv[l, b, h])[None]])
                for g in range(G):
                    r = O.attend(WL.to_f64(dq[l, b, h * G + g]), kc, vc, p.scale)
                    assert np.abs(og[l, b, h * G + g] - r).max() <= PU.DECODE_ATOL
    eng.close()


@pytest.mark.parametrize("shape", [
    dict(ctx_len=3, window=1, budget=2),                  # one candidate kept of two
    dict(ctx_len=2, window=1, budget=2),                  # budget = context: keep all
    dict(ctx_len=40, window=1, budget=2),                 # a single proxy token, one candidate per head
    dict(ctx_len=33, window=32, budget=33),               # window = context - 1
    dict(ctx_len=300, window=16, budget=299),             # all but one candidate
    dict(ctx_len=257, window=16, budget=17),              # beta = 1
])
def test_degenerate_shapes(shape):
    L, W = shape["ctx_len"], shape["window"]
    t0 = max(1, (L - W) // 3)
    im = (L - W) - t0
    layout = ((0, t0),) + (((1, im),) if im > 0 else ()) + ((0, W),)          # text, image, the (text) window
    wl = WL.CONFIGS["tiny"].scaled(name="degenerate", dtype="bf16", n_layers=2, batch=1, n_q_heads=2, n_kv_heads=2,
                                   head_dim=64, pool_k=3, fixed_layout=layout, **shape)
    _run_and_check_whole_path(wl)


def test_widest_shapes():
    """64 KV heads (the lane limit of the allocation kernel), 8 query heads per KV head (the group limit)."""
    wl = WL.CONFIGS["llava_layer"].scaled(name="wide", n_layers=2, batch=1, n_q_heads=64, n_kv_heads=64, head_dim=64,
                                          ctx_len=900, window=8, budget=120, n_images=1)
    _run_and_check_whole_path(wl)
    wl = WL.CONFIGS["llava_layer"].scaled(name="g8", n_layers=1, batch=2, n_q_heads=16, n_kv_heads=2, head_dim=128,
                                          ctx_len=1300, window=32, budget=200, n_images=1)
    _run_and_check_whole_path(wl)
    # 20 layers of 64 heads: a layer group lays out 320 segments per batch item, more than one trip of the
    # segment-layout workgroup
    wl = WL.CONFIGS["llava_layer"].scaled(name="deep_wide", n_layers=20, batch=1, n_q_heads=64, n_kv_heads=64, head_dim=64,
                                          ctx_len=900, window=8, budget=120, n_images=1)
    _run_and_check_whole_path(wl)

@pytest.mark.parametrize("shape", ["m128_d128", "m192_d64", "m80_d64_odd", "m224_long", "m96_one_tile", "m256_two_tiles",
                                   "m192_short_last_chunk", "m128_short_last_chunk"])
def test_more_than_64_proxy_rows(shape):
    """G*W between 65 and 256: the two-sweep scoring kernels whose waves own blocks of proxy rows and share the keys
    through an LDS ring.  One and two row blocks per wave, both head dims, several chunks per head in both sweeps
    (the second sweep cuts the keys its own way), a ragged last tile; with and without given row normalisers."""
    kw = {"m128_d128": dict(n_q_heads=8, n_kv_heads=2, head_dim=128, window=32, ctx_len=5000),
          "m192_d64": dict(n_q_heads=6, n_kv_heads=2, head_dim=64, window=64, ctx_len=4100),
          "m80_d64_odd": dict(n_q_heads=4, n_kv_heads=2, head_dim=64, window=40, ctx_len=3001),
          "m224_long": dict(n_q_heads=7, n_kv_heads=1, head_dim=128, window=32, ctx_len=9001),
          # the first sweep's last chunk holds 34 keys, fewer than the window: the first 30 rows of every query head
          # see none of them (a workgroup whose rows have nothing to add up)
          "m192_short_last_chunk": dict(n_q_heads=3, n_kv_heads=1, head_dim=128, window=64, ctx_len=9250),
          "m128_short_last_chunk": dict(n_q_heads=2, n_kv_heads=1, head_dim=64, window=64, ctx_len=9250),
          # contexts of one and two LDS tiles: the ring's start-up and its end meet
          "m96_one_tile": dict(n_q_heads=3, n_kv_heads=1, head_dim=128, window=32, ctx_len=60, budget=44, n_images=1,
                               image_tokens=(10, 10), text_tokens=(4, 30)),
          "m256_two_tiles": dict(n_q_heads=8, n_kv_heads=1, head_dim=64, window=32, ctx_len=150, budget=60, n_images=1,
                                 image_tokens=(40, 40), text_tokens=(4, 60))}[shape]
    kw = dict(dict(budget=300, n_images=3), **kw)
    wl = WL.CONFIGS["llava_layer"].scaled(name=shape, n_layers=2, batch=1, decode_steps=1, **kw)
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    G = wl.n_q_heads // H
    assert 64 < G * W <= 256
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    qh, kh = WL.to_f64(q), WL.to_f64(k)
    psi_o = np.stack([np.stack([O.window_scores(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    eng = engine(wl)
    say(f"{shape}: madakv_score, {G * W} proxy rows")
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    psi_1 = eng.psi.clone()
    nbad, worst = PU.psi_close(psi_1.cpu().numpy(), psi_o, G, W, L)
    say(f"{shape}: psi worst scaled error {worst:.2e}")
    assert nbad == 0, f"psi: {nbad} entries outside tolerance (worst {worst})"
    np.testing.assert_allclose(psi_1.cpu().numpy().sum(-1), G * W, rtol=2e-4)
    eng.score(0, NL, q, k, mask)                                        # run to run: bit for bit
    torch.cuda.synchronize()
    assert torch.equal(eng.psi, psi_1)
    lse_o = np.stack([np.stack([O.proxy_row_lse(qh[l, b], kh[l, b], p.scale) for b in range(B)]) for l in range(NL)])
    say(f"{shape}: madakv_score_lse")
    eng.score_lse(0, NL, q, k, mask, torch.from_numpy(lse_o.astype(np.float32)).to(DEV).contiguous())
    torch.cuda.synchronize()
    assert torch.allclose(eng.psi, psi_1, rtol=2e-5, atol=1e-12)
    _run_and_check_whole_path(wl)
    eng.close()


def test_seeded_shapes_with_many_proxy_rows():
    """Twenty seeded random shapes with 33..256 proxy rows (group sizes 1..8, windows 16..64, both head dims, lengths
    around the chunk boundaries of both sweeps): psi of madakv_score and of madakv_window_attn_score, and the
    attention output, against the oracle."""
    rng = np.random.default_rng(20250615)
    for it in range(20):
        d = int(rng.choice([64, 128]))
        while True:
            G = int(rng.integers(1, 9)); W = int(rng.choice([16, 20, 32, 40, 64]))
            if 32 < G * W <= 256:
                break
        H = int(rng.integers(1, 4)); NL = int(rng.integers(1, 3))
        L = max(W + 40, int(rng.choice([300, 1024, 2048, 4096, 9216, 10240])) + int(rng.integers(-70, 70)))
        budget = W + 20 + int(rng.integers(0, min(L - W - 30, 300)))
        wl = WL.CONFIGS["llava_layer"].scaled(name=f"seeded{it}", n_layers=NL, batch=1, n_q_heads=G * H, n_kv_heads=H, head_dim=d,
                                              window=W, ctx_len=L, budget=budget, n_images=1, image_tokens=(20, 60),
                                              text_tokens=(10, 100), decode_steps=1)
        say(f"shape {it}: d={d} G={G} W={W} ({G * W} rows) H={H} layers={NL} L={L}")
        p = PU.oracle_params(wl)
        q, k, v, mask, masks = PU.make_inputs(wl, DEV)
        qh, kh, vh = WL.to_f64(q), WL.to_f64(k), WL.to_f64(v)
        eng = engine(wl, out_fp32=1)
        eng.score(0, NL, q, k, mask)
        torch.cuda.synchronize()
        psi_s = eng.psi.cpu().numpy().copy()
        out = torch.full((NL, 1, G * H, W, d), float("nan"), dtype=torch.float32, device=DEV)
        eng.window_attn_score(0, NL, q, k, v, mask, out)
        torch.cuda.synchronize()
        psi_w = eng.psi.cpu().numpy()
        for l in range(NL):
            psi_o = O.window_scores(qh[l, 0], kh[l, 0], p.scale)
            for what, pg in (("score", psi_s[l, 0]), ("window attention", psi_w[l, 0])):
                nbad, worst = PU.psi_close(pg, psi_o, G, W, L)
                assert nbad == 0, (it, what, l, nbad, worst)
            o_ref, _ = O.window_attention(qh[l, 0], kh[l, 0], vh[l, 0], p.scale)
            assert np.abs(out[l, 0].cpu().numpy() - o_ref).max() <= PU.DECODE_ATOL, (it, l)
        eng.close()


def test_long_heads_take_the_chunk_parallel_path():
    """Heads of more than 16384 candidates on a handful of heads: statistics (Eq. 6, 9, pooling) and selection give
    every 16384-candidate chunk a workgroup of its own and meet in memory between launches.  Four chunks per head
    here, the last one ragged.  Statistics and pooled scores against the oracle on the GPU's own psi, kept positions
    against the oracle on the GPU's pooled scores and budgets, then hand-made scores with few distinct values, so
    that the threshold-valued candidates to keep are counted across chunk boundaries."""
    wl = small_workloads()["bf16_mha"].scaled(name="bf16_long_ctx", n_layers=2, batch=1, n_q_heads=2, n_kv_heads=2,
                                               ctx_len=50001, budget=3000, n_images=3, decode_steps=1)
    NL, B, H, L, W = wl.n_layers, wl.batch, wl.n_kv_heads, wl.ctx_len, wl.window
    G, nc = wl.n_q_heads // H, L - W
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl)
    say("long heads: madakv_score")
    eng.score(0, NL, q, k, mask)
    torch.cuda.synchronize()
    psi_g, pool_g = eng.psi.cpu().numpy(), eng.psi_pool.cpu().numpy()
    w_g, k_g = eng.stats_host()
    nmod_g = eng.n_mod.cpu().numpy()
    for l in range(NL):
        psi_in = psi_g[l, 0].astype(np.float64)
        w_o, k_o, n_o = O.modality_stats(psi_in, masks[0], W, p.theta)
        assert tuple(nmod_g[0]) == tuple(n_o)
        PU.assert_masses_close(w_g[l, 0], w_o, L)
        np.testing.assert_array_equal(pool_g[l, 0], O.pool_scores(psi_in, W, p.pool_k).astype(np.float32))
        for h in range(H):
            for m in (0, 1):
                if k_g[l, 0, h, m] != k_o[h, m]:
                    assert PU.k_count_ok(int(k_g[l, 0, h, m]), psi_in[h, :nc][masks[0][:nc] == m], p.theta)
    eng.allocate(0, NL)
    eng.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    bud_g = eng.budgets.cpu().numpy()
    kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    kc_all = eng.k_c.cpu()
    for l in range(NL):
        for h in range(H):
            bt, bv = (int(x) for x in bud_g[l, 0, h])
            ref = O.select(pool_g[l, 0, h].astype(np.float64), masks[0], bt, bv, L, W)
            np.testing.assert_array_equal(kept_all[off[l, 0, h]:off[l, 0, h] + ln[l, 0, h]], ref)
            assert torch.equal(kc_all[off[l, 0, h]:off[l, 0, h] + len(ref)], k[l, 0, h].cpu()[ref])
    # few distinct values: ties everywhere, resolved by position across the chunks
    r = np.random.default_rng(11)
    m0 = masks[0]
    n_t, n_v = int((m0[:nc] == 0).sum()), int((m0[:nc] == 1).sum())
    pool = r.integers(0, 4, size=(NL, 1, H, nc)).astype(np.float32) * 0.5
    pool[1, 0, 1] = 2.0                                            # one value only
    tot = wl.budget - W                                            # what a head's segment has room for on average
    bud = np.array([[[[min(n_t, tot // 3), min(n_v, tot - tot // 3)], [0, min(n_v, tot)]]],
                    [[[min(n_t, 17), min(n_v, tot - 17)], [min(n_t, tot // 2), min(n_v, tot - tot // 2)]]]], dtype=np.int32)
    assert int(bud.sum()) + NL * H * (W + wl.decode_steps) <= eng.capacity
    eng.select_gather(0, NL, k, v, mask, psi_pool=torch.from_numpy(pool).to(DEV), budgets=torch.from_numpy(bud).to(DEV))
    torch.cuda.synchronize()
    kept_all, off, ln = eng.kept_idx.cpu().numpy(), eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    for l in range(NL):
        for h in range(H):
            ref = O.select(pool[l, 0, h].astype(np.float64), m0, int(bud[l, 0, h, 0]), int(bud[l, 0, h, 1]), L, W)
            np.testing.assert_array_equal(kept_all[off[l, 0, h]:off[l, 0, h] + ln[l, 0, h]], ref)
    eng.close()


def test_decode_long_heads_across_a_chunk_boundary():
    """Eq. 3-5 on heads of 2300 rows (nine 256-row chunks per head, merged in chunk order) that grow past 2304
    during the steps: one step appends the row that opens a tenth chunk, which then holds nothing but that row.
    Outputs against the oracle step by step, lengths and appended rows exactly."""
    wl = small_workloads()["bf16_mha"].scaled(name="bf16_long_heads", n_layers=2, batch=1, n_q_heads=3, n_kv_heads=3,
                                               ctx_len=3000, budget=2300, decode_steps=8)
    NL, B, H, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.head_dim
    p = PU.oracle_params(wl)
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = engine(wl, hcc_mode=0)                                   # every head keeps exactly `budget` rows
    eng.evict(0, NL, q, k, v, mask)
    torch.cuda.synchronize()
    kv_off, kv_len = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    assert (kv_len == wl.budget).all()
    kc_all, vc_all = eng.k_c.cpu(), eng.v_c.cpu()
    k_cache = [[[WL.to_f64(kc_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]]) for h in range(H)]
                for b in range(B)] for l in range(NL)]
    v_cache = [[[WL.to_f64(vc_all[kv_off[l, b, h]:kv_off[l, b, h] + kv_len[l, b, h]]) for h in range(H)]
                for b in range(B)] for l in range(NL)]
    out = torch.full((NL, B, wl.n_q_heads, d), float("nan"), dtype=torch.float32, device=DEV)
    for step in range(wl.decode_steps):
        rows = [[WL.decode_inputs(wl, l, b, step, DEV) for b in range(B)] for l in range(NL)]
        dq = torch.stack([torch.stack([r[0] for r in row]) for row in rows]).contiguous()
        dk = torch.stack([torch.stack([r[1] for r in row]) for row in rows]).contiguous()
        dv = torch.stack([torch.stack([r[2] for r in row]) for row in rows]).contiguous()
        say(f"decode step {step}, head length {wl.budget + step}")
        for l in range(NL):                                        # one call per layer: 256-row chunks
            eng.decode_attn(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out[l:l + 1])
        torch.cuda.synchronize()
        out_g = out.cpu().numpy()
        for l in range(NL):
            for b in range(B):
                ref = O.decode_step(WL.to_f64(dq[l, b]), WL.to_f64(dk[l, b]), WL.to_f64(dv[l, b]),
                                    k_cache[l][b], v_cache[l][b], p.scale)
                err = np.abs(out_g[l, b] - ref).max()
                assert err <= PU.DECODE_ATOL, (step, l, b, err)
        assert (eng.kv_len.cpu().numpy() == kv_len + step + 1).all(), step
    kc2 = eng.k_c.cpu()
    for l in range(NL):
        for b in range(B):
            for h in range(H):
                o = kv_off[l, b, h]
                np.testing.assert_array_equal(WL.to_f64(kc2[o:o + wl.budget + wl.decode_steps]), k_cache[l][b][h])
    eng.close()


@pytest.mark.parametrize("nl,groups", [(3, "4"), (6, "4"), (9, "4"), (6, "2"), (9, None)])
def test_fused_eviction_call_matches_the_three_calls(nl, groups, monkeypatch):
    """madakv_evict (pipelined over layer groups on two streams) against score + allocate + select_gather.
    groups None: the library's own choice (one group for a shape this small)."""
    if groups is None:
        monkeypatch.delenv("MADAKV_LAYER_GROUPS")
    else:
        monkeypatch.setenv("MADAKV_LAYER_GROUPS", groups)
    wl = small_workloads()["bf16_mha"].scaled(n_layers=nl, batch=2, ctx_len=1900)
    NL = wl.n_layers
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    a = engine(wl)
    a.score(0, NL, q, k, mask); a.allocate(0, NL); a.select_gather(0, NL, k, v, mask)
    torch.cuda.synchronize()
    b = engine(wl)
    for rep in range(2):                                    # twice: the handle's streams and carries are reused
        say(f"madakv_evict over {NL} layers, pass {rep}")
        b.evict(0, NL, q, k, v, mask)
        torch.cuda.synchronize()
        for name in ("psi", "psi_pool", "stats", "n_mod", "budgets", "kv_off", "kv_len"):
            assert torch.equal(getattr(a, name), getattr(b, name)), name
        off, ln = a.kv_off.cpu().numpy(), a.kv_len.cpu().numpy()
        for l in range(NL):
            for bb in range(wl.batch):
                for h in range(wl.n_kv_heads):
                    o, n = off[l, bb, h], ln[l, bb, h]
                    assert torch.equal(a.kept_idx[o:o + n], b.kept_idx[o:o + n])
                    assert torch.equal(a.k_c[o:o + n], b.k_c[o:o + n]) and torch.equal(a.v_c[o:o + n], b.v_c[o:o + n])
    # decode right after the fused call (sized from the lengths it handed to the host)
    dq, dk, dv = WL.decode_inputs_all(wl, 0, DEV)
    oa = torch.empty(NL, wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device=DEV); ob = torch.empty_like(oa)
    a.decode_attn(0, NL, dq, dk, dv, oa); b.decode_attn(0, NL, dq, dk, dv, ob)
    torch.cuda.synchronize()
    assert torch.equal(oa, ob)
    a.close(); b.close()
