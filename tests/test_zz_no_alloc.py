"""madakv_decode_attn_static (the decode step for callers that cannot allocate: its scratch is an
array inside the library's device code) against madakv_decode_attn on the same cache, through the
C ABI: two calls in a row, the second on a smaller input, then an appending call against the
oracle.  Collected last, so that a failure here hides no other test."""
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


def say(msg):
    print(f"[no_alloc] {msg}", flush=True)
    sys.stdout.flush()


def evicted_engine(wl, **kw):
    q, k, v, mask, masks = PU.make_inputs(wl, DEV)
    eng = MB.MadaKV(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                    head_dim=wl.head_dim, ctx_len=wl.ctx_len, window=wl.window, budget=wl.budget, dtype=wl.dtype,
                    pool_k=wl.pool_k, max_new_tokens=wl.decode_steps, out_fp32=1, device=DEV, **kw)
    eng.score(0, wl.n_layers, q, k, mask)
    eng.allocate(0, wl.n_layers)
    eng.select_gather(0, wl.n_layers, k, v, mask)
    torch.cuda.synchronize()
    return eng


def step_inputs(wl, step):
    rows = [[WL.decode_inputs(wl, l, b, step, DEV) for b in range(wl.batch)] for l in range(wl.n_layers)]
    pick = lambda i: torch.stack([torch.stack([r[i] for r in row]) for row in rows]).contiguous()
    return pick(0), pick(1), pick(2)


def oracle_outputs(eng, wl, dq):
    """Eq. 5 over the cache rows as they are now, per layer and batch item."""
    off, ln = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
    p = PU.oracle_params(wl)
    ref = np.zeros((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim))
    for l in range(wl.n_layers):
        for b in range(wl.batch):
            kc = [WL.to_f64(eng.k_c[off[l, b, h]:off[l, b, h] + ln[l, b, h]]) for h in range(wl.n_kv_heads)]
            vc = [WL.to_f64(eng.v_c[off[l, b, h]:off[l, b, h] + ln[l, b, h]]) for h in range(wl.n_kv_heads)]
            ref[l, b] = O.decode_step(WL.to_f64(dq[l, b]), None, None, kc, vc, p.scale)
    return ref


def test_static_scratch_decode_matches_the_workspace_call():
    # heads of a few hundred rows at 256-row chunks: several chunks per head, so the partial
    # results do pass through the scratch array
    big = WL.CONFIGS["llava_layer"].scaled(name="na_big", n_layers=3, batch=2, n_q_heads=8, n_kv_heads=4, ctx_len=3000,
                                           budget=700, n_images=3, decode_steps=2)
    small = WL.CONFIGS["llava_layer"].scaled(name="na_small", n_layers=1, batch=1, n_q_heads=4, n_kv_heads=4, ctx_len=1200,
                                             budget=300, n_images=1, decode_steps=2)
    e_big, e_small = evicted_engine(big), evicted_engine(small)
    assert int(e_big.kv_len.max()) > 256 and int(e_small.kv_len.max()) > 256

    def both(eng, wl, l0, n, dq):
        shape = (n, wl.batch, wl.n_q_heads, wl.head_dim)
        ref = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
        got = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
        eng.decode_attn(l0, n, dq[l0:l0 + n], None, None, ref)
        eng.decode_attn_static(l0, n, dq[l0:l0 + n], None, None, got)
        torch.cuda.synchronize()
        return ref, got

    dq_big, dk_big, dv_big = step_inputs(big, 0)
    dq_small, dk_small, dv_small = step_inputs(small, 0)
    say("first call: three layers, one layer at a time (several chunks per head)")
    want = oracle_outputs(e_big, big, dq_big)
    for l in range(big.n_layers):
        ref, got = both(e_big, big, l, 1, dq_big)
        assert torch.equal(ref, got)
        assert np.abs(got.cpu().numpy()[0] - want[l]).max() <= PU.DECODE_ATOL
    say("second call: the smaller input right after it")
    ref, got = both(e_small, small, 0, 1, dq_small)
    assert torch.equal(ref, got)
    assert np.abs(got.cpu().numpy() - oracle_outputs(e_small, small, dq_small)).max() <= PU.DECODE_ATOL
    say("and the large one again, all layers in one call")
    ref, got = both(e_big, big, 0, big.n_layers, dq_big)
    assert torch.equal(ref, got)
    assert np.abs(got.cpu().numpy() - want).max() <= PU.DECODE_ATOL

    say("appending calls")
    len0 = e_big.kv_len.clone()
    out = torch.empty(big.n_layers, big.batch, big.n_q_heads, big.head_dim, dtype=torch.float32, device=DEV)
    for l in range(big.n_layers):
        e_big.decode_attn_static(l, 1, dq_big[l:l + 1], dk_big[l:l + 1], dv_big[l:l + 1], out[l:l + 1])
    torch.cuda.synchronize()
    assert torch.equal(e_big.kv_len, len0 + 1)
    assert np.abs(out.cpu().numpy() - oracle_outputs(e_big, big, dq_big)).max() <= PU.DECODE_ATOL   # the cache now holds the new rows
    off = e_big.kv_off.cpu().numpy(); ln = e_big.kv_len.cpu().numpy()
    for l in range(big.n_layers):
        for b in range(big.batch):
            for h in range(big.n_kv_heads):
                last = int(off[l, b, h] + ln[l, b, h] - 1)
                assert torch.equal(e_big.k_c[last], dk_big[l, b, h]) and torch.equal(e_big.v_c[last], dv_big[l, b, h])
    e_big.close(); e_small.close()


def test_static_scratch_refuses_what_does_not_fit():
    # 64 heads x up to 129 chunks x 8 query heads x 130 floats is far beyond 8 MiB when the lengths
    # are not yet known to the host (no eviction on this handle): refused on the host, nothing runs
    eng = MB.MadaKV(n_layers=1, batch=2, n_q_heads=256, n_kv_heads=32, head_dim=128, ctx_len=131072, window=32, budget=1024,
                    dtype="bf16", max_new_tokens=1, device=DEV)
    q = torch.zeros(1, 2, 256, 128, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, 2, 256, 128, dtype=torch.float32, device=DEV)
    with pytest.raises(MB.MadaKVError) as ei:
        eng.decode_attn_static(0, 1, q, None, None, out)
    assert ei.value.status == -4
    eng.close()


def test_captured_decode_step_replays_while_heads_grow():
    """The use the entry point names first: a decode step (one call per layer) captured into a HIP graph and replayed.
    Heads of 2300 rows that grow past 2304 during the replays, so the captured launch has to cover a chunk that did
    not exist at capture time.  Every replay (with eager work and a synchronisation in between) against an engine that
    takes the same steps with ordinary calls: outputs bit for bit, lengths and the appended rows exactly."""
    wl = WL.CONFIGS["llava_layer"].scaled(name="na_graph", n_layers=2, batch=1, n_q_heads=3, n_kv_heads=3, ctx_len=3000,
                                          budget=2300, n_images=2, decode_steps=8)
    NL = wl.n_layers
    eager, graphed = evicted_engine(wl, hcc_mode=0), evicted_engine(wl, hcc_mode=0)
    assert (graphed.kv_len.cpu().numpy() == wl.budget).all()
    shape = (NL, wl.batch, wl.n_q_heads, wl.head_dim)
    out_e = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    out_g = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    # one ordinary step on both (the length of the longest head reaches the host meanwhile)
    dq, dk, dv = step_inputs(wl, 0)
    for eng, out in ((eager, out_e), (graphed, out_g)):
        for l in range(NL):
            eng.decode_attn_static(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out[l:l + 1])
    torch.cuda.synchronize()
    assert torch.equal(out_e, out_g)
    # the step as a graph: inputs at fixed addresses
    sq, sk, sv = dq.clone(), dk.clone(), dv.clone()
    g = torch.cuda.CUDAGraph()
    say("capturing one decode step (two layers) on the static scratch")
    with torch.cuda.graph(g):
        for l in range(NL):
            graphed.decode_attn_static(l, 1, sq[l:l + 1], sk[l:l + 1], sv[l:l + 1], out_g[l:l + 1])
    torch.cuda.synchronize()
    assert (graphed.kv_len.cpu().numpy() == wl.budget + 1).all(), "capturing runs nothing"
    for step in range(1, 7):                                   # lengths 2301 .. 2307: a tenth chunk appears on the way
        dq, dk, dv = step_inputs(wl, step)
        sq.copy_(dq); sk.copy_(dk); sv.copy_(dv)               # eager work between the replays
        out_g.fill_(float("nan"))
        torch.cuda.synchronize()
        say(f"replay {step}: head length {wl.budget + step}")
        g.replay()
        for l in range(NL):
            eager.decode_attn_static(l, 1, dq[l:l + 1], dk[l:l + 1], dv[l:l + 1], out_e[l:l + 1])
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), (step, float((out_g - out_e).abs().max()))
        assert torch.equal(graphed.kv_len, eager.kv_len) and int(graphed.kv_len.max()) == wl.budget + step + 1
    off, ln = eager.kv_off.cpu().numpy().ravel(), eager.kv_len.cpu().numpy().ravel()
    for o, n in zip(off, ln):                                   # the rows in use (the room beyond them was never written)
        assert torch.equal(graphed.k_c[o:o + n], eager.k_c[o:o + n]) and torch.equal(graphed.v_c[o:o + n], eager.v_c[o:o + n])
    want = oracle_outputs(eager, wl, dq)                        # the last step's queries over the cache as it is now ...
    got = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    for l in range(NL):
        eager.decode_attn_static(l, 1, dq[l:l + 1], None, None, got[l:l + 1])   # ... attended once more without appending
    torch.cuda.synchronize()
    assert np.abs(got.cpu().numpy() - want).max() <= PU.DECODE_ATOL
    eager.close(); graphed.close()
