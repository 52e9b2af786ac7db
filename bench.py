"""Benchmark of the MadaKV hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input of the 16K-context
workload (32 layers, batch 4, 32 heads, L = 16384, budget 2048, window 32):
    eviction   madakv_evict (= madakv_score + madakv_allocate + madakv_select_gather) over all layers
    decode     128 steps of madakv_decode_attn over the reduced cache, one call per layer
Inputs are resident in HBM before the timed region.  The metric is evicted-context
tokens/s = B * L / (time of the eviction part); the decode step time is reported beside it.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_inputs(wl, dev):
    import torch
    from paper_2506_15724_amd import workloads as WL
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    masks = [WL.modality_mask(wl, b) for b in range(B)]
    k = torch.empty(NL, B, H, L, d, dtype=wl.torch_dtype, device=dev)
    v = torch.empty(NL, B, H, L, d, dtype=wl.torch_dtype, device=dev)
    q = torch.empty(NL, B, Hq, W, d, dtype=wl.torch_dtype, device=dev)
    for l in range(NL):
        for b in range(B):
            q[l, b], k[l, b], v[l, b] = WL.layer_inputs(wl, l, b, masks[b], dev)
    import numpy as np
    mask = torch.from_numpy(np.stack(masks)).to(dev)
    return q, k, v, mask, masks


class LayerCalls:
    """Pre-marshalled arguments of the per-layer madakv_decode_attn calls (pointer arithmetic
    done once, so the timed loop is one foreign call per layer)."""

    def __init__(self, eng, q_all, kn_all, vn_all, out):
        from paper_2506_15724_amd import binding as MB
        self.fn = MB.lib().madakv_decode_attn
        self.h = eng.h
        c = eng.cfg
        NL = c.n_layers
        es = q_all.element_size()
        self.steps = q_all.shape[0]
        q_l = q_all[0, 0].numel() * es
        kn_l = kn_all[0, 0].numel() * es
        self.q_step, self.kn_step = q_all[0].numel() * es, kn_all[0].numel() * es
        self.args = []
        for l in range(NL):
            self.args.append((l, q_all.data_ptr() + l * q_l, kn_all.data_ptr() + l * kn_l, vn_all.data_ptr() + l * kn_l,
                              C.c_void_p(eng.kv_off[l].data_ptr()), C.c_void_p(eng.kv_len[l].data_ptr()),
                              C.c_void_p(out[l].data_ptr())))
        self.kc, self.vc = C.c_void_p(eng.k_c.data_ptr()), C.c_void_p(eng.v_c.data_ptr())
        self.ws = C.c_void_p(eng.decode_ws.data_ptr())
        self.ws_bytes = eng.decode_ws.numel()

    def run_step(self, s, stream):
        fn, h, kc, vc, ws, wsb = self.fn, self.h, self.kc, self.vc, self.ws, self.ws_bytes
        qo, ko = s * self.q_step, s * self.kn_step
        for (l, qp, kp, vp, off, ln, out) in self.args:
            rc = fn(h, l, 1, C.c_void_p(qp + qo), C.c_void_p(kp + ko), C.c_void_p(vp + ko), kc, vc, off, ln, out, ws, wsb, stream)
            if rc != 0:
                raise RuntimeError(f"madakv_decode_attn layer {l} -> {rc}")


def cpu_baseline(wl, q, k, v, masks, n_sample_layers=8, eng=None, dq0=None):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same
    workload: the whole eviction (Eq. 7, 6, 9, pooling, Eq. 8/10/11, selection, gather) of every
    `stride`-th layer of every batch item, run as a model of that many layers; scaled to the
    full layer count."""
    from oracle import madakv_oracle as O
    from paper_2506_15724_amd import workloads as WL
    NL, B = wl.n_layers, wl.batch
    n_s = min(n_sample_layers, NL)
    layers = [int(round(i * (NL - 1) / max(1, n_s - 1))) for i in range(n_s)] if n_s > 1 else [0]
    p = O.Params(n_layers=n_s, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                 ctx_len=wl.ctx_len, window=wl.window, budget=wl.budget, pool_k=wl.pool_k)
    dt = 0.0
    for b in range(B):
        qh = WL.to_f64(q[layers, b]); kh = WL.to_f64(k[layers, b]); vh = WL.to_f64(v[layers, b])
        t0 = time.perf_counter()
        O.evict(qh, kh, vh, masks[b], p)
        dt += time.perf_counter() - t0
        if b == 0:                                    # the same thing with the BLAS pool held to one thread
            try:
                from threadpoolctl import threadpool_limits
                with threadpool_limits(limits=1):
                    t0 = time.perf_counter()
                    O.evict(qh, kh, vh, masks[b], p)
                    dt_single = time.perf_counter() - t0
            except Exception:
                dt_single = None
        del qh, kh, vh
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = 1
    cores = min(threads, len(os.sched_getaffinity(0)))
    full_seconds = dt * NL / n_s                      # all layers of all batch items
    dec = None
    if eng is not None:
        # the oracle's decode step (Eq. 3-5) over the reduced cache the GPU built: the sampled layers of
        # every batch item, attend only (the rows are already appended), scaled to all layers
        off, ln = eng.kv_off.cpu().numpy(), eng.kv_len.cpu().numpy()
        t_dec = 0.0
        for l in layers:
            for b in range(B):
                kc = [WL.to_f64(eng.k_c[off[l, b, h]:off[l, b, h] + ln[l, b, h]]) for h in range(wl.n_kv_heads)]
                vc = [WL.to_f64(eng.v_c[off[l, b, h]:off[l, b, h] + ln[l, b, h]]) for h in range(wl.n_kv_heads)]
                qd = WL.to_f64(dq0[l, b])
                t0 = time.perf_counter()
                O.decode_step(qd, None, None, kc, vc, p.scale)
                t_dec += time.perf_counter() - t0
        dec = {"value": t_dec * NL / n_s * 1e6, "unit": "us per decode step (all layers, all batch items)", "cores": cores,
               "sample": f"oracle decode_step over the reduced cache of layers {layers} x all {B} batch items: "
                         f"{t_dec:.2f} s measured, scaled by {NL}/{n_s}"}
    return {"value": B * wl.ctx_len / full_seconds, "unit": "ctx-tokens/s", "cores": cores, "kind": "oracle", "decode_step": dec,
            "sample": f"NumPy fp64 oracle, eviction of {n_s} of {NL} layers (layers {layers}) x all {B} batch items, "
                      f"{wl.n_kv_heads} heads, L={wl.ctx_len}: {dt:.1f} s measured, scaled by {NL}/{n_s}",
            "seconds_measured": dt,
            "one_blas_thread": None if dt_single is None else
            {"value": wl.ctx_len / (dt_single * NL / n_s), "unit": "ctx-tokens/s", "cores": 1,
             "sample": f"same {n_s} layers, batch item 0 only: {dt_single:.1f} s"}}


def read_profile(fname, key):
    """`key=<number>` from a committed rocprofv3 summary under profiles/, or None."""
    try:
        for line in open(os.path.join(ROOT, "profiles", fname)):
            if line.startswith(key + "="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def time_config(name, budget=None, steps=None):
    """Eviction and per-layer decode timing of one of the other named configurations (inputs
    generated here, resident before the timed regions)."""
    import torch
    from paper_2506_15724_amd import binding as MB
    from paper_2506_15724_amd import workloads as WL
    dev = "cuda:0"
    wl = WL.CONFIGS[name]
    if budget is not None:
        wl = wl.scaled(budget=budget)
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    S = steps or wl.decode_steps
    q, k, v, mask, masks = build_inputs(wl, dev)
    eng = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=wl.budget,
                    dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=S, out_fp32=0, device=dev)
    dq = torch.empty(S, NL, B, Hq, d, dtype=wl.torch_dtype, device=dev)
    dk = torch.empty(S, NL, B, H, d, dtype=wl.torch_dtype, device=dev)
    dv = torch.empty(S, NL, B, H, d, dtype=wl.torch_dtype, device=dev)
    for s_ in range(S):
        dq[s_], dk[s_], dv[s_] = WL.decode_inputs_all(wl, s_, dev)
    out = torch.empty(NL, B, Hq, d, dtype=wl.torch_dtype, device=dev)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev_ms, dec_ms = [], []
    for rep in range(4):
        eng.evict(0, NL, q, k, v, mask)
        calls = LayerCalls(eng, dq, dk, dv, out)
        torch.cuda.synchronize()
        e[0].record()
        eng.evict(0, NL, q, k, v, mask)
        e[1].record()
        for s_ in range(S):
            calls.run_step(s_, stream)
        e[2].record()
        torch.cuda.synchronize()
        ev_ms.append(e[0].elapsed_time(e[1])); dec_ms.append(e[1].elapsed_time(e[2]))
    import numpy as np
    ev, de = float(np.median(ev_ms[1:])), float(np.median(dec_ms[1:]))
    rows_end = int(eng.kv_len.to(torch.int64).sum().item())
    nh = NL * B * H
    rows_streamed = sum(rows_end - S * nh + (s_ + 1) * nh for s_ in range(S))
    es = 2 if wl.dtype == "bf16" else 4
    dec_bytes = rows_streamed * 2 * d * es
    kept = rows_end - S * nh
    ev_bytes = nh * L * d * es + kept * 4 * d * es
    flops = 2.0 * (Hq // H) * W * L * d * nh
    res = {"workload": f"{wl.name}: {NL} layers, batch {B}, {Hq} query / {H} KV heads, head_dim {d}, L={L}, window {W}, budget {wl.budget}, {S} decode steps",
           "evict_ms": ev, "ctx_tokens_per_s": B * L / (ev * 1e-3), "evict_algorithmic_GBps": ev_bytes / (ev * 1e-3) / 1e9,
           "evict_frac_of_hbm_peak": ev_bytes / (ev * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "score_flops": flops, "proxy_rows_M": (Hq // H) * W,
           "decode_step_us": de * 1e3 / S, "decode_us_per_layer_call": de * 1e3 / (S * NL),
           "decode_GBps": dec_bytes / (de * 1e-3) / 1e9, "decode_frac_of_hbm_peak": dec_bytes / (de * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "decode_bytes_per_layer_call": dec_bytes / (S * NL)}
    # the prefill's last-window attention with the scores as a by-product, where the library takes the shape
    # (more than 32 proxy rows: one pass over K and V per block of 32 rows)
    try:
        wout = torch.empty(NL, B, Hq, W, d, dtype=wl.torch_dtype, device=dev)
        ts = []
        for rep in range(3):
            e[0].record(); eng.window_attn_score(0, NL, q, k, v, mask, wout); e[1].record()
            torch.cuda.synchronize()
            ts.append(e[0].elapsed_time(e[1]))
        res["window_attn_score_ms"] = float(np.median(ts[1:]))
        res["window_attn_passes_over_k_and_v"] = ((Hq // H) * W + 31) // 32
        del wout
    except MB.MadaKVError as ex:
        res["window_attn_score_ms"] = None
        res["window_attn_note"] = str(ex)[:120]
    eng.close()
    del q, k, v, dq, dk, dv, eng
    torch.cuda.empty_cache()
    return res


def read_traffic(kernel_tag):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/<kernel_tag>_traffic.txt, line `traffic_bytes_per_launch=<n>`), or None."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llava_16k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the multi-layer-launch and full-cache decode timings")
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="decode steps per bench step (default: the workload's own count; fewer only for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives in the method's hot path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_15724_amd import binding as MB
    from paper_2506_15724_amd import workloads as WL

    MB.lib()                                   # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if a.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 1 << 30, "calibrate_copy_bytes_written": 1 << 30, "launches": 4}))
        return
    wl = WL.CONFIGS[a.workload]
    NL, B, H, Hq, L, W, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.ctx_len, wl.window, wl.head_dim
    es = 2 if wl.dtype == "bf16" else 4
    S = a.decode_steps if a.decode_steps > 0 else wl.decode_steps
    G_ = Hq // H
    log(f"workload {wl.name}: {NL} layers, B={B}, H={H}, L={L}, d={d}, W={W}, budget={wl.budget}, {S} decode steps")
    t0 = time.time()
    q, k, v, mask, masks = build_inputs(wl, dev)
    torch.cuda.synchronize()
    log(f"inputs resident in HBM ({(k.numel() + v.numel()) * es / 1e9:.1f} GB of K,V) after {time.time() - t0:.1f} s")

    eng = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=wl.budget,
                    dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=S, out_fp32=0, device=dev)
    dq = torch.empty(S, NL, B, Hq, d, dtype=wl.torch_dtype, device=dev)
    dk = torch.empty(S, NL, B, H, d, dtype=wl.torch_dtype, device=dev)
    dv = torch.empty(S, NL, B, H, d, dtype=wl.torch_dtype, device=dev)
    for s in range(S):
        dq[s], dk[s], dv[s] = WL.decode_inputs_all(wl, s, dev)
    out = torch.empty(NL, B, Hq, d, dtype=wl.torch_dtype, device=dev)
    calls = LayerCalls(eng, dq, dk, dv, out)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    log(f"decode inputs ready after {time.time() - t0:.1f} s")

    def evict():
        # score + allocate + select + gather over all layers, the library's one-call form
        eng.evict(0, NL, q, k, v, mask)

    def one_step(ev):
        ev[0].record()
        evict()
        ev[1].record()
        for s in range(S):
            calls.run_step(s, stream)
        ev[2].record()

    for _ in range(a.warmup):
        one_step([torch.cuda.Event(enable_timing=True) for _ in range(3)])
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(a.steps)]
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for i in range(a.steps):
        one_step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    evict_ms = [e[0].elapsed_time(e[1]) for e in events]
    decode_ms = [e[1].elapsed_time(e[2]) for e in events]
    ms_per_step = wall * 1e3 / a.steps
    evict_med = float(np.median(evict_ms))
    decode_med = float(np.median(decode_ms))
    value = B * L / (evict_med * 1e-3)

    # bytes the decode launches had to move: K and V rows of every head, once per step
    kv_len_end = eng.kv_len.to(torch.int64).sum().item()          # lengths after the S appends
    n_heads_total = NL * B * H
    rows_first = kv_len_end - S * n_heads_total                    # rows before the first append
    rows_streamed = sum(rows_first + (s + 1) * n_heads_total for s in range(S))
    decode_bytes = rows_streamed * 2 * d * es
    launches = S * NL
    per_launch_us = decode_med * 1e3 / launches
    achieved = decode_bytes / (decode_med * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_attn_kernel (+ its merge kernel), one launch per layer",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": read_traffic("decode_attn_kernel_llava_16k") if wl.name == "llava_16k" else None,
                "bytes_per_launch": decode_bytes / launches, "us_per_launch": per_launch_us}

    # eviction bytes: K read once for scoring, kept K,V rows read and written by the gather
    kept_rows = rows_first
    evict_bytes = NL * B * H * L * d * es + kept_rows * 4 * d * es
    result = {
        "metric": "evicted-context tokens/s (score+select+gather); decode step us at 16K ctx",
        "value": value, "unit": "ctx-tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {NL} layers, batch {B}, {H} heads MHA, head_dim {d}, L={L}, window {W}, "
                               f"budget {wl.budget}/head, {S} decode steps", "launches": "eviction: madakv_evict over all layers; decode: one call per layer"},
        "evict_ms": evict_med, "evict_ms_min": float(min(evict_ms)),
        "evict_layer_tokens_per_s": B * L * NL / (evict_med * 1e-3),
        "evict_algorithmic_GBps": evict_bytes / (evict_med * 1e-3) / 1e9,
        "decode_step_us": decode_med * 1e3 / S, "decode_step_us_min": float(min(decode_ms)) * 1e3 / S,
        "decode_GBps": achieved,
        "roofline": roofline,
    }

    # ---- the other bandwidth-bound kernels of the step, from HIP events around single calls over all layers.
    # score_call = the score sweep(s) of every layer group with the statistics kernels under them (the last
    # group's statistics are exposed); select_gather_call = segment layout + selection + gather.  Kernel-only
    # durations from the committed rocprofv3 trace of this same command stand beside them.
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=3):
        fn(); torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    if wl.budget < L:
        score_ms = timed(lambda: eng.score(0, NL, q, k, mask))
        eng.allocate(0, NL)
        # (select_gather resets the decode-step counters; the timed decode region above is over)
        sg_ms = timed(lambda: eng.select_gather(0, NL, k, v, mask))
        kept_now = int(eng.kv_len.to(torch.int64).sum().item())
        k_bytes = NL * B * H * L * d * es
        psi_bytes = NL * B * H * L * 4
        gather_bytes = kept_now * 4 * d * es
        score_flops = 2.0 * (Hq // H) * W * L * d * NL * B * H
        prof = "bench_" + wl.name + "_kernel_trace.txt"
        def entry(kernel, byts, ms, note, prof_key=None):
            d_ = {"kernel": kernel, "bound": "hbm", "algorithmic_bytes": byts, "us": ms * 1e3, "achieved": byts / (ms * 1e-3) / 1e9,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "note": note}
            ko = read_profile(prof, prof_key) if prof_key else None
            if ko:
                d_["kernel_only_us_from_profile"] = ko
                d_["kernel_only_frac_from_profile"] = byts / (ko * 1e-6) / 1e9 / HBM_PEAK_GBS
            return d_
        result["roofline_by_kernel"] = [
            entry("score_fused_kernel (one sweep over K; statistics kernels overlapped)" if (Hq // H) * W <= 64 else
                  "score_wide_dma_kernel x 2 sweeps (more than 64 proxy rows: bound by the vector arithmetic; statistics kernels overlapped)",
                  k_bytes + psi_bytes, score_ms,
                  "algorithmic bytes = K read once + psi written; the statistics of the last layer group are not hidden; "
                  "a plain streaming read reaches 6.1-6.5 TB/s on this machine", "score_total_us_per_eviction"),
            entry("gather_kernel (+ segment layout and selection kernels)", gather_bytes + 5 * NL * B * H * (L - W), sg_ms,
                  "algorithmic bytes = kept K,V rows read and written + pooled scores and mask read; a plain copy reaches "
                  "5.2-5.7 TB/s on this machine", None),
            entry("gather_kernel launches of an eviction (kernel time only)", gather_bytes,
                  read_profile(prof, "gather_total_us_per_eviction") / 1e3 if read_profile(prof, "gather_total_us_per_eviction") else sg_ms,
                  "duration summed over an eviction's gather launches in the committed rocprofv3 trace when present (else the call "
                  "above); in madakv_evict three of the four run beside the next group's statistics and selection kernels and "
                  "hold 4 workgroups per compute unit; one gather over all layers with nothing beside it takes 1.49 ms "
                  "(0.72 of peak); copy ceiling 5.2-5.7 TB/s", None),
            dict(roofline, kernel="decode_attn_kernel + decode_merge_kernel (one call per layer)",
                 note="a plain streaming read of the same 135 MB takes 22.6-25.6 us on this machine (0.66-0.75 of peak)",
                 kernel_only_us_from_profile=read_profile(prof, "decode_attn_kernel_avg_us"),
                 kernel_only_frac_from_profile=(decode_bytes / launches) / (read_profile(prof, "decode_attn_kernel_avg_us") * 1e-6) / 1e9 / HBM_PEAK_GBS
                 if read_profile(prof, "decode_attn_kernel_avg_us") else None)]
        if (Hq // H) * W > 64:
            # more than 64 proxy rows: the scoring kernels are bound by the vector unit.  Issue slots per logit
            # (a wave instruction occupies a SIMD's 16 lanes for 4 cycles, exp2 for 16): sweep 1 = 1.06 exp2 + 3.25
            # plain instructions = 7.5 slots, sweep 2 = 1 exp2 + 2 plain = 6; peak = 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
            rows_pad = ((Hq // H) * W + 31) // 32 * 32
            slots = 13.5 * rows_pad * L * NL * B * H
            alu_peak = 256 * 4 * 16 * 2.4e9
            e0_ = result["roofline_by_kernel"][0]
            e0_.update({"bound": "alu", "alu_lane_slots": slots, "alu_achieved_Tslots_per_s": slots / (score_ms * 1e-3) / 1e12,
                        "alu_peak_Tslots_per_s": alu_peak / 1e12, "alu_frac": slots / (score_ms * 1e-3) / alu_peak,
                        "alu_note": "vector-unit issue slots of the two sweeps' arithmetic (13.5 per logit, padded rows included) against "
                                    "256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz; the HBM figures beside it count K once"})
        # the contraction side of scoring: flops of Eq. 7's Q K^T (computed once per key) against the dense bf16 MFMA peak
        ctr = "score_fused_kernel_" + wl.name + "_mfma_counters.txt"
        result["score_mfma"] = {"flops_per_eviction": score_flops, "achieved": score_flops / (score_ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                                "peak": 2500.0, "frac": score_flops / (score_ms * 1e-3) / 1e12 / 2500.0,
                                "intensity_flop_per_byte": score_flops / k_bytes,
                                "mfma_busy_pct_from_counters": read_profile(ctr, "mfma_busy_pct"),
                                "mfma_flops_per_launch_from_counters": read_profile(ctr, "mfma_flops_per_launch"),
                                "note": "HBM-bound (intensity = G*W flop per byte of K against a ridge of about 310): the matrix cores idle most of the time by design"
                                if (Hq // H) * W <= 64 else
                                "two sweeps (the contraction runs twice: the flops counted here are one sweep's); bound by one exp2 per logit and sweep on the vector unit"}
        # restore the state the sections below expect (cache rebuilt, counters reset)
        eng.evict(0, NL, q, k, v, mask)
        torch.cuda.synchronize()
        kv_len_end = eng.kv_len.to(torch.int64).sum().item()

    if not a.no_extras:
        # (b) the same decode as ONE launch over all layers per step (attend-only, cache as left by the last step)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        eng.decode_attn(0, NL, dq[0], None, None, out)
        e0.record()
        for _ in range(reps):
            eng.decode_attn(0, NL, dq[0], None, None, out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        by = kv_len_end * 2 * d * es
        result["decode_all_layers_one_launch"] = {"us_per_step": ms * 1e3, "GBps": by / (ms * 1e-3) / 1e9,
                                                  "frac_of_peak": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # per-stage eviction times
        stage = {}
        for name, fn in (("score", lambda: eng.score(0, NL, q, k, mask)), ("allocate", lambda: eng.allocate(0, NL)),
                         ("select_gather", lambda: eng.select_gather(0, NL, k, v, mask))):
            fn(); torch.cuda.synchronize()
            e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            stage[name + "_ms"] = e0.elapsed_time(e1)
        result["evict_stage_ms"] = stage
        # the same eviction with the two-sweep scoring kernels (K read twice), switched on from the host
        os.environ["MADAKV_SCORE_TWO_SWEEPS"] = "1"
        try:
            result["evict_two_sweeps_ms"] = timed(lambda: eng.evict(0, NL, q, k, v, mask))
        finally:
            del os.environ["MADAKV_SCORE_TWO_SWEEPS"]
        # the same eviction as three separate calls (no overlap between them)
        for rep in range(2):
            e0.record()
            eng.score(0, NL, q, k, mask); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
            e1.record()
        torch.cuda.synchronize()
        result["evict_three_calls_ms"] = e0.elapsed_time(e1)
        # eviction time of the switchable readings / baseline policies on the same inputs
        variants = {"heads_share_layer_total": dict(hcc_mode=2), "text_first": dict(mpa_mode=2),
                    "modality_agnostic_uniform": dict(mpa_mode=0, hcc_mode=0), "average_pool": dict(pool_mode=1),
                    "shares_over_all_columns": dict(share_mode=1), "sink_recent": dict(select_mode=1)}
        variants["three_modalities"] = dict(n_modalities=3)
        mask3 = torch.from_numpy(np.stack([WL.modality_mask(wl.scaled(n_modalities=3), b) for b in range(B)])).to(dev)
        vres = {}
        for name, kw in variants.items():
            vmask = mask3 if name == "three_modalities" else mask
            ve = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W,
                           budget=wl.budget, dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=1, out_fp32=0, device=dev, **kw)
            for rep in range(2):
                e0.record()
                ve.score(0, NL, q, k, vmask); ve.allocate(0, NL); ve.select_gather(0, NL, k, v, vmask)
                e1.record()
            torch.cuda.synchronize()
            vres[name] = {"evict_ms": e0.elapsed_time(e1), "ctx_tokens_per_s": B * L / (e0.elapsed_time(e1) * 1e-3)}
            ve.close()
            del ve
        result["evict_variants"] = vres
        # the same eviction called layer by layer (three calls per layer), as a prefill that frees each
        # layer's full K, V right after evicting it would drive it
        for rep in range(2):
            e0.record()
            for l in range(NL):
                eng.score(l, 1, q[l:l + 1], k[l:l + 1], mask)
                eng.allocate(l, 1)
                eng.select_gather(l, 1, k[l:l + 1], v[l:l + 1], mask)
            e1.record()
        torch.cuda.synchronize()
        result["evict_layer_by_layer"] = {"evict_ms": e0.elapsed_time(e1), "ctx_tokens_per_s": B * L / (e0.elapsed_time(e1) * 1e-3)}
        # the 8-bit (E4M3) reduced cache: eviction, then decode one call per layer and all layers in one call
        try:
            f8 = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W,
                           budget=wl.budget, dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=S, out_fp32=0, cache_fp8=1,
                           device=dev)
            for rep in range(2):
                e0.record()
                f8.score(0, NL, q, k, mask); f8.allocate(0, NL); f8.select_gather(0, NL, k, v, mask)
                e1.record()
            torch.cuda.synchronize()
            f8_evict = e0.elapsed_time(e1)
            f8c = LayerCalls(f8, dq, dk, dv, out)
            nst = min(S, 32)
            f8c.run_step(0, stream)
            e0.record()
            for s_ in range(1, nst):
                f8c.run_step(s_, stream)
            e1.record()
            torch.cuda.synchronize()
            f8_step = e0.elapsed_time(e1) / (nst - 1)
            rows8 = int(f8.kv_len.to(torch.int64).sum().item())
            f8.decode_attn(0, NL, dq[0], None, None, out)
            e0.record()
            for _ in range(10):
                f8.decode_attn(0, NL, dq[0], None, None, out)
            e1.record()
            torch.cuda.synchronize()
            f8_all = e0.elapsed_time(e1) / 10
            by8 = rows8 * 2 * d                          # one byte per element
            result["fp8_cache"] = {"evict_ms": f8_evict, "decode_step_us": f8_step * 1e3,
                                   "decode_GBps": by8 / (f8_step * 1e-3) / 1e9,
                                   "decode_all_layers_one_launch_us": f8_all * 1e3,
                                   "decode_all_layers_GBps": by8 / (f8_all * 1e-3) / 1e9,
                                   "speedup_of_decode_step_vs_bf16_cache": result["decode_step_us"] / (f8_step * 1e3)}
            f8.close()
            del f8, f8c
        except Exception as ex:
            result["fp8_cache"] = {"error": str(ex)[:200]}
        # the paged reduced cache (64-row pages, appended rows in pages taken on demand): eviction and decode step
        try:
            pgd = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=wl.budget,
                            dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=S, out_fp32=0, page_rows=64, device=dev)
            pg_evict = timed(lambda: pgd.evict(0, NL, q, k, v, mask))
            pgc = LayerCalls(pgd, dq, dk, dv, out)
            nst = min(S, 96)                             # far enough for every head to take a page
            pgc.run_step(0, stream)
            e0.record()
            for s_ in range(1, nst):
                pgc.run_step(s_, stream)
            e1.record()
            torch.cuda.synchronize()
            result["paged_cache"] = {"page_rows": 64, "evict_ms": pg_evict, "decode_step_us": e0.elapsed_time(e1) / (nst - 1) * 1e3,
                                     "capacity_rows_vs_contiguous": pgd.capacity / eng.capacity}
            pgd.close()
            del pgd, pgc
        except Exception as ex:
            result["paged_cache"] = {"error": str(ex)[:200]}
        # the prefill's last-window attention with the scores as a by-product (one pass over K and V, timed as the
        # producer it is), and what is left of the eviction after it: allocation, selection, gather
        try:
            wout = torch.empty(NL, B, Hq, W, d, dtype=wl.torch_dtype, device=dev)
            wlse = torch.empty(NL, B, Hq, W, dtype=torch.float32, device=dev)
            t_prod = timed(lambda: eng.window_attn_score(0, NL, q, k, v, mask, wout, wlse))
            t_rest = timed(lambda: (eng.allocate(0, NL), eng.select_gather(0, NL, k, v, mask)))
            kvb = 2 * NL * B * H * L * d * es
            result["evict_after_window_attn"] = {"window_attn_score_ms": t_prod, "window_attn_GBps": kvb / (t_prod * 1e-3) / 1e9,
                                                 "window_attn_frac_of_hbm_peak": kvb / (t_prod * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                                 "allocate_select_gather_ms": t_rest, "ctx_tokens_per_s": B * L / (t_rest * 1e-3),
                                                 "note": "the attention of the last W prompt positions is prefill work (K and V read once, out and "
                                                         "log-sum-exp written); psi, the statistics and pooled scores come out of the same pass"}
            del wout, wlse
        except Exception as ex:
            result["evict_after_window_attn"] = {"error": str(ex)[:200]}
        # eviction when the caller's prefill hands over the proxy rows' log-sum-exp (one pass over K).
        # The normalisers are made here with torch, outside the timed region, as a prefill kernel would.
        scale = 1.0 / (d ** 0.5)
        G = Hq // H
        lse = torch.empty(NL, B, Hq, W, dtype=torch.float32, device=dev)
        pos = torch.arange(L, device=dev)[None, None, :]
        rowpos = (L - W + torch.arange(W, device=dev))[None, :, None]
        for l in range(NL):
            for b in range(B):
                lg = torch.einsum("hgwd,hld->hgwl", q[l, b].view(H, G, W, d).float(), k[l, b].float()).mul_(scale)
                lg = lg.view(Hq, W, L).masked_fill_(pos > rowpos, float("-inf"))
                lse[l, b] = torch.logsumexp(lg, dim=-1)
                del lg
        for rep in range(2):
            e0.record()
            eng.score_lse(0, NL, q, k, mask, lse); eng.allocate(0, NL); eng.select_gather(0, NL, k, v, mask)
            e1.record()
        torch.cuda.synchronize()
        result["evict_with_row_lse"] = {"evict_ms": e0.elapsed_time(e1), "ctx_tokens_per_s": B * L / (e0.elapsed_time(e1) * 1e-3)}
        del lse
        # (c) the same decode kernel over the un-evicted cache (budget >= L keeps every token)
        try:
            full = MB.MadaKV(n_layers=NL, batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, ctx_len=L, window=W, budget=L,
                             dtype=wl.dtype, pool_k=wl.pool_k, max_new_tokens=1, out_fp32=0, layers_per_call=NL, device=dev)
            # psi buffers of this engine are not needed: free them before the big cache copy
            full.psi = full.psi_pool = None
            MB.madakv_select_gather(full.h, 0, NL, None, mask, None, k, v, full.kept_idx, full.kv_off, full.kv_len,
                                    full.k_c, full.v_c, full.select_ws)
            fc = LayerCalls(full, dq, dk, dv, out)
            torch.cuda.synchronize()
            for l, qp, kp, vp, off, ln, o in fc.args:
                fc.fn(fc.h, l, 1, C.c_void_p(qp), None, None, fc.kc, fc.vc, off, ln, o, fc.ws, fc.ws_bytes, stream)
            e0.record()
            reps = 3
            for _ in range(reps):
                for l, qp, kp, vp, off, ln, o in fc.args:
                    fc.fn(fc.h, l, 1, C.c_void_p(qp), None, None, fc.kc, fc.vc, off, ln, o, fc.ws, fc.ws_bytes, stream)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            by = NL * B * H * L * 2 * d * es
            result["decode_full_cache"] = {"us_per_step": ms * 1e3, "GBps": by / (ms * 1e-3) / 1e9,
                                           "frac_of_peak": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                           "speedup_of_evicted_cache": ms * 1e3 / result["decode_step_us"]}
            full.close()
            del full, fc
        except Exception as ex:                       # memory for the second cache may be short on a shared box
            result["decode_full_cache"] = {"error": str(ex)[:200]}

    if not a.no_extras and wl.budget < L and G_ * W <= 64:
        # re-eviction during generation: 64 decode steps, then every head back to its prompt-time length
        # (one-sweep scoring over the rows of the reduced cache, per-head split, selection, in-place compaction)
        try:
            eng.evict(0, NL, q, k, v, mask)
            nst = min(S, 64)
            for s_ in range(nst):
                calls.run_step(s_, stream)
            qr = dq[:W].permute(1, 2, 3, 0, 4).contiguous() if S >= W else torch.randn(NL, B, Hq, W, d, device=dev).to(wl.torch_dtype)
            rows_before = int(eng.kv_len.to(torch.int64).sum().item())
            eng.reevict_ws = torch.empty(MB.madakv_reevict_workspace_bytes(eng.h, NL), dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            e0.record(); eng.reevict(0, NL, qr, mask); e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            result["reevict"] = {"after_decode_steps": nst, "ms": ms, "cache_rows_before": rows_before,
                                 "cache_rows_after": int(eng.kv_len.to(torch.int64).sum().item()),
                                 "algorithmic_GBps": (rows_before * d * es + 4 * int(eng.kv_len.to(torch.int64).sum().item()) * d * es) / (ms * 1e-3) / 1e9,
                                 "note": "bytes = K rows of the grown cache read once for scoring + surviving K,V rows read and written"}
        except Exception as ex:
            result["reevict"] = {"error": str(ex)[:200]}

    if not a.no_extras and wl.name == "llava_16k":
        # the other named configurations that are large enough to time: the Qwen-shaped grouped-query model
        # (224 proxy rows per KV head: the two-sweep kernels with the LDS ring, and the MFMA decode kernel) and
        # the 128K context at both budgets of its sweep (two-level exchange, chunk-parallel statistics / selection)
        others = {}
        for key, (nm, bud) in {"qwen_gqa": ("qwen_gqa", None), "long_128k_budget_512": ("long_128k", 512),
                               "long_128k_budget_4096": ("long_128k", 4096)}.items():
            try:
                log(f"timing {key}")
                others[key] = time_config(nm, bud)
            except Exception as ex:
                others[key] = {"error": str(ex)[:200]}
        result["other_configs"] = others

    if not a.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        result["cpu_baseline"] = cpu_baseline(wl, q, k, v, masks, eng=eng, dq0=dq[0])
    else:
        result["cpu_baseline"] = None
    eng.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
