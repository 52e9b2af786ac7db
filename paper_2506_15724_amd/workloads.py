"""Seeded synthetic inputs shaped like the paper's long multimodal workloads.

This module only draws inputs (modality layouts, Q/K/V, decode rows).  It holds none
of the method's arithmetic and is the one piece that both the HIP path's tests and the
CPU checker's tests may use.  The paper evaluates on MileBench prompts (on average
15.2 images per sample, Sec. 4.1) run through LLaVA-1.5 / Qwen2.5-VL; neither the
benchmark nor the weights are used here, and these generators stand in for them:
interleaved text / image runs with LLaVA-sized image blocks, Gaussian activations and
a per-head modality preference injected through a shared bias direction.

Tensors are made with torch on the requested device (CPU for small cases, the GPU for
the large ones, whose bits are then copied back for the checker), one generator seed
per (config, layer, batch item).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

BASE_SEED = 20250615


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_len: int
    window: int
    budget: int
    dtype: str                 # "fp32" | "bf16"
    pool_k: int
    decode_steps: int
    image_tokens: tuple        # (lo, hi) image-run length, log-uniform if lo != hi
    text_tokens: tuple         # (lo, hi) text-run length, uniform
    n_images: int              # 0 = add runs until the context is full
    heavy_hitters: float       # fraction of key positions scaled by 4
    bimodal_pref: bool
    fixed_layout: tuple = ()   # explicit (modality, length) runs
    cfg_id: int = 0
    n_modalities: int = 2      # > 2: the non-text runs cycle through modality ids 1 .. M-1

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five configurations named for this hot path.  Budgets are tokens per KV head.
CONFIGS = {
    "tiny": Workload("tiny", 1, 1, 8, 8, 64, 1024, 16, 256, "fp32", 1, 8, (256, 256), (128, 192), 2, 0.0, False,
                     fixed_layout=((0, 128), (1, 256), (0, 192), (1, 256), (0, 192)), cfg_id=1),
    "llava_layer": Workload("llava_layer", 1, 1, 32, 32, 128, 8192, 32, 1024, "bf16", 7, 16, (576, 576), (32, 256),
                            12, 0.01, False, cfg_id=2),
    "llava_16k": Workload("llava_16k", 32, 4, 32, 32, 128, 16384, 32, 2048, "bf16", 7, 128, (576, 576), (32, 256),
                          20, 0.01, False, cfg_id=3),
    "qwen_gqa": Workload("qwen_gqa", 28, 1, 28, 4, 128, 32768, 32, 2048, "bf16", 7, 16, (64, 1280), (16, 512),
                         0, 0.01, False, cfg_id=4),
    "long_128k": Workload("long_128k", 1, 1, 32, 32, 128, 131072, 64, 4096, "bf16", 7, 256, (576, 576), (32, 256),
                          200, 0.01, True, cfg_id=5),
}


def _np_rng(wl: Workload, *key) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[BASE_SEED + 1000003 * wl.cfg_id, _mix(key)]))


def _mix(key) -> int:
    h = 1469598103934665603
    for x in key:
        h = ((h ^ (int(x) + 0x9E37)) * 1099511628211) % (1 << 63)
    return h


def _torch_gen(wl: Workload, device, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((BASE_SEED + 1000003 * wl.cfg_id + 7919 * _mix(key)) % (1 << 62))
    return g


def _spread(total: int, weights: np.ndarray, floor_each: int = 1) -> np.ndarray:
    """Integers proportional to weights, each >= floor_each, summing to total."""
    n = len(weights)
    spare = total - floor_each * n
    assert spare >= 0, "context too short for this layout"
    raw = weights / weights.sum() * spare
    out = np.floor(raw).astype(np.int64)
    rest = spare - int(out.sum())
    order = np.argsort(-(raw - out), kind="stable")
    out[order[:rest]] += 1
    return out + floor_each


def modality_mask(wl: Workload, b: int) -> np.ndarray:
    """uint8[L]: 0 = text, 1 = image.  Alternating runs, text first and last, the last
    text run at least `window` long so that the proxy tokens are text."""
    L = wl.ctx_len
    if wl.fixed_layout:
        parts = [np.full(n, m, np.uint8) for m, n in wl.fixed_layout]
        mask = np.concatenate(parts)
        assert mask.shape[0] == L
        return mask
    r = _np_rng(wl, 1, b)
    if wl.n_images > 0:
        img = [int(wl.image_tokens[0])] * wl.n_images
        n_text = wl.n_images + 1
        text_total = L - sum(img)
        draw = r.integers(wl.text_tokens[0], wl.text_tokens[1] + 1, size=n_text).astype(np.float64)
        text = _spread(text_total - wl.window, draw, 1)
        text[-1] += wl.window
    else:
        img, text, used = [], [], 0
        lo, hi = wl.image_tokens
        while True:
            t = int(r.integers(wl.text_tokens[0], wl.text_tokens[1] + 1))
            i = int(round(math.exp(r.uniform(math.log(lo), math.log(hi)))))
            if used + t + i + wl.text_tokens[1] + wl.window >= L:
                text.append(L - used)
                break
            text.append(t); img.append(i); used += t + i
        text = np.asarray(text)
    parts = []
    for j in range(len(img)):
        parts.append(np.zeros(int(text[j]), np.uint8))
        parts.append(np.full(int(img[j]), 1 + j % (wl.n_modalities - 1), np.uint8))
    parts.append(np.zeros(int(text[len(img)]), np.uint8))
    mask = np.concatenate(parts)
    assert mask.shape[0] == L and (mask[L - wl.window:] == 0).all()
    return mask


def layer_temperature(wl: Workload, l: int) -> float:
    """Scale on the window queries: flat attention (0.5) in the first and last two
    layers, sharp (1.5) mid-stack, linear in between, so that a multi-layer run sees
    both over- and under-drafts of the layer budget."""
    n = wl.n_layers
    if n < 6:
        return 1.0
    if l < 2 or l >= n - 2:
        return 0.5
    mid = (n - 1) / 2.0
    span = mid - 2.0
    return 0.5 + (1.0 - abs(l - mid) / span) if span > 0 else 1.5


def head_preferences(wl: Workload, l: int, b: int, device="cpu"):
    """(p[H] preference for text in [0,1], u[H,d] bias direction with |u|^2 = 2 sqrt(d))."""
    g = _torch_gen(wl, "cpu", 2, l, b)
    H, d = wl.n_kv_heads, wl.head_dim
    if wl.bimodal_pref:
        p = torch.where(torch.rand(H, generator=g) < 0.5, 0.05, 0.95)
    else:
        p = torch.rand(H, generator=g)
    u = torch.randn(H, d, generator=g)
    u = u / u.norm(dim=1, keepdim=True) * math.sqrt(2.0 * math.sqrt(d))
    return p.to(device), u.to(device)


def modality_coefficients(wl: Workload, l: int, b: int, device="cpu"):
    """coef[H, M]: how strongly the keys of each modality carry the head's bias direction.
    Two modalities: (2 p_h, 2 (1 - p_h)).  More: M times a seeded point of the simplex."""
    p, _ = head_preferences(wl, l, b, device)
    if wl.n_modalities == 2:
        return torch.stack([2.0 * p, 2.0 * (1.0 - p)], dim=1)
    g = _torch_gen(wl, "cpu", 6, l, b)
    e = -torch.log(torch.rand(wl.n_kv_heads, wl.n_modalities, generator=g).clamp_min(1e-6))
    return (wl.n_modalities * e / e.sum(dim=1, keepdim=True)).to(device)


def layer_inputs(wl: Workload, l: int, b: int, mask: np.ndarray, device="cpu"):
    """(q_win[Hq,W,d], k[H,L,d], v[H,L,d]) of one layer of one batch item, in wl's dtype.
    K,V,Q ~ N(0,1); the head bias u_h is added to the window queries, and to the keys
    scaled by 2 p_h on text positions and 2 (1 - p_h) on image positions; a seeded
    fraction of key positions per head is multiplied by 4 (heavy hitters)."""
    H, Hq, d, L, W = wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.ctx_len, wl.window
    G = Hq // H
    g = _torch_gen(wl, device, 3, l, b)
    p, u = head_preferences(wl, l, b, device)
    if wl.n_modalities == 2:
        m = torch.from_numpy(mask.astype(np.float32)).to(device)             # 1 on image
        coef = 2.0 * (p[:, None] * (1.0 - m)[None, :] + (1.0 - p)[:, None] * m[None, :])   # [H, L]
    else:
        table = modality_coefficients(wl, l, b, device)                      # [H, M]
        coef = table[:, torch.from_numpy(mask.astype(np.int64)).to(device)]  # [H, L]
    k = torch.randn(H, L, d, generator=g, device=device)
    k += coef[:, :, None] * u[:, None, :]
    if wl.heavy_hitters > 0:
        hh = torch.rand(H, L, generator=g, device=device) < wl.heavy_hitters
        k = torch.where(hh[:, :, None], 4.0 * k, k)
    v = torch.randn(H, L, d, generator=g, device=device)
    q = torch.randn(Hq, W, d, generator=g, device=device)
    q += u.repeat_interleave(G, dim=0)[:, None, :]
    q *= layer_temperature(wl, l)
    dt = wl.torch_dtype
    return q.to(dt), k.to(dt), v.to(dt)


def decode_inputs(wl: Workload, l: int, b: int, step: int, device="cpu"):
    """(q[Hq,d], k_new[H,d], v_new[H,d]) of one decode step (new tokens are text)."""
    H, Hq, d = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    G = Hq // H
    g = _torch_gen(wl, device, 4, l, b, step)
    p, u = head_preferences(wl, l, b, device)
    q = torch.randn(Hq, d, generator=g, device=device) + u.repeat_interleave(G, dim=0)
    kn = torch.randn(H, d, generator=g, device=device) + 2.0 * p[:, None] * u
    vn = torch.randn(H, d, generator=g, device=device)
    dt = wl.torch_dtype
    return q.to(dt), kn.to(dt), vn.to(dt)


def decode_inputs_all(wl: Workload, step: int, device="cpu"):
    """(q[NL,B,Hq,d], k_new[NL,B,H,d], v_new[NL,B,H,d]) of one decode step for the whole model,
    drawn in one go (one generator per step); same recipe as decode_inputs."""
    NL, B, H, Hq, d = wl.n_layers, wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    G = Hq // H
    g = _torch_gen(wl, device, 5, step)
    ps, us = zip(*[zip(*[head_preferences(wl, l, b, device) for b in range(B)]) for l in range(NL)])
    p = torch.stack([torch.stack(x) for x in ps])                    # [NL, B, H]
    u = torch.stack([torch.stack(x) for x in us])                    # [NL, B, H, d]
    q = torch.randn(NL, B, Hq, d, generator=g, device=device) + u.repeat_interleave(G, dim=2)
    kn = torch.randn(NL, B, H, d, generator=g, device=device) + 2.0 * p[..., None] * u
    vn = torch.randn(NL, B, H, d, generator=g, device=device)
    dt = wl.torch_dtype
    return q.to(dt).contiguous(), kn.to(dt).contiguous(), vn.to(dt).contiguous()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of a tensor's values on the host (what the checker reads)."""
    return t.detach().to("cpu", torch.float64).numpy()
