"""The synthetic input recipe: layouts, shapes, dtypes, determinism (CPU only)."""
import numpy as np
import pytest
import torch

from paper_2506_15724_amd import workloads as WL


def test_tiny_layout_is_the_fixed_one():
    wl = WL.CONFIGS["tiny"]
    m = WL.modality_mask(wl, 0)
    runs = [(0, 128), (1, 256), (0, 192), (1, 256), (0, 192)]
    want = np.concatenate([np.full(n, v, np.uint8) for v, n in runs])
    assert (m == want).all() and m.shape == (1024,)


@pytest.mark.parametrize("name,n_img,img_tokens", [("llava_layer", 12, 6912), ("llava_16k", 20, 11520), ("long_128k", 200, 115200)])
def test_fixed_image_layouts(name, n_img, img_tokens):
    wl = WL.CONFIGS[name]
    for b in range(2):
        m = WL.modality_mask(wl, b)
        assert m.shape == (wl.ctx_len,) and int(m.sum()) == img_tokens
        starts = np.flatnonzero(np.diff(np.concatenate([[0], m.astype(np.int8)])) == 1)
        assert len(starts) == n_img
        assert m[0] == 0 and (m[-wl.window:] == 0).all()
    assert (WL.modality_mask(wl, 0) != WL.modality_mask(wl, 1)).any()
    assert (WL.modality_mask(wl, 0) == WL.modality_mask(wl, 0)).all()


def test_variable_image_layout():
    wl = WL.CONFIGS["qwen_gqa"]
    m = WL.modality_mask(wl, 0)
    assert m.shape == (32768,) and m[0] == 0 and (m[-32:] == 0).all()
    d = np.diff(np.concatenate([[0], m.astype(np.int8), [0]]))
    lens = np.flatnonzero(d == -1) - np.flatnonzero(d == 1)
    assert lens.min() >= 64 and lens.max() <= 1280 and len(set(lens.tolist())) > 5


def test_layer_inputs_shapes_dtype_determinism():
    wl = WL.CONFIGS["tiny"]
    m = WL.modality_mask(wl, 0)
    q, k, v = WL.layer_inputs(wl, 0, 0, m)
    assert q.shape == (8, 16, 64) and k.shape == (8, 1024, 64) and v.shape == k.shape and k.dtype == torch.float32
    q2, k2, v2 = WL.layer_inputs(wl, 0, 0, m)
    assert torch.equal(k, k2) and torch.equal(q, q2) and torch.equal(v, v2)
    small = WL.CONFIGS["llava_layer"].scaled(ctx_len=2048, n_images=2, n_kv_heads=2, n_q_heads=4)
    ms = WL.modality_mask(small, 0)
    qs, ks, vs = WL.layer_inputs(small, 0, 0, ms)
    assert ks.dtype == torch.bfloat16 and qs.shape == (4, 32, 128)
    # heavy hitters: about 1% of key rows carry 4x the norm
    nrm = ks.float().norm(dim=-1)
    frac = (nrm > 2.5 * nrm.median()).float().mean().item()
    assert 0.003 < frac < 0.03
    qd, kn, vn = WL.decode_inputs(small, 0, 0, 3)
    assert qd.shape == (4, 128) and kn.shape == (2, 128) and vn.dtype == torch.bfloat16
    assert WL.to_f64(ks).dtype == np.float64


def test_layer_temperature_profile():
    wl = WL.CONFIGS["llava_16k"]
    t = [WL.layer_temperature(wl, l) for l in range(32)]
    assert t[0] == t[1] == t[30] == t[31] == 0.5 and max(t) > 1.4 and t[15] == t[16]
    assert WL.layer_temperature(WL.CONFIGS["tiny"], 0) == 1.0
