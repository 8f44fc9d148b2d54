"""Pins of the oracle's 8-bit expert weights (E4M3 codes with fp32 row scales), CPU only: the
decoder against the format's closed forms and against torch's float8_e4m3fn, the feed-forward and
the whole layer against a dense numpy evaluation that dequantises with torch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import workloads as wl

from test_oracle_pins import np_softmax, np_topk_order


def torch_decode(codes: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(codes, np.uint8)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def dequant(blob: np.ndarray, H: int, I: int):
    """(W_gate [I,H], W_up [I,H], W_down [H,I]) in float64 from an 8-bit blob, decoded by torch."""
    n = 3 * H * I
    q = torch_decode(blob[:n])
    s = blob[n:].view(np.float32).astype(np.float64)
    assert s.size == 2 * I + H
    return (q[:I * H].reshape(I, H) * s[:I, None], q[I * H:2 * I * H].reshape(I, H) * s[I:2 * I, None],
            q[2 * I * H:].reshape(H, I) * s[2 * I:, None])


def dense_swiglu(xf, blob, H, I):
    Wg, Wu, Wd = dequant(blob, H, I)
    g, u = xf @ Wg.T, xf @ Wu.T
    return ((g / (1.0 + np.exp(-g))) * u) @ Wd.T


def test_e4m3_decoder_closed_forms_and_torch():
    codes = np.arange(256, dtype=np.uint8)
    v = oracle.e4m3_decode(codes)
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x38] == 1.0 and v[0x40] == 2.0 and v[0x30] == 0.5 and v[0xB8] == -1.0
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0            # largest finite: 1.75 * 2^8
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9  # subnormals: m/8 * 2^-6
    assert v[0x08] == 2.0 ** -6                               # smallest normal
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.isfinite(np.delete(v, [0x7F, 0xFF])).all()
    pos = v[:0x7F]
    assert (np.diff(pos) > 0).all()                            # codes order like their values
    ref = torch_decode(codes)
    ok = ~np.isnan(ref)
    assert np.array_equal(v[ok], ref[ok]) and np.array_equal(np.isnan(v), np.isnan(ref))


def w8_cfg(**kw):
    base = dict(name="w8", T=21, H=48, E=6, I=40, k_big=3, k_little=1, shared_I=(24,), dtype="bf16w8",
                gate_std=0.3, w_std=0.2, gate_bias_std=0.3)
    base.update(kw)
    return wl.LayerConfig(**base)


def test_blob_layout_and_generator():
    cfg = w8_cfg()
    b = wl.make_expert_blob(cfg, 3, 2)
    assert b.dtype == np.uint8 and b.size == oracle.w8_blob_bytes(cfg.H, cfg.I) == wl.w8_blob_bytes(cfg.H, cfg.I)
    Wg, Wu, Wd = dequant(b, cfg.H, cfg.I)
    # a row's largest magnitude sits on the largest finite code, and the rows resemble N(0, w_std)
    for W in (Wg, Wu, Wd):
        assert 0.1 < W.std() < 0.3
    n = 3 * cfg.H * cfg.I
    q = torch_decode(b[:n])
    assert np.abs(q).max() == 448.0 and not np.isnan(q).any()
    assert (np.abs(q[:cfg.I * cfg.H].reshape(cfg.I, cfg.H)).max(axis=1) == 448.0).all()


@pytest.mark.parametrize("tok", [None, [5, 0, 20, 5]])
def test_feed_forward_equals_dense_numpy(tok):
    cfg = w8_cfg()
    layer = wl.make_layer(cfg, seed=4)
    xf = wl.as_f32(layer.x).astype(np.float64)
    for blob, I in ((layer.expert_w[1], cfg.I), (layer.shared_w[0], cfg.shared_I[0])):
        y = oracle.swiglu_rows(layer.x, blob, I, None if tok is None else np.array(tok, np.int32))
        ref = dense_swiglu(xf if tok is None else xf[tok], blob, cfg.H, I)
        np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("renorm", [False, True])
def test_layer_equals_dense_numpy(renorm):
    cfg = w8_cfg(renorm=renorm)
    layer = wl.make_layer(cfg, seed=7)
    r = oracle.moe_layer(layer.x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I, layer.shared_w, cfg.shared_I,
                         layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm)
    xf = wl.as_f32(layer.x).astype(np.float64)
    logits = (xf @ wl.as_f32(layer.Wg).astype(np.float64).T + layer.gate_bias.astype(np.float64)).astype(np.float32)
    p, order = np_softmax(logits), np_topk_order(logits)
    important = ~(layer.conf > np.float32(cfg.gamma))
    dense = np.stack([dense_swiglu(xf, b, cfg.H, cfg.I) for b in layer.expert_w], axis=1)
    out = np.zeros_like(xf)
    for t in range(cfg.T):
        sel = order[t, :(cfg.k_big if important[t] else cfg.k_little)]
        w = p[t, sel]
        if renorm:
            w = w / w.sum()
        out[t] = (w.astype(np.float32).astype(np.float64)[:, None] * dense[t, sel]).sum(axis=0)
    out += dense_swiglu(xf, layer.shared_w[0], cfg.H, cfg.shared_I[0])
    np.testing.assert_allclose(r["out"], out, rtol=1e-9, atol=1e-10)


def test_quantised_layer_is_close_to_the_unquantised_one():
    """The same random weights stored in bf16 and in 8 bits: 3 mantissa bits per weight, errors
    averaging over the contraction -- a misplaced scale or matrix would be far outside."""
    c8 = w8_cfg(T=16, shared_I=())
    c16 = c8.with_(dtype="bf16")
    l8, l16 = wl.make_layer(c8, seed=9), wl.make_layer(c16, seed=9)
    assert np.array_equal(l8.x, l16.x) and np.array_equal(l8.Wg, l16.Wg)
    y8 = oracle.swiglu_rows(l8.x, l8.expert_w[0], c8.I)
    y16 = oracle.swiglu_rows(l16.x, l16.expert_w[0], c16.I)
    rel = np.linalg.norm(y8 - y16) / np.linalg.norm(y16)
    assert 1e-4 < rel < 0.08, rel
