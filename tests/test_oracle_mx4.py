"""Pins of the oracle's MXFP4 expert weights (OCP microscaling: E2M1 elements, one E8M0 scale per
block of 32 along the contraction), CPU only: the element decoder against the value table of the
format (tests/golden/mxfp4_element_values.txt), the scale decoder against torch's float8_e8m0fnu
and closed forms, the feed-forward and the whole layer against a dense numpy evaluation that
unpacks and dequantises on its own, layout mistakes (nibble order, block direction) shown to
fail, and closeness to the unquantised layer."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import workloads as wl

from test_oracle_pins import np_softmax, np_topk_order

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "mxfp4_element_values.txt")


def table_values():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        code, v = line.split()
        vals[int(code, 2)] = float(v)
    assert len(vals) == 16
    return vals


TABLE = table_values()


def unpack(packed: np.ndarray, low_first=True) -> np.ndarray:
    """[rows, K/2] bytes -> [rows, K] table values; element 2i in the low four bits of byte i."""
    lo, hi = packed & 15, packed >> 4
    pair = np.stack([lo, hi] if low_first else [hi, lo], axis=-1).reshape(packed.shape[0], -1)
    lut = np.array([TABLE[c] for c in range(16)], np.float64)
    return lut[pair]


def e8m0_torch(b: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(b, np.uint8)).view(torch.float8_e8m0fnu).to(torch.float32) \
        .to(torch.float64).numpy()


def dequant(blob: np.ndarray, H: int, I: int, low_first=True, along_k=True):
    """(W_gate [I,H], W_up [I,H], W_down [H,I]) in float64 from an MXFP4 blob."""
    HI = H * I
    assert blob.size == 3 * HI // 2 + 3 * HI // 32
    q, s = blob[:3 * HI // 2], blob[3 * HI // 2:]
    out = []
    for m, (rows, K) in enumerate(((I, H), (I, H), (H, I))):
        v = unpack(q[m * HI // 2:(m + 1) * HI // 2].reshape(rows, K // 2), low_first)
        sc = e8m0_torch(s[m * HI // 32:(m + 1) * HI // 32])
        if along_k:
            v = v * np.repeat(sc.reshape(rows, K // 32), 32, axis=1)
        else:                                   # (a wrong reading: blocks of 32 rows of one column)
            v = v * np.repeat(sc.reshape(rows // 32, K), 32, axis=0)
        out.append(v)
    return out


def dense_swiglu(xf, blob, H, I, **kw):
    Wg, Wu, Wd = dequant(blob, H, I, **kw)
    g, u = xf @ Wg.T, xf @ Wu.T
    return ((g / (1.0 + np.exp(-g))) * u) @ Wd.T


def test_element_decoder_equals_the_format_table():
    v = oracle.e2m1_decode(np.arange(16, dtype=np.uint8))
    for c in range(16):
        assert v[c] == TABLE[c] and np.signbit(v[c]) == np.signbit(TABLE[c]), c
    # only the low four bits of a byte are the code
    assert np.array_equal(oracle.e2m1_decode(np.arange(16, dtype=np.uint8) | 0xA0), v)
    # what the format says in words: sign-symmetric, magnitudes ascending with the code, largest 6
    assert np.array_equal(v[8:], -v[:8]) and (np.diff(v[:8]) > 0).all() and v[7] == 6.0 and v[1] == 0.5


def test_scale_decoder_closed_forms_and_torch():
    b = np.arange(256, dtype=np.uint8)
    v = oracle.e8m0_decode(b)
    assert v[127] == 1.0 and v[128] == 2.0 and v[126] == 0.5 and v[0] == 2.0 ** -127 and v[254] == 2.0 ** 127
    assert np.isnan(v[255]) and np.isfinite(v[:255]).all()
    assert np.array_equal(v[1:255] / v[:254], np.full(254, 2.0))
    ref = e8m0_torch(b)
    assert np.array_equal(v[:255], ref[:255]) and np.isnan(ref[255])


def mx_cfg(**kw):
    base = dict(name="mx4", T=21, H=64, E=6, I=96, k_big=3, k_little=1, shared_I=(32,), dtype="bf16mx4",
                gate_std=0.3, w_std=0.2, gate_bias_std=0.3)
    base.update(kw)
    return wl.LayerConfig(**base)


def test_blob_layout_and_generator():
    cfg = mx_cfg()
    b = wl.make_expert_blob(cfg, 3, 2)
    assert b.dtype == np.uint8 and b.size == oracle.mx4_blob_bytes(cfg.H, cfg.I) == wl.mx4_blob_bytes(cfg.H, cfg.I)
    Wg, Wu, Wd = dequant(b, cfg.H, cfg.I)
    for W in (Wg, Wu, Wd):
        assert 0.1 < W.std() < 0.3                      # the rows resemble N(0, w_std)
    # every block's largest magnitude sits in the element's top binade (4 or 6 times the scale)
    HI = cfg.H * cfg.I
    top = np.abs(unpack(b[:HI // 2].reshape(cfg.I, cfg.H // 2))).reshape(cfg.I, cfg.H // 32, 32).max(axis=2)
    assert np.isin(top, (4.0, 6.0)).all()
    # the generator rounds to the nearest element value (ties to the even code), saturating at 6
    m = np.array([[0.24, 0.25, 0.26, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 5.1, 6.0, -0.75, -5.0, 0.0, 4.0, 2.9] + [0.0] * 16])
    codes, scales = wl.quantize_rows_mx4(m)
    assert scales[0, 0] == 127                          # largest magnitude 6 = 1.5 * 2^2: scale 2^0
    want = [0.0, 0.0, 0.5, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, 6.0, 6.0, -1.0, -4.0, 0.0, 4.0, 3.0]
    assert unpack(codes)[0, :16].tolist() == want
    codes, scales = wl.quantize_rows_mx4(m * 1024.0)    # a power of two moves into the scale alone
    assert scales[0, 0] == 127 + 10 and unpack(codes)[0, :16].tolist() == want


@pytest.mark.parametrize("tok", [None, [5, 0, 20, 5]])
def test_feed_forward_equals_dense_numpy(tok):
    cfg = mx_cfg()
    layer = wl.make_layer(cfg, seed=4)
    xf = wl.as_f32(layer.x).astype(np.float64)
    for blob, I in ((layer.expert_w[1], cfg.I), (layer.shared_w[0], cfg.shared_I[0])):
        y = oracle.swiglu_rows(layer.x, blob, I, None if tok is None else np.array(tok, np.int32))
        ref = dense_swiglu(xf if tok is None else xf[tok], blob, cfg.H, I)
        np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-12)
        # the two plausible layout mistakes are far away
        for kw in (dict(low_first=False), dict(along_k=False)):
            if kw.get("along_k") is False and (I % 32 or cfg.H % 32):
                continue
            bad = dense_swiglu(xf if tok is None else xf[tok], blob, cfg.H, I, **kw)
            assert np.linalg.norm(bad - y) > 0.3 * np.linalg.norm(y)


@pytest.mark.parametrize("renorm", [False, True])
def test_layer_equals_dense_numpy(renorm):
    cfg = mx_cfg(renorm=renorm)
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
    """The same random weights stored in bf16 and in MXFP4: one mantissa bit per weight, errors
    averaging over the contraction -- a misplaced scale or matrix would be far outside."""
    c4 = mx_cfg(T=16, shared_I=(), H=256, I=128)
    c16 = c4.with_(dtype="bf16")
    l4, l16 = wl.make_layer(c4, seed=9), wl.make_layer(c16, seed=9)
    assert np.array_equal(l4.x, l16.x) and np.array_equal(l4.Wg, l16.Wg)
    y4 = oracle.swiglu_rows(l4.x, l4.expert_w[0], c4.I)
    y16 = oracle.swiglu_rows(l16.x, l16.expert_w[0], c16.I)
    rel = np.linalg.norm(y4 - y16) / np.linalg.norm(y16)
    assert 0.02 < rel < 0.4, rel


def test_a_nan_scale_poisons_its_rows_only():
    cfg = mx_cfg(shared_I=())
    layer = wl.make_layer(cfg, seed=2)
    blob = layer.expert_w[0].copy()
    HI = cfg.H * cfg.I
    blob[3 * HI // 2 + 5 * (cfg.H // 32)] = 255            # first block of gate row 5
    y = oracle.swiglu_rows(layer.x, blob, cfg.I)
    assert np.isnan(y).all()                               # h[:, 5] is NaN and feeds every output column
    blob = layer.expert_w[0].copy()
    blob[3 * HI // 2 + 2 * (HI // 32) + 7 * (cfg.I // 32)] = 255   # first block of down row 7
    y = oracle.swiglu_rows(layer.x, blob, cfg.I)
    assert np.isnan(y[:, 7]).all() and np.isfinite(np.delete(y, 7, axis=1)).all()
