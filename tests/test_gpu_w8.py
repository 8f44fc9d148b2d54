"""Expert weights in 8 bits (E4M3 codes with fp32 row scales, bf16 activations) on the GPU against
the oracle, through the same C-ABI calls as the bf16 layer."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl
from gpu_util import TOL_OUT, DeviceLayer, out_to_f64, rel_err, run_gpu_layer, run_oracle_layer
from test_gpu_parity import check_layer, check_sampled_prefill

pytestmark = pytest.mark.gpu


def cfg_w8(**kw):
    # several row tiles with a ragged last one, K with a partial last chunk, E not a multiple of 16
    base = dict(name="w8_small", T=37, H=272, E=10, I=144, k_big=4, k_little=2, shared_I=(80,),
                dtype="bf16w8", gate_std=0.3, w_std=0.1, gate_bias_std=0.5)
    base.update(kw)
    return wl.LayerConfig(**base)


@pytest.mark.parametrize("r", [0.0, 0.3, 1.0])
def test_small_ragged_layer(r):
    check_layer(cfg_w8(fallback_ratio=r), seed=1)


def test_long_contractions_and_many_token_blocks():
    # K beyond one 512-wide chunk in both projections, several token blocks per expert
    check_layer(cfg_w8(T=200, H=1040, E=4, I=656, k_big=3, k_little=1, shared_I=(1200, 48)), seed=2)
    check_layer(cfg_w8(T=97, H=512, E=6, I=1024, k_big=4, k_little=2, shared_I=()), seed=3)


@pytest.mark.parametrize("T", [1, 8, 64])
def test_fine60_decode_full_size(T):
    check_layer(wl.CONFIGS["fine60_decode"].with_(T=T, dtype="bf16w8"), seed=0)


@pytest.mark.parametrize("T,seed", [(256, 4), (300, 6), (700, 7)])
def test_tiled_regime_small_ragged(T, seed):
    # T >= 256: the LDS-tiled kernel; ragged token tiles, weight tiles and K tails (K = 272, 144, 80: a
    # partial last chunk of 64), experts without tokens, a shared expert cut into K chunks
    check_layer(cfg_w8(T=T, fallback_ratio=0.3), seed=seed)
    check_layer(cfg_w8(T=T, H=528, E=5, I=400, k_big=2, k_little=1, shared_I=(1200, 48), fallback_ratio=0.5), seed=seed + 10)


def test_tiled_regime_every_code():
    """T >= 256: all 256 codes in every position of a 16-byte column, in gate rows of one expert."""
    check_every_code(T=256)


def test_fine64_prefill_full_size_sampled():
    cfg = wl.CONFIGS["fine64_prefill"].with_(dtype="bf16w8")
    layer = wl.make_layer(cfg, seed=0)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = run_gpu_layer(dl, logits=logits)
    _, tokens = check_sampled_prefill(cfg, layer, b, logits, n_random=160, seed=0)
    assert len(tokens) >= 256


def test_every_code_reaches_the_sum_with_its_value():
    check_every_code(T=16)


def check_every_code(T):
    """One expert whose W_gate rows hold all 256 codes: the layer output equals the oracle's, i.e.
    the kernel's widening agrees with the format for every code that is not NaN."""
    cfg = cfg_w8(T=T, H=256, E=2, I=16, k_big=1, k_little=1, shared_I=())
    layer = wl.make_layer(cfg, seed=5)
    codes = np.arange(256, dtype=np.uint8)
    codes[codes == 0x7F] = 0x7E
    codes[codes == 0xFF] = 0xFE
    for e in range(cfg.E):
        b = layer.expert_w[e]
        for i in range(cfg.I):
            b[i * cfg.H:(i + 1) * cfg.H] = np.roll(codes, 17 * i + e)
        # small scales keep silu(g) * u in a range where bf16 storage of h is harmless
        sc = b[3 * cfg.H * cfg.I:].view(np.float32)
        sc[:cfg.I] = 2.0 ** -12
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = run_gpu_layer(dl, conf=dl.conf, logits=logits)
    ref = run_oracle_layer(layer, logits=logits)
    assert rel_err(b.y[:int(ref["expert_offsets"][-1])].cpu().numpy(), ref["y"]) <= TOL_OUT
    assert rel_err(out_to_f64(b.out), ref["out"]) <= TOL_OUT


@pytest.mark.parametrize("T", [48, 300])
def test_little_pass_then_fallback_pass(T):
    # T = 300: both passes in the tiled regime, the second with routed experts only
    cfg = cfg_w8(T=T, shared_I=(80,))
    layer = wl.make_layer(cfg, seed=8)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = mm.StepBuffers(cfg)
    b.logits.copy_(torch.from_numpy(logits))
    ones = torch.full((cfg.T,), 2.0, device="cuda")
    mm.layer_step(b, dl.x, dl.Wg, dl.gate_bias, ones, dl.table, dl.shared, logits_given=True)
    mm.fallback_step(b, dl.x, dl.conf, dl.table)
    torch.cuda.synchronize()
    ref = run_oracle_layer(layer, logits=logits)
    assert rel_err(out_to_f64(b.out), ref["out"]) <= TOL_OUT


def test_limits_and_blob_size():
    cfg = cfg_w8()
    c = mm.make_config(cfg)
    assert mm.moe_expert_blob_bytes(c, cfg.I) == wl.w8_blob_bytes(cfg.H, cfg.I) == wl.make_expert_blob(cfg, 0, 0).size
    assert mm.moe_expert_blob_bytes(c, cfg.shared_I[0]) == wl.w8_blob_bytes(cfg.H, cfg.shared_I[0])
    assert mm.moe_expert_blob_bytes(mm.make_config(cfg.with_(dtype="bf16")), cfg.I) == 6 * cfg.H * cfg.I
    assert mm.moe_expert_blob_bytes(c, 12) == 0
    lib = mm.load_library()
    for bad in (cfg.with_(H=264), cfg.with_(I=136), cfg.with_(shared_I=(72,))):
        cb = mm.make_config(bad)
        rc = lib.moe_combine(ctypes.byref(cb), None, None, None, None, None, None, None)
        assert rc == -3, (bad, rc)
