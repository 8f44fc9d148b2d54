"""moe_layer_decode (one decode step of the layer in one kernel launch) against the oracle and
against the four separate calls: selection, importance flags and every dispatch array bit-exact
given the same gate logits, the layer output within the output tolerance, y / shared_out / out
identical to the separate calls (same arithmetic in the same order), and no wait inside the
kernel ever giving up."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl
from gpu_util import TOL_OUT, DeviceLayer, out_to_f64, rel_err, run_oracle_layer

pytestmark = pytest.mark.gpu


def i32(t):
    return t.cpu().numpy().astype(np.int32)


def check_step(cfg, seed, logits_given=True, conf="layer", steps=1, check_separate=True):
    layer = wl.make_layer(cfg, seed=seed)
    dl = DeviceLayer(layer)
    print(f"decode step: {cfg.name} T={cfg.T} E={cfg.E} H={cfg.H} I={cfg.I} shared={cfg.shared_I} "
          f"dtype={cfg.dtype} renorm={cfg.renorm} seed={seed}", flush=True)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    c = dl.conf if isinstance(conf, str) else conf
    conf_h = layer.conf if isinstance(conf, str) else None
    b = mm.StepBuffers(cfg)
    for it in range(steps):                                  # the same workspace again: the counters are back at zero
        b.y.fill_(float("nan"))
        b.out.fill_(float("nan"))
        if logits_given:
            b.logits.copy_(torch.from_numpy(logits))
        mm.layer_decode_step(b, dl.x, dl.Wg, dl.gate_bias, c, dl.table, dl.shared, logits_given=logits_given)
        torch.cuda.synchronize()
        assert mm.moe_layer_decode_status(b.lws) == 0, "a wait inside the kernel gave up"
        ref = oracle.moe_layer(layer.x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I, layer.shared_w, cfg.shared_I,
                               conf_h, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm,
                               logits=logits if logits_given else b.logits.cpu().numpy())
        assert np.array_equal(i32(b.topk_idx), ref["topk_idx"])
        assert np.array_equal(b.important.cpu().numpy(), ref["important"])
        assert np.array_equal(i32(b.k_t), ref["k_t"])
        assert np.array_equal(i32(b.expert_offsets), ref["expert_offsets"])
        assert np.array_equal(i32(b.sorted_token), ref["sorted_token"])
        assert np.array_equal(i32(b.sorted_rank), ref["sorted_rank"])
        assert np.array_equal(i32(b.inv_pos), ref["inv_pos"])
        assert np.abs(b.topk_w.cpu().numpy() - ref["topk_w"]).max() <= 2e-6
        e = rel_err(out_to_f64(b.out), ref["out"])
        assert e <= TOL_OUT, (it, e)
    if check_separate:
        b2 = mm.StepBuffers(cfg)
        if logits_given:
            b2.logits.copy_(torch.from_numpy(logits))
        mm.layer_step(b2, dl.x, dl.Wg, dl.gate_bias, c, dl.table, dl.shared, logits_given=logits_given)
        torch.cuda.synchronize()
        P = int(b2.expert_offsets[-1])
        assert torch.equal(b.logits, b2.logits)
        assert torch.equal(b.topk_w, b2.topk_w)
        assert torch.equal(b.y[:P], b2.y[:P])
        if b.shared_out is not None:
            assert torch.equal(b.shared_out, b2.shared_out)
        assert torch.equal(b.out, b2.out)
    return b


def cfg_small(**kw):
    base = dict(name="dsmall", T=37, H=264, E=10, I=136, k_big=4, k_little=2, shared_I=(72,), dtype="bf16",
                renorm=False, gate_std=0.3, w_std=0.1, fallback_ratio=0.3)
    base.update(kw)
    return wl.LayerConfig(**base)


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 33, 64])
def test_small_ragged_layers(T):
    check_step(cfg_small(T=T), seed=T, steps=2)


@pytest.mark.parametrize("kw", [dict(shared_I=()), dict(shared_I=(72, 40)), dict(renorm=True), dict(E=1, k_big=1, k_little=1),
                                dict(E=200, k_big=6, k_little=3, T=21), dict(H=1032, I=520, shared_I=(2064,), T=40),
                                dict(fallback_ratio=0.0), dict(fallback_ratio=1.0), dict(k_big=16, k_little=8, E=20, T=64)])
def test_shapes_and_modes(kw):
    check_step(cfg_small(**kw), seed=3)


def test_router_computed_in_the_kernel():
    """Without given logits the kernel computes the router dot products itself: same bits as the
    stand-alone router, selection checked against the oracle on those logits."""
    check_step(cfg_small(T=64, gate_bias_std=1.0), seed=8, logits_given=False, steps=2)
    check_step(cfg_small(T=3, H=2048, E=60, shared_I=()), seed=9, logits_given=False)


def test_all_tokens_important_without_confidences():
    check_step(cfg_small(T=24), seed=4, conf=None)


@pytest.mark.parametrize("T", [1, 8, 32, 64])
def test_fine60_decode_full_size(T):
    cfg = wl.CONFIGS["fine60_decode"].with_(T=T)
    check_step(cfg, seed=0, logits_given=False, steps=2)


def test_8_bit_expert_weights():
    check_step(cfg_small(T=19, H=272, I=144, shared_I=(80,), dtype="bf16w8"), seed=5, steps=2)
    check_step(wl.CONFIGS["fine60_decode"].with_(T=8, dtype="bf16w8"), seed=1, logits_given=False)


def test_limits():
    cfg = cfg_small(T=65)
    c = mm.make_config(cfg)
    assert mm.moe_layer_decode_workspace_bytes(c) == 0
    x = torch.zeros((65, cfg.H), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_layer_decode(c, x, x, None, None, x, (), x, False, x, x, x, x, x, x, x, x, x, None, x, x, 1 << 20)
    assert ei.value.code == -3
    assert mm.moe_layer_decode_workspace_bytes(mm.make_config(cfg_small(dtype="fp32"))) == 0
