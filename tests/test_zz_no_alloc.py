"""moe_expert_ffn_static (the execution stage on the library's built-in scratch buffer, for callers
that cannot allocate) against moe_expert_ffn with a caller workspace: same kernels, so the results
must be identical bit for bit; two calls in a row on the shared buffer, the second one smaller."""
import numpy as np
import pytest
import torch

from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl
from gpu_util import DeviceLayer

pytestmark = pytest.mark.gpu


def run_both(cfg, seed):
    layer = wl.make_layer(cfg, seed=seed)
    dl = DeviceLayer(layer)
    b = mm.StepBuffers(cfg)
    mm.moe_route(b.c, dl.x, dl.Wg, dl.gate_bias, dl.conf, b.logits, False, b.topk_idx, b.topk_w, b.important, b.k_t)
    mm.moe_dispatch(b.c, b.topk_idx, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos, b.dws,
                    b.dws_bytes)
    mm.moe_expert_ffn(b.c, dl.x, b.expert_offsets, b.sorted_token, dl.table, dl.shared, True, True, b.y, b.shared_out,
                      b.fws, b.fws_bytes)
    mm.moe_combine(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, b.shared_out, b.out)
    torch.cuda.synchronize()
    P = int(b.expert_offsets[-1])
    want = (b.y[:P].clone(), None if b.shared_out is None else b.shared_out.clone(), b.out.clone())
    b.y.fill_(float("nan"))
    if b.shared_out is not None:
        b.shared_out.fill_(float("nan"))
    print(f"static ffn: cfg={cfg.name} T={cfg.T} P={P} need={b.fws_bytes}", flush=True)
    mm.moe_expert_ffn_static(b.c, dl.x, b.expert_offsets, b.sorted_token, dl.table, dl.shared, True, True, b.y,
                             b.shared_out)
    mm.moe_combine(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, b.shared_out, b.out)
    torch.cuda.synchronize()
    assert P > 0
    assert torch.equal(b.y[:P], want[0])
    if want[1] is not None:
        assert torch.equal(b.shared_out, want[1])
    assert torch.equal(b.out, want[2])


def test_static_scratch_equals_workspace_two_calls_second_smaller():
    big = wl.LayerConfig("na_big", T=48, H=512, E=16, I=264, k_big=4, k_little=2, shared_I=(520,), gate_std=0.3,
                         w_std=0.1, fallback_ratio=0.3)
    small = big.with_(name="na_small", T=5, I=136, shared_I=(72,))
    assert mm.moe_expert_ffn_workspace_bytes(mm.make_config(big)) <= mm.moe_expert_ffn_static_max_bytes()
    run_both(big, seed=11)
    run_both(small, seed=12)          # reads only what it wrote itself into the shared buffer
    run_both(big.with_(dtype="fp32", T=20), seed=13)


def test_static_scratch_rejects_steps_beyond_its_size():
    cfg = wl.CONFIGS["fine64_prefill"]            # 2048 tokens x 8 experts x 1024: 32 MB of activations
    c = mm.make_config(cfg)
    assert mm.moe_expert_ffn_workspace_bytes(c) > mm.moe_expert_ffn_static_max_bytes() == 8 << 20
    x = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_expert_ffn_static(c, x, x, x, x, (), True, False, x, None)
    assert ei.value.code == -6
