"""Shared plumbing of the GPU parity tests: upload a synthetic layer, run the C-ABI step, and
the error metric.  The expected values always come from ``oracle`` on the same host buffers."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl

TOL_OUT = 2e-2      # max relative error on layer outputs (bf16 storage, fp32 accumulation)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - o_i| / max(|o_i|, RMS(o)): element-wise relative error, floored at the RMS of
    the reference so that entries near zero do not blow the ratio up."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float((np.abs(got - ref) / den).max())


class DeviceLayer:
    """Device copies of a workloads.Layer; experts live in one [E, 3*H*I] tensor."""

    def __init__(self, layer: wl.Layer, device="cuda"):
        cfg = layer.cfg
        self.cfg, self.layer = cfg, layer
        self.x = mm.to_device(layer.x, cfg, device)
        self.Wg = mm.to_device(layer.Wg, cfg, device)
        self.gate_bias = None if layer.gate_bias is None else torch.from_numpy(layer.gate_bias).to(device)
        self.conf = torch.from_numpy(layer.conf).to(device)
        if layer.expert_w:
            self.experts = torch.stack([mm.to_device(b, cfg, "cpu") for b in layer.expert_w]).to(device)
            stride = self.experts.stride(0) * self.experts.element_size()
            base = self.experts.data_ptr()
            self.table = torch.tensor([base + e * stride for e in range(cfg.E)], dtype=torch.int64,
                                      device=device)
        self.shared = [mm.to_device(b, cfg, device) for b in layer.shared_w]


def run_gpu_layer(dl: DeviceLayer, conf="layer", logits: np.ndarray | None = None, T=None):
    """Runs the four C calls; returns the StepBuffers (device tensors)."""
    cfg = dl.cfg
    b = mm.StepBuffers(cfg, T)
    c = dl.conf if isinstance(conf, str) else conf
    given = logits is not None
    if given:
        b.logits.copy_(torch.from_numpy(logits))
    mm.layer_step(b, dl.x, dl.Wg, dl.gate_bias, c, dl.table, dl.shared, logits_given=given)
    torch.cuda.synchronize()
    return b


def run_oracle_layer(layer: wl.Layer, conf="layer", logits=None, tokens=None):
    cfg = layer.cfg
    c = layer.conf if isinstance(conf, str) else conf
    x = layer.x
    if tokens is not None:
        x = x[tokens]
        c = None if c is None else c[tokens]
        logits = None if logits is None else logits[tokens]
    return oracle.moe_layer(x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I, layer.shared_w,
                            cfg.shared_I, c, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm, logits=logits)


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)
