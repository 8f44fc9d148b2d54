"""Seeded synthetic MoE layers (inputs only -- none of the method's arithmetic lives here).

Both the CPU oracle's tests and the GPU tests / benchmark take their host buffers from this
module, so the two sides always see bit-identical inputs.  Everything is numpy on the host;
bf16 tensors are carried as ``uint16`` bit patterns.

The shapes follow the layer configurations this build is measured on (fine-grained MoE
layers like the two models of the paper's evaluation section, plus a coarse 8-expert layer
and a tiny fp32 layer); the value distributions are N(0,1) activations, N(0,0.02) expert
weights and a per-token confidence whose fraction below the threshold gamma equals a chosen
fallback ratio r (the paper's tables report r between 0.10 and 0.29 at gamma = 0.7).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                      # tokens in the step
    H: int                      # hidden size
    E: int                      # routed experts
    I: int                      # routed expert intermediate size
    k_big: int                  # experts of an important token (the model's default K)
    k_little: int               # experts of every other token (K/2)
    shared_I: Tuple[int, ...] = ()   # always-on shared experts (intermediate sizes)
    dtype: str = "bf16"         # storage type of x and all weights: "bf16" | "fp32" | "bf16w8" (bf16
                                # activations and router, expert weights in 8 bits with row scales) |
                                # "bf16mx4" (bf16 activations and router, expert weights in MXFP4)
    renorm: bool = False        # renormalise routing weights over the selected experts
    gamma: float = 0.7          # fallback threshold
    gate_std: float = 0.02
    gate_bias_std: float = 0.0  # > 0: per-expert logit bias (imbalanced expert loads)
    w_std: float = 0.02
    fallback_ratio: float = 0.2

    def with_(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)

    @property
    def expert_params(self) -> int:
        return 3 * self.H * self.I


# The five measured configurations (tokens T is the default; decode sweeps override it).
CONFIGS = {
    "tiny_fp32": LayerConfig("tiny_fp32", T=64, H=256, E=8, I=512, k_big=2, k_little=1,
                             dtype="fp32", renorm=True, gate_std=0.1),
    "fine60_decode": LayerConfig("fine60_decode", T=64, H=2048, E=60, I=1408, k_big=4,
                                 k_little=2, shared_I=(5632,)),
    "fine64_prefill": LayerConfig("fine64_prefill", T=2048, H=2048, E=64, I=1024, k_big=8,
                                  k_little=4, gate_bias_std=1.0),
    "shared2_offload": LayerConfig("shared2_offload", T=16, H=2048, E=64, I=1408, k_big=6,
                                   k_little=3, shared_I=(1408, 1408)),
    "coarse8": LayerConfig("coarse8", T=4096, H=4096, E=8, I=14336, k_big=2, k_little=1,
                           renorm=True),
}


# ----------------------------------------------------------------------------- storage types
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Activations, router weights, embeddings: "bf16w8" and "bf16mx4" store them as bf16."""
    if dtype == "fp32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype in ("bf16", "bf16w8", "bf16mx4"):
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def f32_to_e4m3_bits(a: np.ndarray) -> np.ndarray:
    """An 8-bit E4M3 ("e4m3fn") code for every entry, by the library cast of torch (this module
    holds no arithmetic of the format itself; it only makes up 8-bit expert weights, for which
    any rounding would do).  Entries are clipped to the format's largest magnitude first."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).clamp_(-448.0, 448.0)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def w8_blob_bytes(H: int, I: int) -> int:
    return 3 * H * I + 4 * (2 * I + H)


def quantize_blob_w8(w: np.ndarray, H: int, I: int) -> np.ndarray:
    """[W_gate I*H | W_up I*H | W_down H*I] in fp32 -> the 8-bit blob: E4M3 codes in the same order,
    then the fp32 row scales [gate I | up I | down H]; a row's scale maps its largest magnitude to 448."""
    w = np.asarray(w, np.float32)
    rows = [w[:I * H].reshape(I, H), w[I * H:2 * I * H].reshape(I, H), w[2 * I * H:].reshape(H, I)]
    codes, scales = [], []
    for m in rows:
        s = (np.abs(m).max(axis=1) / np.float32(448.0)).astype(np.float32)
        s[s == 0] = np.float32(1.0)
        codes.append(f32_to_e4m3_bits(m / s[:, None]).ravel())
        scales.append(s)
    return np.concatenate(codes + [np.concatenate(scales).view(np.uint8)])


def mx4_blob_bytes(H: int, I: int) -> int:
    return 3 * H * I // 2 + 3 * H * I // 32


_E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float64)   # magnitudes of codes 0..7


def quantize_rows_mx4(m: np.ndarray):
    """[rows, K] fp32 (K a multiple of 32) -> (codes uint8 [rows, K/2], scales uint8 [rows, K/32]) in
    the OCP microscaling layout MXFP4: per block of 32 along K one power-of-two scale (E8M0 byte =
    exponent + 127, chosen so that the block's largest magnitude lands in the top binade of the
    4-bit element) and 32 E2M1 codes, nearest value, ties to the even code, saturating; two codes
    per byte, even k in the low four bits.  Only makes up 4-bit expert weights for the benchmarks
    and tests; any rounding would do."""
    m = np.asarray(m, np.float64)
    rows, K = m.shape
    assert K % 32 == 0
    blk = m.reshape(rows, K // 32, 32)
    amax = np.abs(blk).max(axis=2)
    exp = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 2.0, 0.0)
    exp = np.clip(exp, -127, 127)
    v = np.abs(blk) / np.exp2(exp)[:, :, None]
    d = np.abs(v[..., None] - _E2M1_GRID)                      # distance to the 8 magnitudes
    best = d.argmin(axis=3)                                    # first minimum = lower code
    tie_up = (best < 7) & (np.take_along_axis(d, np.minimum(best + 1, 7)[..., None], 3)[..., 0]
                           == np.take_along_axis(d, best[..., None], 3)[..., 0]) & (best % 2 == 1)
    code = (best + tie_up).astype(np.uint8) | ((blk < 0).astype(np.uint8) << 3)
    code = code.reshape(rows, K)
    packed = (code[:, 0::2] | (code[:, 1::2] << 4)).astype(np.uint8)
    return packed, (exp + 127).astype(np.uint8)


def quantize_blob_mx4(w: np.ndarray, H: int, I: int) -> np.ndarray:
    """[W_gate I*H | W_up I*H | W_down H*I] in fp32 -> the MXFP4 blob: the packed codes of the three
    matrices in the same order, then their scales [gate I*H/32 | up I*H/32 | down H*I/32]."""
    w = np.asarray(w, np.float32)
    mats = [w[:I * H].reshape(I, H), w[I * H:2 * I * H].reshape(I, H), w[2 * I * H:].reshape(H, I)]
    q = [quantize_rows_mx4(m) for m in mats]
    return np.concatenate([c.ravel() for c, _ in q] + [s.ravel() for _, s in q])


def as_f32(a: np.ndarray) -> np.ndarray:
    """Exact fp32 view of a stored tensor (uint16 bf16 bits or float32)."""
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else np.asarray(a, dtype=np.float32)


# ----------------------------------------------------------------------------- generators
def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    # one independent counter-based stream per (seed, tensor)
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(tensor_id)]))


_ID_X, _ID_WG, _ID_BIAS, _ID_CONF, _ID_LM, _ID_HS = 1, 2, 3, 4, 5, 6
_ID_EXPERT0, _ID_SHARED0 = 1000, 100000


def _normal(seed: int, tid: int, shape, std: float) -> np.ndarray:
    return (_rng(seed, tid).standard_normal(shape, dtype=np.float32) * np.float32(std))


@dataclasses.dataclass
class Layer:
    cfg: LayerConfig
    x: np.ndarray                       # [T,H]
    Wg: np.ndarray                      # [E,H]
    gate_bias: Optional[np.ndarray]     # [E] fp32 or None
    expert_w: List[np.ndarray]          # E flat blobs [W_gate I*H | W_up I*H | W_down H*I]
    shared_w: List[np.ndarray]          # one flat blob per shared expert
    conf: np.ndarray                    # [T] fp32 per-token confidence


def make_confidence(seed: int, T: int, gamma: float, r: float) -> np.ndarray:
    """conf with P(conf <= gamma) = r: u ~ U(0,1]; u <= r maps below gamma, else above."""
    u = 1.0 - _rng(seed, _ID_CONF).random(T)           # (0,1]
    if r <= 0.0:
        c = gamma + (1.0 - gamma) * u
    elif r >= 1.0:
        c = gamma * u
    else:
        c = np.where(u <= r, gamma * u / r, gamma + (1.0 - gamma) * (u - r) / (1.0 - r))
    return c.astype(np.float32)


def make_lm_logits(seed: int, T: int, V: int, r: float, std: float = 3.0,
                   spike: float = 16.0) -> np.ndarray:
    """Synthetic LM-head outputs [T,V]: N(0,std) noise; a fraction 1-r of the rows gets one
    dominant entry so that their largest softmax probability is close to 1."""
    g = _rng(seed, _ID_LM)
    z = g.standard_normal((T, V), dtype=np.float32) * np.float32(std)
    confident = g.random(T) >= r
    hot = g.integers(0, V, size=T)
    z[np.arange(T)[confident], hot[confident]] += np.float32(spike)
    return z


def make_router_noise(seed: int, T: int, E: int, sigma: float) -> np.ndarray:
    """Additive noise that turns a layer's logits into stale "router states" of an earlier
    pass (used to drive prefetch with imperfect predictions)."""
    return _normal(seed, _ID_HS, (T, E), sigma)


def make_expert_blob(cfg: LayerConfig, seed: int, e: int, I: Optional[int] = None,
                     shared: bool = False) -> np.ndarray:
    I = cfg.I if I is None else I
    tid = (_ID_SHARED0 if shared else _ID_EXPERT0) + e
    w = _normal(seed, tid, (3 * cfg.H * I,), cfg.w_std)
    if cfg.dtype == "bf16w8":
        return quantize_blob_w8(w, cfg.H, I)
    if cfg.dtype == "bf16mx4":
        return quantize_blob_mx4(w, cfg.H, I)
    return _store(w, cfg.dtype)


def make_layer(cfg: LayerConfig, seed: int = 0, experts: bool = True) -> Layer:
    x = _store(_normal(seed, _ID_X, (cfg.T, cfg.H), 1.0), cfg.dtype)
    Wg = _store(_normal(seed, _ID_WG, (cfg.E, cfg.H), cfg.gate_std), cfg.dtype)
    bias = _normal(seed, _ID_BIAS, (cfg.E,), cfg.gate_bias_std) if cfg.gate_bias_std > 0 else None
    ew = [make_expert_blob(cfg, seed, e) for e in range(cfg.E)] if experts else []
    sw = [make_expert_blob(cfg, seed, s, I=Is, shared=True) for s, Is in enumerate(cfg.shared_I)] \
        if experts else []
    conf = make_confidence(seed, cfg.T, cfg.gamma, cfg.fallback_ratio)
    return Layer(cfg, x, Wg, bias, ew, sw, conf)


# ----------------------------------------------------------------------------- toy language model
_ID_EMBED, _ID_HEAD, _ID_PROMPT = 7, 8, 9


@dataclasses.dataclass
class ToyLM:
    """Random weights of a tiny attention-free "language model": token embedding, L MoE layers
    applied one after the other (the output of a layer is the input of the next), and an output
    head.  It only exists to drive Alg. 1 (little pass, confidence test, fallback pass) over many
    decoding steps; the next token depends on the current one alone."""
    cfg: LayerConfig                    # shape of every layer (cfg.T is not used)
    V: int                              # vocabulary; token 0 is <eos>
    embed: np.ndarray                   # [V,H] stored dtype
    layers: List[Layer]                 # x / conf of these are not used
    head: np.ndarray                    # [V,H] stored dtype
    norm: bool = False                  # rescale every layer's output rows to unit RMS (deep stacks)


def make_toy_lm(cfg: LayerConfig, V: int, L: int, seed: int = 0, head_std: float = 1.0,
                norm: bool = False) -> ToyLM:
    embed = _store(_normal(seed, _ID_EMBED, (V, cfg.H), 1.0), cfg.dtype)
    head = _store(_normal(seed, _ID_HEAD, (V, cfg.H), head_std), cfg.dtype)
    small = cfg.with_(T=1)
    layers = [make_layer(small, seed=seed * 1009 + 17 * (l + 1)) for l in range(L)]
    return ToyLM(cfg, V, embed, layers, head, norm)


def make_prompt_tokens(seed: int, n: int, V: int) -> np.ndarray:
    """First tokens of n sequences, never <eos>."""
    return _rng(seed, _ID_PROMPT).integers(1, V, size=n).astype(np.int64)
