"""Alg. 1 over a batch of sequences (continuous batching) on a toy MoE language model.

The method's arithmetic runs in the library's kernels: the layers are `layer_step` calls; the
output head reuses `moe_route` with the vocabulary in the place of the experts (its logits are
x . head^T and its rank-0 selection is the most probable token, lowest id among equals); the
confidence is `moe_token_confidence`.  torch gathers embedding rows, optionally rescales a layer's
output rows to unit RMS (the toy model's glue between layers: a stack of SwiGLU layers is quadratic
in its input and needs it beyond a few layers) and carries a few small arrays to the host, where the
loop of Alg. 1 takes its decisions.

Scheduling (Sec. III-A, Alg. 1, batched): each slot of the batch holds one sequence that is either
in little mode (its next token is tried with k_little experts per layer) or in big mode (the
little model's token was rejected, the same position is run again with k_big experts).  One step
runs all slots together as one mixed batch: the per-token confidence handed to the layers is
+inf for little-mode slots (not important) and the rejected confidence (<= gamma: important) for
big-mode slots, so that the layer kernels see exactly the mixed k of the paper's method.  A
finished sequence (<eos> or the length cap) is replaced by the next prompt at once.

Offloaded experts (Sec. II-B, III-B): with one expert cache per layer the routed experts live in
pinned host memory and every layer fetches what its router selected.  For a slot in big mode the
router logits of its rejected little pass are known for ALL layers before the big pass starts, so
the experts they name (k_big per layer, the selection rule of the layer itself) are prefetched
`prefetch_distance` layers ahead of the layer that is being computed: before layer l of a step runs,
the prefetch for layer l + d is issued (layers 0 .. d-1 at the start of the step).  Little-mode slots
have no prediction; their experts are demand misses.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as mm
from . import workloads as wl


class ToyLMDevice:
    """A toy language model on the device: embedding [V,H], head [V,H] (both in the layers' dtype)
    and per layer a dict with Wg, gate_bias (or None), table (int64 device pointers of the E expert
    blobs) and shared (list of blobs).  `block_work` (a callable or None) is enqueued once per layer
    in front of the MoE layer: a stand-in for the rest of a transformer block (attention), which
    the toy model does not have, for measurements that need its time."""

    def __init__(self, cfg: wl.LayerConfig, V: int, embed: torch.Tensor, head: torch.Tensor, layers: list,
                 norm: bool = False, block_work=None):
        if V > 256:
            raise ValueError("the output head runs on the router kernel: at most 256 tokens in the vocabulary")
        self.cfg, self.V, self.device = cfg, V, embed.device
        self.embed, self.head, self.layers, self.norm = embed, head, layers, norm
        self.block_work = block_work
        # the head as a "router" over V outputs with one selected entry
        self.head_cfg = wl.LayerConfig("lm_head", T=1, H=cfg.H, E=V, I=16, k_big=1, k_little=1,
                                       dtype="fp32" if cfg.dtype == "fp32" else "bf16", gamma=cfg.gamma)

    @classmethod
    def upload(cls, lm: wl.ToyLM, device="cuda") -> "ToyLMDevice":
        """Device copies of a workloads.ToyLM."""
        cfg = lm.cfg
        if lm.V > 256:
            raise ValueError("the output head runs on the router kernel: at most 256 tokens in the vocabulary")
        layers = []
        for l in lm.layers:
            experts = torch.stack([mm.to_device(b, cfg, "cpu") for b in l.expert_w]).to(device)
            stride = experts.stride(0) * experts.element_size()
            table = torch.tensor([experts.data_ptr() + e * stride for e in range(cfg.E)], dtype=torch.int64,
                                 device=device)
            layers.append(dict(
                Wg=mm.to_device(l.Wg, cfg, device),
                gate_bias=None if l.gate_bias is None else torch.from_numpy(l.gate_bias).to(device),
                experts=experts, table=table,
                shared=[mm.to_device(b, cfg, device) for b in l.shared_w]))
        return cls(cfg, lm.V, mm.to_device(lm.embed, cfg, device), mm.to_device(lm.head, cfg, device), layers,
                   lm.norm)

    def between_layers(self, out: torch.Tensor) -> torch.Tensor:
        """What the next layer (or the head) reads: the layer's stored output, with `norm` its rows
        divided by sqrt(mean of squares + 1e-6) and stored in the same type."""
        if not self.norm:
            return out
        f = out.float()
        return (f * torch.rsqrt((f * f).mean(dim=1, keepdim=True) + 1e-6)).to(out.dtype)


class LayerCaches:
    """One expert cache per layer: `host_experts[l]` is a pinned host tensor [E, blob elements] with
    the layer's expert blobs, each cache gets n_slots HBM slots of one blob."""

    def __init__(self, host_experts: list, n_slots: int, device="cuda"):
        self.handles, self.slots, self.host = [], [], host_experts
        try:
            for h in host_experts:
                E, blob = h.shape
                dev = torch.zeros((n_slots, blob), dtype=h.dtype, device=device)
                self.slots.append(dev)
                self.handles.append(mm.moe_cache_create(E, blob * h.element_size(), n_slots, h, dev))
        except Exception:
            self.close()
            raise

    def close(self) -> None:
        for h in self.handles:
            mm.moe_cache_sync(h)
            mm.moe_cache_destroy(h)
        self.handles = []


class Alg1Batch:
    """B sequences advancing together.  `prompts` holds the first token of every sequence that will
    ever be started (the run ends when they are used up and all slots have drained, or after the
    number of steps the caller runs).  With `record` (a list) every step appends the host copies a
    checker needs.  `always_big` runs the model without the method (every pass a big pass, every
    token kept): the T of Eq. 1."""

    def __init__(self, dev: ToyLMDevice, B: int, prompts: np.ndarray, max_new: int, eos: int = 0,
                 record: Optional[list] = None, always_big: bool = False, caches: Optional[list] = None,
                 prefetch_distance: int = 0, fetch_log: Optional[list] = None, in_flight_limit: Optional[int] = None,
                 n_slots: Optional[int] = None, yield_to_demand: bool = False):
        self.dev, self.B, self.max_new, self.eos, self.record = dev, B, max_new, eos, record
        if caches is not None and len(caches) != len(dev.layers):
            raise ValueError("one expert cache per layer")
        if prefetch_distance < 0:
            raise ValueError("prefetch_distance must not be negative")
        self.caches, self.distance, self.fetch_log = caches, prefetch_distance, fetch_log
        self.always_big = always_big        # the model without the method: one big pass per token
        self.gamma = np.float32(dev.cfg.gamma)
        self.prompts, self.next_prompt = np.asarray(prompts, np.int64), 0
        d = dev.device
        self.bufs = [mm.StepBuffers(dev.cfg, B, d) for _ in dev.layers]
        self.hb = mm.StepBuffers(dev.head_cfg, B, d)
        self.conf_out = torch.empty((B,), dtype=torch.float32, device=d)
        self.tok_dev = torch.empty((B,), dtype=torch.int64, device=d)
        self.conf_dev = torch.empty((B,), dtype=torch.float32, device=d)
        # host state of the slots
        self.seq_id = [-1] * B
        self.tokens: List[List[int]] = [[] for _ in range(B)]
        self.from_big: List[List[bool]] = [[] for _ in range(B)]
        self.big = np.zeros(B, bool)
        self.rejected_conf = np.zeros(B, np.float32)
        self.finished = []                  # (seq_id, tokens, from_big)
        self.n_steps = self.n_accepted = self.n_fallbacks = self.n_little = self.n_big = 0
        # offloading: the prediction made from the router logits of the rejected passes (experts per
        # layer, most likely first), and the counters
        L = len(dev.layers)
        self.predicted: List[List[int]] = [[] for _ in range(L)]
        self.sched = None
        if caches is not None and prefetch_distance > 0:
            self.sched = mm.moe_prefetcher_create(caches, dev.cfg.k_big)
            if in_flight_limit is not None:
                mm.moe_prefetcher_set_in_flight_limit(self.sched, in_flight_limit)
            mm.moe_prefetcher_set_yield_to_demand(self.sched, yield_to_demand)
        if fetch_log is not None and caches is not None and n_slots is None:
            raise ValueError("a fetch log records the caches' residency: pass the caches' n_slots")
        self.n_slots = n_slots
        self.demand_hits = self.demand_misses = self.prefetch_copies = self.prefetch_dropped = 0
        self.bytes_h2d = self.waves = 0
        for b in range(B):
            self._refill(b)

    # ---- slots
    def _refill(self, b: int) -> None:
        if self.next_prompt < len(self.prompts):
            self.seq_id[b] = self.next_prompt
            self.tokens[b] = [int(self.prompts[self.next_prompt])]
            self.next_prompt += 1
        else:
            self.seq_id[b] = -1
            self.tokens[b] = []
        self.from_big[b] = []
        self.big[b] = self.always_big

    def active(self) -> np.ndarray:
        return np.array([s >= 0 for s in self.seq_id])

    # ---- one step of the whole batch
    def step(self) -> None:
        """Enqueues the step on torch's current stream and waits for its confidences and tokens."""
        dev, B = self.dev, self.B
        act = self.active()
        if not act.any():
            return
        # an empty slot runs a padding token in little mode; its results are ignored
        tok = np.array([self.tokens[b][-1] if act[b] else self.eos for b in range(B)], np.int64)
        conf_in = np.where(self.big, self.rejected_conf, np.float32(np.inf)).astype(np.float32)
        self.tok_dev.copy_(torch.from_numpy(tok))
        self.conf_dev.copy_(torch.from_numpy(conf_in))
        x = dev.embed.index_select(0, self.tok_dev)
        xs = [x]
        L = len(dev.layers)
        if self.sched is not None:
            self._prefetch(-1)
        for l, (ly, b) in enumerate(zip(dev.layers, self.bufs)):
            if self.sched is not None:
                self._prefetch(l)           # layer l is about to run: request what layer l + d will need
            if dev.block_work is not None:
                dev.block_work()
            if self.caches is None:
                # resident experts: a batch of at most 64 slots is one launch per layer
                step = mm.layer_decode_step if b.lws is not None else mm.layer_step
                x = step(b, x, ly["Wg"], ly["gate_bias"], self.conf_dev, ly["table"], ly["shared"])
            else:
                x, st, waves = mm.layer_step_cached(b, x, ly["Wg"], ly["gate_bias"], self.conf_dev,
                                                    self.caches[l], ly["shared"])
                self.demand_hits += st.hits
                self.demand_misses += st.misses
                self.bytes_h2d += st.bytes_h2d
                self.waves += waves
            x = dev.between_layers(x)
            xs.append(x)
        hb = self.hb
        mm.moe_route(hb.c, x, dev.head, None, None, hb.logits, False, hb.topk_idx, hb.topk_w, hb.important,
                     hb.k_t, None)
        mm.moe_token_confidence(hb.logits, B, dev.V, self.conf_out, None)
        conf = self.conf_out.cpu().numpy()          # synchronises
        top = hb.topk_idx[:, 0].cpu().numpy()
        if self.record is not None:
            self.record.append(dict(
                seq_id=list(self.seq_id), pos=[len(t) for t in self.tokens], tokens_in=tok.copy(),
                big_in=self.big.copy(), conf_in=conf_in.copy(),
                layers=[dict(x_in=xi.detach().cpu(), logits=b.logits.cpu().numpy(),
                             topk_idx=b.topk_idx.cpu().numpy(), k_t=b.k_t.cpu().numpy(),
                             important=b.important.cpu().numpy(), out=b.out.detach().cpu())
                        for xi, b in zip(xs, self.bufs)],
                x_head=x.detach().cpu(), lm_logits=hb.logits.cpu().numpy(), conf=conf.copy(), top=top.copy()))
        self.n_steps += 1
        rejected: List[int] = []
        for b in range(B):
            if not act[b]:
                continue
            if self.big[b]:
                self.n_big += 1
            else:
                self.n_little += 1
            if not self.big[b] and not (conf[b] > self.gamma):
                # Alg. 1: the little model's token is dropped, the position runs again in big mode
                self.big[b] = True
                self.rejected_conf[b] = conf[b]
                self.n_fallbacks += 1
                rejected.append(b)
                continue
            self.tokens[b].append(int(top[b]))
            self.from_big[b].append(bool(self.big[b]))
            self.big[b] = self.always_big
            self.n_accepted += 1
            if int(top[b]) == self.eos or len(self.from_big[b]) >= self.max_new:
                self.finished.append((self.seq_id[b], self.tokens[b], self.from_big[b]))
                self._refill(b)
        if self.caches is not None:
            self._predict(rejected)

    # ---- prefetch from the router states of the rejected passes (Sec. III-B)
    def _predict(self, rejected: List[int]) -> None:
        """Hands the router logits of the step's passes and the slots that were rejected to the
        library's prefetch scheduler, which keeps one request list per layer (the experts the big
        pass will most likely select, by the layer's own rule, most likely rank first)."""
        if self.sched is None:
            return
        if self.always_big:
            rejected = []                   # a slot is in big mode only right after its rejection
        mm.moe_prefetcher_predict(self.sched, [b.logits for b in self.bufs], self.B, rejected)
        E = self.dev.cfg.E
        self.predicted = [mm.moe_prefetcher_predicted(self.sched, l, E) for l in range(len(self.bufs))]

    def _prefetch(self, layer: int) -> None:
        """Reports a point of the pass (-1: it starts; l: layer l is about to run) to the scheduler."""
        L = len(self.bufs)
        for l, limit, st in mm.moe_prefetcher_advance(self.sched, layer, self.distance, L):
            self.prefetch_copies += st.misses
            self.prefetch_dropped += st.dropped
            self.bytes_h2d += st.bytes_h2d
            if self.fetch_log is not None:
                self.fetch_log.append((self.n_steps, l, list(self.predicted[l]), limit,
                                       mm.moe_cache_snapshot(self.caches[l], self.n_slots),
                                       (st.hits, st.misses, st.dropped)))

    def close(self) -> None:
        if self.sched is not None:
            mm.moe_prefetcher_destroy(self.sched)
            self.sched = None

    def stats(self) -> dict:
        return dict(steps=self.n_steps, accepted_tokens=self.n_accepted, fallbacks=self.n_fallbacks,
                    little_passes=self.n_little, big_passes=self.n_big,
                    fallback_ratio=self.n_fallbacks / max(self.n_accepted, 1),
                    finished_sequences=len(self.finished), demand_hits=self.demand_hits,
                    demand_misses=self.demand_misses, prefetch_copies=self.prefetch_copies,
                    prefetch_dropped=self.prefetch_dropped, bytes_h2d=self.bytes_h2d, waves=self.waves)
