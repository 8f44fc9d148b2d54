"""Alg. 1 driven over many decoding steps on the GPU (toy MoE language model, continuous
batching), checked against the oracle: every layer of every step from the layer's own input
(element by element), the output head, the confidence, and the loop's decisions and bookkeeping
against the oracle's single-sequence loop of Alg. 1."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import workloads as wl
from gpu_util import TOL_OUT, out_to_f64, rel_err

pytestmark = pytest.mark.gpu


def layers_of(lm):
    c = lm.cfg
    return [dict(Wg=l.Wg, gate_bias=l.gate_bias, expert_w=l.expert_w, I=c.I, shared_w=l.shared_w,
                 shared_I=c.shared_I) for l in lm.layers]


def host_bits(t: torch.Tensor) -> np.ndarray:
    """Stored form of a device activation: float32, or bf16 bit patterns as uint16."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def toy(dtype, V=48, L=3, seed=3, head_std=0.25, norm=False, **kw):
    base = dict(name="toy", T=1, H=64, E=8, I=48, k_big=4, k_little=2, shared_I=(32,), dtype=dtype,
                renorm=False, gate_std=0.3, w_std=0.18, gate_bias_std=0.2)
    base.update(kw)
    return wl.make_toy_lm(wl.LayerConfig(**base), V=V, L=L, seed=seed, head_std=head_std, norm=norm)


def handed_over(lm, out_bits, x_in, where):
    """The next layer's stored input against the layer's stored output: the same bits, or with the
    model's normalisation the oracle's rescaled rows up to the last stored bit."""
    if not lm.norm:
        assert np.array_equal(x_in, out_bits), where
        return
    want = wl.as_f32(oracle.rms_normalize(out_bits)).astype(np.float64)
    got = wl.as_f32(x_in).astype(np.float64)
    ulp = 2.0 ** -7 if lm.cfg.dtype == "bf16" else 2.0 ** -22
    assert (np.abs(got - want) <= ulp * np.abs(want) + 1e-30).all(), where
    assert (got == want).mean() > 0.98, where


@pytest.mark.parametrize("dtype,renorm,norm,L", [("bf16", False, False, 3), ("bf16", True, False, 3),
                                                 ("fp32", False, False, 3), ("bf16", False, True, 6)])
def test_alg1_over_many_steps(dtype, renorm, norm, L):
    from paper_2510_12357_amd.alg1_driver import Alg1Batch, ToyLMDevice
    lm = toy(dtype, renorm=renorm, norm=norm, L=L, head_std=0.25 if not norm else 0.55)
    c, ls = lm.cfg, layers_of(lm)
    B, steps, max_new = 12, 40, 9
    prompts = wl.make_prompt_tokens(11, 200, lm.V)
    rec = []
    run = Alg1Batch(ToyLMDevice.upload(lm), B, prompts, max_new, eos=0, record=rec)
    for _ in range(steps):
        run.step()
    torch.cuda.synchronize()
    st = run.stats()
    assert st["steps"] == steps and len(rec) == steps

    gamma32 = np.float32(c.gamma)
    tol = TOL_OUT if dtype == "bf16" else 1e-4
    agree_rows = total_rows = 0
    little_p, big_p, little_h, big_h = {}, {}, {}, {}
    for s, r in enumerate(rec):
        tok, big = r["tokens_in"], r["big_in"]
        # ---- the mixed batch: big-mode slots, and only they, are important in every layer
        x_prev = None
        same_sel = np.ones(B, bool)
        for l, (ly, g) in enumerate(zip(ls, r["layers"])):
            x_in = host_bits(g["x_in"])
            if l == 0:
                assert np.array_equal(x_in, lm.embed[tok]), s      # the embedding rows, bit for bit
            else:
                handed_over(lm, x_prev, x_in, (s, l))
            assert np.array_equal(g["important"].astype(bool), big), (s, l)
            assert np.array_equal(g["k_t"], np.where(big, c.k_big, c.k_little)), (s, l)
            # the layer from its own input; selection on the logits the GPU's router produced
            ref = oracle.moe_layer(x_in, ly["Wg"], ly["gate_bias"], ly["expert_w"], ly["I"], ly["shared_w"],
                                   ly["shared_I"], r["conf_in"], c.gamma, c.k_big, c.k_little, c.renorm,
                                   logits=g["logits"])
            assert np.array_equal(g["topk_idx"], ref["topk_idx"]), (s, l)
            e = rel_err(out_to_f64(g["out"]), ref["out"])
            assert e <= tol, (s, l, e)
            own = oracle.gate_logits(x_in, ly["Wg"], ly["gate_bias"])
            assert rel_err(g["logits"], own) <= tol, (s, l)
            same_sel &= (oracle.route(own, r["conf_in"], c.gamma, c.k_big, c.k_little, c.renorm)[0]
                         == g["topk_idx"]).all(axis=1)
            x_prev = host_bits(g["out"])
        # ---- output head, confidence, most probable token
        z = r["lm_logits"]
        x_head = host_bits(r["x_head"])
        handed_over(lm, x_prev, x_head, (s, "head"))
        assert rel_err(z, oracle.gate_logits(x_head, lm.head, None)) <= tol, s
        np.testing.assert_allclose(r["conf"], oracle.token_confidence(z), rtol=2e-6, atol=0)
        assert np.array_equal(r["top"], np.argmax(z, axis=1)), s
        # ---- the whole step from the tokens alone, where the oracle's own routing agrees
        full = oracle.toy_lm_next(lm.embed, ls, lm.head, tok, big, c.gamma, c.k_big, c.k_little, c.renorm,
                                  norm=lm.norm)
        total_rows += B
        agree_rows += int(same_sel.sum())
        if same_sel.any() and L <= 3:
            # three layers deep, each hand-over rounded to the storage type on both sides: a
            # norm-wise bound (the element-wise bar is applied layer by layer above).  A SwiGLU
            # layer is quadratic in its input and doubles a relative perturbation, so deeper
            # stacks are checked layer by layer only.
            d = z[same_sel].astype(np.float64) - full["lm_logits"][same_sel]
            assert np.linalg.norm(d) <= 3 * tol * np.linalg.norm(full["lm_logits"][same_sel]), s
        # ---- what the replay below needs
        zz = z.astype(np.float64)
        p = np.exp(zz - zz.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        for b in range(B):
            if r["seq_id"][b] < 0:
                continue
            key = (r["seq_id"][b], r["pos"][b])
            pb = p[b].copy()
            pb[int(np.argmax(z[b]))] = float(r["conf"][b])      # the decision is taken on the fp32 confidence
            (big_p if big[b] else little_p)[key] = pb
            (big_h if big[b] else little_h)[key] = r["layers"][0]["logits"][b].copy()
    assert agree_rows > 0.8 * total_rows

    # ---- decisions and bookkeeping: every sequence is what Alg. 1 generates from the recorded
    # distributions, run one sequence at a time
    seqs = list(run.finished) + [(run.seq_id[b], run.tokens[b], run.from_big[b]) for b in range(B)
                                 if run.seq_id[b] >= 0]
    assert len(run.finished) >= 3
    n_tok = n_fall = 0
    for sid, tokens, from_big in seqs:
        def little_model(y):
            return little_p[(sid, len(y))], little_h[(sid, len(y))]

        def big_model(y, h):
            # the router states of the rejected pass are those the big pass computes itself
            assert np.array_equal(h, big_h[(sid, len(y))])
            return big_p[(sid, len(y))]

        n = len(from_big)
        y, fb = oracle.alg1_generate(little_model, big_model, [tokens[0]], float(gamma32), 0, max_new=n)
        assert y == tokens and fb == from_big, sid
        assert tokens[0] == int(prompts[sid])
        if (sid, tokens, from_big) in run.finished:
            assert tokens[-1] == 0 or n == max_new
        n_tok += n
        n_fall += sum(fb)
    # a slot that was rejected in the last step has a fallback that is not yet a token
    pending = int(run.big.sum())
    assert st["accepted_tokens"] == n_tok and st["fallbacks"] == n_fall + pending
    assert 0 < n_fall < n_tok
    assert st["little_passes"] + st["big_passes"] == int(sum(sum(1 for q in r["seq_id"] if q >= 0) for r in rec))
    assert st["big_passes"] == n_fall


def test_gamma_limits_on_the_gpu():
    """gamma = 1: every token falls back (no probability exceeds 1), two passes per token; a gamma
    below every confidence: the little model alone."""
    from paper_2510_12357_amd.alg1_driver import Alg1Batch, ToyLMDevice
    for gamma, expect_all_big in ((1.0, True), (1e-6, False)):
        lm = toy("bf16", L=2, gamma=gamma)
        run = Alg1Batch(ToyLMDevice.upload(lm), 8, wl.make_prompt_tokens(5, 64, lm.V), max_new=6)
        for _ in range(12):
            run.step()
        st = run.stats()
        flags = [f for _, _, fb in run.finished for f in fb]
        assert len(flags) > 0 and all(f == expect_all_big for f in flags)
        if expect_all_big:
            assert st["big_passes"] == st["accepted_tokens"] and st["little_passes"] == st["fallbacks"]
        else:
            assert st["fallbacks"] == 0 and st["big_passes"] == 0


def test_vocabulary_limit():
    from paper_2510_12357_amd.alg1_driver import ToyLMDevice
    lm = toy("bf16", V=300, L=1)
    with pytest.raises(ValueError):
        ToyLMDevice.upload(lm)


# ------------------------------------------------------------------ experts in host memory, prefetch ahead
def pinned_experts(lm):
    from paper_2510_12357_amd import binding as mm
    return [torch.stack([mm.to_device(b, lm.cfg, "cpu") for b in l.expert_w]).pin_memory() for l in lm.layers]


def run_driver(lm, B, steps, max_new, prompts, caches=None, d=0, n_slots=None, in_flight=None, yield_to_demand=False):
    from paper_2510_12357_amd.alg1_driver import Alg1Batch, ToyLMDevice
    rec, log = [], []
    run = Alg1Batch(ToyLMDevice.upload(lm), B, prompts, max_new, record=rec,
                    caches=None if caches is None else caches.handles, prefetch_distance=d, fetch_log=log,
                    n_slots=n_slots, in_flight_limit=in_flight, yield_to_demand=yield_to_demand)
    for _ in range(steps):
        run.step()
    torch.cuda.synchronize()
    run.close()
    return run, rec, log


def test_offloaded_model_equals_resident_model_and_cache_follows_the_policy():
    """Sec. II-B / III-B over several layers: the experts of every layer live in pinned host memory
    behind a small cache; the experts of a rejected slot's big pass are prefetched d layers ahead
    from the router states of the rejected pass.  Nothing of that may change a single bit of the
    results, every fetch must follow the cache policy (host-only model), the predictions must be
    the layer's own selection rule on the rejected pass's logits, and prefetching must turn
    demand misses into hits."""
    from oracle.cache_model import DEMAND, PREFETCH, CacheModel
    from paper_2510_12357_amd import binding as mm
    from paper_2510_12357_amd.alg1_driver import LayerCaches
    lm = toy("bf16", L=4, E=32, head_std=0.3)
    c = lm.cfg
    B, steps, max_new, n_slots = 4, 40, 8, 16
    prompts = wl.make_prompt_tokens(21, 200, lm.V)
    base, rec0, _ = run_driver(lm, B, steps, max_new, prompts)
    assert base.stats()["fallbacks"] >= 5
    host = pinned_experts(lm)
    misses = {}
    # (distance, bound on prefetch copies in flight, yield to demand copies): in the last two cases
    # what a request may start depends on how far earlier copies have come; the bound each request
    # ran under is logged and replayed
    for d, in_flight, yields in ((0, None, False), (1, None, False), (2, None, False), (7, None, False),
                                 (2, 3, False), (1, None, True)):
        caches = LayerCaches(host, n_slots)
        try:
            run, rec, log = run_driver(lm, B, steps, max_new, prompts, caches, d, n_slots, in_flight, yields)
            st = run.stats()
            # ---- bit-identical to the model with all experts resident
            assert run.finished == base.finished and run.tokens == base.tokens
            for r, r0 in zip(rec, rec0):
                assert np.array_equal(r["conf"], r0["conf"]) and np.array_equal(r["top"], r0["top"])
                for g, g0 in zip(r["layers"], r0["layers"]):
                    assert np.array_equal(g["topk_idx"], g0["topk_idx"])
                    assert torch.equal(g["out"], g0["out"])
            # ---- the predictions: k_big experts of the rejected pass's router logits, most likely rank first
            by_call = {(s, l): (ids, limit, snap, cnt) for s, l, ids, limit, snap, cnt in log}
            assert (len(log) > 0) == (d > 0)
            for (s, l), (ids, limit, _, _) in by_call.items():
                if yields:
                    assert limit in (-1, 0)
                else:
                    assert (limit < 0) == (in_flight is None) and limit <= (in_flight if in_flight is not None else 0)
                rej = [b for b in range(B) if rec[s]["big_in"][b] and not rec[s - 1]["big_in"][b]]
                assert rej == [b for b in range(B) if rec[s]["big_in"][b]]
                idx = oracle.route(rec[s - 1]["layers"][l]["logits"][rej], None, c.gamma, c.k_big, c.k_little,
                                   c.renorm)[0]
                want = []
                for j in range(c.k_big):
                    for e in idx[:, j]:
                        if int(e) not in want:
                            want.append(int(e))
                assert ids == want, (s, l)
            if d > 0:
                # every layer of every step that has a slot in big mode gets its prefetch, once
                expect = {(s, l) for s in range(1, steps) if rec[s]["big_in"].any() for l in range(len(lm.layers))}
                assert set(by_call) == expect
            # ---- every fetch against the host-only model of the policy
            hits = miss = 0
            for l in range(len(lm.layers)):
                model = CacheModel(c.E, n_slots)
                for s in range(steps):
                    if (s, l) in by_call:
                        ids, limit, snap, cnt = by_call[(s, l)]
                        _, h, m, dr = model.fetch(ids, PREFETCH, None if limit < 0 else limit)
                        assert snap == model.slot_expert and cnt == (h, m, dr), (d, s, l)
                    g = rec[s]["layers"][l]
                    need = sorted({int(e) for e in g["topk_idx"].ravel() if e >= 0})
                    order = [e for e in need if model.slot_of(e) >= 0] + \
                            [e for e in need if model.slot_of(e) < 0]
                    for i in range(0, len(order), n_slots):
                        _, h, m, _ = model.fetch(order[i:i + n_slots], DEMAND)
                        hits, miss = hits + h, miss + m
                assert mm.moe_cache_snapshot(caches.handles[l], n_slots) == model.slot_expert, (d, l)
            assert (st["demand_hits"], st["demand_misses"]) == (hits, miss)
            if in_flight is None and not yields:
                misses[d] = miss
                assert (st["prefetch_copies"] > 0) == (d > 0)
        finally:
            caches.close()
    assert misses[1] < misses[0] and misses[2] < misses[0] and misses[7] < misses[0]


def test_driver_argument_checks():
    from paper_2510_12357_amd.alg1_driver import Alg1Batch, ToyLMDevice
    lm = toy("bf16", L=2)
    dev = ToyLMDevice.upload(lm)
    with pytest.raises(ValueError):
        Alg1Batch(dev, 4, wl.make_prompt_tokens(1, 8, lm.V), 4, caches=[1])
    with pytest.raises(ValueError):
        Alg1Batch(dev, 4, wl.make_prompt_tokens(1, 8, lm.V), 4, prefetch_distance=-1)
