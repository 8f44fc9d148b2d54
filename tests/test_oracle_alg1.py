"""Pins of the oracle's Alg. 1 loop and of its toy language model step (CPU only).

The loop is checked against traces worked out by hand from scripted models, against its limits
(gamma below every probability: the little model alone; gamma = 1: the big model alone) and
against a chain written out separately; the toy model step against a dense numpy computation
that shares nothing with the oracle."""
import numpy as np
import pytest

import oracle
from paper_2510_12357_amd import workloads as wl

from test_oracle_pins import np_softmax, np_topk_order, np_swiglu


def onehotish(V, tok, pmax):
    """A distribution whose largest entry pmax sits at tok."""
    p = np.full(V, (1.0 - pmax) / (V - 1))
    p[tok] = pmax
    return p


# ------------------------------------------------------------------ scripted models, traces by hand
def test_loop_follows_a_hand_worked_trace():
    V, eos, gamma = 5, 0, 0.7
    # little model: token and confidence as a function of how many tokens there are so far
    little = {1: (3, 0.9), 2: (4, 0.7), 3: (2, 0.71), 4: (1, 0.2), 5: (0, 0.99)}
    big = {2: 1, 4: 3}                      # the big model's token where it is asked
    asked = []

    def little_model(y):
        tok, c = little[len(y)]
        return onehotish(V, tok, c), ("h", len(y))

    def big_model(y, h):
        assert h == ("h", len(y))           # the router states of the rejected pass are handed over
        asked.append(len(y))
        return onehotish(V, big[len(y)], 0.5)

    y, from_big = oracle.alg1_generate(little_model, big_model, [2], gamma, eos, max_new=10)
    # step 1: 0.9 > 0.7 keep 3; step 2: 0.7 is not above 0.7 -> big gives 1; step 3: 0.71 keep 2;
    # step 4: 0.2 -> big gives 3; step 5: 0.99 keep <eos> and stop
    assert y == [2, 3, 1, 2, 3, 0]
    assert from_big == [False, True, False, True, False]
    assert asked == [2, 4]


def test_loop_stops_at_eos_and_at_the_length_cap():
    V = 4
    calls = []

    def little_model(y):
        calls.append(len(y))
        return onehotish(V, 2, 0.95), None

    def no_big(y, h):
        raise AssertionError("big model must not run")

    y, fb = oracle.alg1_generate(little_model, no_big, [1, 3], 0.7, 0, max_new=4)
    assert y == [1, 3, 2, 2, 2, 2] and fb == [False] * 4 and calls == [2, 3, 4, 5]
    # a prompt that already ends in <eos> generates nothing
    y, fb = oracle.alg1_generate(little_model, no_big, [1, 0], 0.7, 0, max_new=4)
    assert y == [1, 0] and fb == []
    # the <eos> may come from the big model as well
    y, fb = oracle.alg1_generate(lambda y: (onehotish(V, 2, 0.3), None), lambda y, h: onehotish(V, 0, 0.4),
                                 [1], 0.7, 0, max_new=4)
    assert y == [1, 0] and fb == [True]


def test_ties_take_the_lowest_token():
    p = np.array([0.1, 0.4, 0.4, 0.1])
    y, fb = oracle.alg1_generate(lambda y: (p, None), lambda y, h: p, [3], 0.3, 0, max_new=1)
    assert y == [3, 1] and fb == [False]
    y, fb = oracle.alg1_generate(lambda y: (p, None), lambda y, h: p[::-1].copy(), [3], 0.5, 0, max_new=1)
    assert y == [3, 1] and fb == [True]


# ------------------------------------------------------------------ the toy model, densely in numpy
def toy(dtype="fp32", L=2, V=24, seed=3, head_std=0.25, norm=False, **kw):
    base = dict(name="toy", T=1, H=40, E=6, I=24, k_big=4, k_little=2, shared_I=(16,), dtype=dtype,
                renorm=False, gate_std=0.3, w_std=0.2, gate_bias_std=0.2)
    base.update(kw)
    return wl.make_toy_lm(wl.LayerConfig(**base), V=V, L=L, seed=seed, head_std=head_std, norm=norm)


def layers_of(lm):
    c = lm.cfg
    return [dict(Wg=l.Wg, gate_bias=l.gate_bias, expert_w=l.expert_w, I=c.I, shared_w=l.shared_w,
                 shared_I=c.shared_I) for l in lm.layers]


def store_like(a, lm):
    f = np.asarray(a, np.float64).astype(np.float32)
    return f if lm.cfg.dtype == "fp32" else wl.f32_to_bf16_bits(f)


def dense_next(lm, tokens, big):
    """Embedding row -> every expert on every token, masked by the routing weights -> head ->
    softmax; a layer's output is stored in the model's dtype before the next layer reads it."""
    c = lm.cfg
    x = lm.embed[np.asarray(tokens)]
    for l in lm.layers:
        xf = wl.as_f32(x).astype(np.float64)
        logits = (xf @ wl.as_f32(l.Wg).astype(np.float64).T + l.gate_bias.astype(np.float64)).astype(np.float32)
        p, order = np_softmax(logits), np_topk_order(logits)
        out = np.zeros_like(xf)
        for t in range(len(tokens)):
            sel = order[t, :(c.k_big if big[t] else c.k_little)]
            w = p[t, sel]
            if c.renorm:
                w = w / w.sum()
            for e, we in zip(sel, w.astype(np.float32)):
                out[t] += float(we) * np_swiglu(xf[t:t + 1], l.expert_w[e], c.H, c.I)[0]
        for b, Is in zip(l.shared_w, c.shared_I):
            out += np_swiglu(xf, b, c.H, Is)
        x = store_like(out, lm)
        if lm.norm:
            f = wl.as_f32(x).astype(np.float64)
            x = store_like(f / np.sqrt(np.mean(f ** 2, axis=1, keepdims=True) + 1e-6), lm)
    z = (wl.as_f32(x).astype(np.float64) @ wl.as_f32(lm.head).astype(np.float64).T).astype(np.float32)
    return np_softmax(z), z


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("renorm,norm,L", [(False, False, 2), (True, False, 2), (False, True, 5)])
def test_toy_step_equals_dense_numpy(dtype, renorm, norm, L):
    lm = toy(dtype=dtype, renorm=renorm, norm=norm, L=L, head_std=0.25 if not norm else 0.5)
    c = lm.cfg
    rng = np.random.default_rng(5)
    tokens = rng.integers(0, lm.V, size=19)
    big = rng.random(19) < 0.4
    r = oracle.toy_lm_next(lm.embed, layers_of(lm), lm.head, tokens, big, c.gamma, c.k_big, c.k_little, c.renorm,
                           norm=lm.norm)
    p, z = dense_next(lm, tokens, big)
    if norm:
        x = wl.as_f32(r["x_last"]).astype(np.float64)
        np.testing.assert_allclose(np.sqrt((x ** 2).mean(axis=1)), 1.0, rtol=1e-2)
    # bf16 storage between the layers can flip the last stored bit where the two summation orders
    # differ; that moves a logit by a few 1e-3 relative
    tol = 1e-9 if dtype == "fp32" else 2e-2
    np.testing.assert_allclose(r["lm_logits"], z, rtol=0, atol=tol * np.abs(z).max() + 1e-6)
    np.testing.assert_allclose(r["p"], p, rtol=0, atol=1e-6 if dtype == "fp32" else 5e-2)
    np.testing.assert_allclose(r["conf"], r["p"].max(axis=1), rtol=1e-6)
    assert len(r["router_logits"]) == len(lm.layers) and r["router_logits"][0].shape == (19, c.E)
    # the mode matters: flipping one token's mode changes that token's row and no other
    big2 = big.copy()
    big2[3] = not big2[3]
    r2 = oracle.toy_lm_next(lm.embed, layers_of(lm), lm.head, tokens, big2, c.gamma, c.k_big, c.k_little, c.renorm,
                            norm=lm.norm)
    changed = np.abs(r2["lm_logits"] - r["lm_logits"]).max(axis=1) > 0
    assert changed[3] and changed.sum() == 1


def test_loop_on_the_toy_model_against_a_chain_written_out():
    lm = toy(dtype="fp32", V=24, head_std=0.25)
    c = lm.cfg
    ls = layers_of(lm)
    asked = []

    def little_model(y):
        r = oracle.toy_lm_next(lm.embed, ls, lm.head, [y[-1]], [False], c.gamma, c.k_big, c.k_little, c.renorm)
        return r["p"][0], r["router_logits"]

    def big_model(y, h):
        asked.append(len(y))
        r = oracle.toy_lm_next(lm.embed, ls, lm.head, [y[-1]], [True], c.gamma, c.k_big, c.k_little, c.renorm)
        # the big model's own router sees, in the first layer, the logits the little pass handed over
        np.testing.assert_array_equal(h[0], r["router_logits"][0])
        return r["p"][0]

    # the same chain, step by step, from the dense model
    def chain(start, gamma, n):
        y, fb = [start], []
        while y[-1] != 0 and len(fb) < n:
            p, _ = dense_next(lm, [y[-1]], [False])
            use_big = not (p[0].max() > gamma)
            if use_big:
                p, _ = dense_next(lm, [y[-1]], [True])
            y.append(int(np.argmax(p[0])))
            fb.append(use_big)
        return y, fb

    total = falls = 0
    for start in (1, 5, 11, 17, 23):
        for gamma in (0.0, 0.5, 0.7, 0.9, 1.0):
            y, fb = oracle.alg1_generate(little_model, big_model, [start], gamma, 0, max_new=12)
            y2, fb2 = chain(start, gamma, 12)
            assert y == y2 and fb == fb2, (start, gamma)
            if gamma == 0.0:
                assert not any(fb)          # every probability maximum exceeds 0
            if gamma == 1.0:
                assert all(fb)              # no probability exceeds 1
            if gamma == 0.7:
                total, falls = total + len(fb), falls + sum(fb)
    assert 0 < falls < total                # the test exercises both branches at the paper's gamma
