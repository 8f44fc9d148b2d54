"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes one part of ``oracle/`` to a definition written independently here with
numpy / torch library routines (dense matmuls, stable sorts, torch.topk), to a closed form,
or to a structural invariant the paper states:

* Sec. III-A: a little token uses exactly K/2 experts, an important one K; the little
  selection is a prefix of the big one on the same router scores.
* Alg. 1: the little result is kept iff max(p) > gamma (so equality falls back).
* Table 4, first row: gamma = 0 gives fallback ratio 0.
* Table 3, "vanilla" rows: with every token important the layer is plain top-K MoE.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import workloads as wl


# ------------------------------------------------------------------ independent definitions
def np_softmax(l):
    l = l.astype(np.float64)
    z = l - l.max(axis=1, keepdims=True)
    p = np.exp(z)
    return p / p.sum(axis=1, keepdims=True)


def np_topk_order(l):
    """experts of each row ordered by (logit desc, index asc) -- stable sort of -logit"""
    return np.argsort(-l.astype(np.float64), axis=1, kind="stable")


def np_swiglu(xf, blob, H, I):
    """dense SwiGLU MLP with library matmuls in fp64"""
    W = wl.as_f32(blob).astype(np.float64)
    Wg, Wu, Wd = W[:I * H].reshape(I, H), W[I * H:2 * I * H].reshape(I, H), W[2 * I * H:].reshape(H, I)
    g = xf @ Wg.T
    u = xf @ Wu.T
    return ((g / (1.0 + np.exp(-g))) * u) @ Wd.T


def brute_force_layer(layer, conf, gamma, k_big, k_little, renorm):
    """Every expert on every token, masked by the routing weights, summed."""
    cfg = layer.cfg
    xf = wl.as_f32(layer.x).astype(np.float64)
    logits = (xf @ wl.as_f32(layer.Wg).astype(np.float64).T)
    if layer.gate_bias is not None:
        logits = logits + layer.gate_bias.astype(np.float64)
    logits = logits.astype(np.float32)
    p = np_softmax(logits)
    order = np_topk_order(logits)
    T, E = logits.shape
    important = np.ones(T, bool) if conf is None else ~(conf > np.float32(gamma))
    M = np.zeros((T, E))
    for t in range(T):
        k = k_big if important[t] else k_little
        sel = order[t, :k]
        w = p[t, sel]
        if renorm:
            w = w / w.sum()
        M[t, sel] = w.astype(np.float32)          # routing weights are stored as fp32
    dense = np.stack([np_swiglu(xf, b, cfg.H, cfg.I) for b in layer.expert_w], axis=1)  # [T,E,H]
    out = np.einsum("te,teh->th", M, dense)
    for b, Is in zip(layer.shared_w, cfg.shared_I):
        out = out + np_swiglu(xf, b, cfg.H, Is)
    return out, logits, important


def small_cfg(**kw):
    base = dict(name="small", T=37, H=48, E=10, I=40, k_big=4, k_little=2, shared_I=(24,),
                dtype="fp32", renorm=False, gate_std=0.3, w_std=0.2)
    base.update(kw)
    return wl.LayerConfig(**base)


def run_oracle(layer, conf="cfg", **over):
    cfg = layer.cfg
    c = layer.conf if isinstance(conf, str) else conf
    args = dict(gamma=cfg.gamma, k_big=cfg.k_big, k_little=cfg.k_little, renorm=cfg.renorm)
    args.update(over)
    return oracle.moe_layer(layer.x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I,
                            layer.shared_w, cfg.shared_I, c, **args)


def relerr(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


# ------------------------------------------------------------------ whole layer
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("renorm", [False, True])
@pytest.mark.parametrize("r", [0.0, 0.3, 1.0])
def test_layer_equals_bruteforce_dense(dtype, renorm, r):
    cfg = small_cfg(dtype=dtype, renorm=renorm, fallback_ratio=r, gate_bias_std=0.5)
    layer = wl.make_layer(cfg, seed=3)
    res = run_oracle(layer)
    ref, logits, important = brute_force_layer(layer, layer.conf, cfg.gamma, cfg.k_big,
                                               cfg.k_little, renorm)
    assert np.array_equal(res["logits"], logits) or relerr(res["logits"], logits) < 1e-6
    assert np.array_equal(res["important"].astype(bool), important)
    assert relerr(res["out"], ref) < 1e-9


def test_tiny_config_equals_bruteforce_dense():
    cfg = wl.CONFIGS["tiny_fp32"]
    layer = wl.make_layer(cfg, seed=0)
    res = run_oracle(layer)
    ref, _, _ = brute_force_layer(layer, layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm)
    assert relerr(res["out"], ref) < 1e-9


def test_all_important_is_textbook_topk_moe():
    """conf=None, or gamma >= every conf: standard top-K MoE written with torch.topk."""
    cfg = small_cfg(renorm=True, shared_I=())
    layer = wl.make_layer(cfg, seed=5)
    xf = torch.from_numpy(wl.as_f32(layer.x)).double()
    logits = oracle.gate_logits(layer.x, layer.Wg)
    probs = torch.softmax(torch.from_numpy(logits).double(), dim=-1)
    topw, topi = torch.topk(probs, cfg.k_big, dim=-1)
    topw = (topw / topw.sum(-1, keepdim=True)).float().double()
    out = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for e in range(cfg.E):
        W = torch.from_numpy(wl.as_f32(layer.expert_w[e])).double()
        H, I = cfg.H, cfg.I
        Wg_, Wu_, Wd_ = W[:I * H].view(I, H), W[I * H:2 * I * H].view(I, H), W[2 * I * H:].view(H, I)
        tok, slot = torch.where(topi == e)
        if tok.numel() == 0:
            continue
        hcur = xf[tok]
        y = (torch.nn.functional.silu(hcur @ Wg_.T) * (hcur @ Wu_.T)) @ Wd_.T
        out.index_add_(0, tok, y * topw[tok, slot, None])
    for conf, gamma in ((None, 0.7), (layer.conf, 1.0), (np.full(cfg.T, 0.7, np.float32), 0.7)):
        res = run_oracle(layer, conf=conf, gamma=gamma)
        assert res["important"].all() and (res["k_t"] == cfg.k_big).all()
        assert np.array_equal(res["topk_idx"], topi.numpy().astype(np.int32))
        assert relerr(res["out"], out.numpy()) < 1e-9


def test_gamma_zero_is_all_little():
    cfg = small_cfg()
    layer = wl.make_layer(cfg, seed=7)
    res = run_oracle(layer, gamma=0.0)
    assert not res["important"].any()
    assert ((res["topk_idx"] >= 0).sum(axis=1) == cfg.k_little).all()
    assert res["expert_offsets"][-1] == cfg.T * cfg.k_little
    # equals a plain top-(K/2) MoE: the same layer configured with k_big = k_little
    ref = run_oracle(layer, conf=None, k_big=cfg.k_little, k_little=cfg.k_little)
    assert relerr(res["out"], ref["out"]) < 1e-12


def test_counts_and_prefix_property():
    cfg = small_cfg(fallback_ratio=0.4)
    layer = wl.make_layer(cfg, seed=11)
    mixed = run_oracle(layer)
    big = run_oracle(layer, conf=None)
    little = run_oracle(layer, gamma=0.0)
    n_imp = int(mixed["important"].sum())
    assert 0 < n_imp < cfg.T
    P = cfg.k_big * n_imp + cfg.k_little * (cfg.T - n_imp)
    assert mixed["expert_offsets"][-1] == P
    assert ((mixed["topk_idx"] >= 0).sum(1) == mixed["k_t"]).all()
    assert (mixed["k_t"] == np.where(mixed["important"] == 1, cfg.k_big, cfg.k_little)).all()
    kl = cfg.k_little
    assert np.array_equal(little["topk_idx"][:, :kl], big["topk_idx"][:, :kl])
    assert np.array_equal(little["topk_w"][:, :kl], big["topk_w"][:, :kl])     # renorm off
    assert (little["topk_idx"][:, kl:] == -1).all() and (little["topk_w"][:, kl:] == 0).all()
    # out_big - out_little = sum over the extra ranks of w_j * y_j
    yb = big["y"]
    extra = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        for j in range(kl, cfg.k_big):
            extra[t] += np.float64(big["topk_w"][t, j]) * yb[big["inv_pos"][t, j]]
    assert relerr(big["out"] - little["out"], extra) < 1e-9
    # mixed rows equal the big rows where important, little rows elsewhere
    imp = mixed["important"].astype(bool)
    assert relerr(mixed["out"][imp], big["out"][imp]) < 1e-12
    assert relerr(mixed["out"][~imp], little["out"][~imp]) < 1e-12


# ------------------------------------------------------------------ importance test
def test_threshold_truth_table():
    logits = np.zeros((6, 4), np.float32)
    conf = np.array([0.0, 0.69999, 0.7, 0.70001, 1.0, np.nan], np.float32)
    _, _, imp, kt = oracle.route(logits, conf, 0.7, 2, 1, False)
    # kept little only when strictly above the threshold; equality and NaN fall back
    assert imp.tolist() == [1, 1, 1, 0, 0, 1]
    assert kt.tolist() == [2, 2, 2, 1, 1, 2]
    _, _, imp0, _ = oracle.route(logits, np.array([1e-30, 0.5, 1.0] * 2, np.float32), 0.0, 2, 1, False)
    assert not imp0.any()


# ------------------------------------------------------------------ softmax / top-k
def test_route_against_numpy_sort_and_softmax():
    g = np.random.default_rng(0)
    logits = g.standard_normal((50, 17)).astype(np.float32)
    logits[3, 5] = logits[3, 9] = logits[3].max() + 1      # tie at the top -> lower index first
    logits[4, :] = 0.25                                     # all equal
    for renorm in (False, True):
        idx, w, _, _ = oracle.route(logits, None, 0.7, 6, 3, renorm)
        order = np_topk_order(logits)[:, :6]
        assert np.array_equal(idx, order.astype(np.int32))
        p = np_softmax(logits)
        ref = np.take_along_axis(p, order, axis=1)
        if renorm:
            ref = ref / ref.sum(1, keepdims=True)
        assert np.abs(w - ref.astype(np.float32)).max() <= 1e-7
    assert idx[3, 0] == 5 and idx[3, 1] == 9
    assert idx[4].tolist() == [0, 1, 2, 3, 4, 5]


def test_route_special_cases():
    # E = 1
    idx, w, _, _ = oracle.route(np.array([[3.0], [-2.0]], np.float32), None, 0.7, 1, 1, False)
    assert idx.ravel().tolist() == [0, 0] and np.allclose(w, 1.0)
    # all-equal logits: w = 1/E without renorm, 1/k with
    eq = np.full((2, 8), -1.5, np.float32)
    _, w0, _, _ = oracle.route(eq, None, 0.7, 4, 2, False)
    _, w1, _, _ = oracle.route(eq, None, 0.7, 4, 2, True)
    assert np.allclose(w0, 1 / 8) and np.allclose(w1, 1 / 4)
    # permuting experts permutes indices; adding a per-row constant changes nothing
    g = np.random.default_rng(1)
    lg = g.standard_normal((20, 12)).astype(np.float32)
    perm = g.permutation(12)
    i0, w0, _, _ = oracle.route(lg, None, 0.7, 4, 2, True)
    i1, w1, _, _ = oracle.route(lg[:, perm], None, 0.7, 4, 2, True)
    assert np.array_equal(perm[i1], i0) and np.array_equal(w0, w1)
    shift = (lg.astype(np.float64) + 8.0).astype(np.float32)     # exact-ish shift keeps order
    i2, w2, _, _ = oracle.route(shift, None, 0.7, 4, 2, True)
    assert np.array_equal(i2, i0) and np.abs(w2 - w0).max() < 1e-5
    # renorm on: weights of a row sum to one; off: they equal the full softmax
    assert np.allclose(w0.sum(1), 1.0, atol=1e-6)
    # NaN / -inf scores rank last and get zero weight
    bad = np.array([[0.0, np.nan, 2.0, -np.inf, 1.0]], np.float32)
    ib, wb, _, _ = oracle.route(bad, None, 0.7, 5, 2, False)
    assert ib[0].tolist() == [2, 4, 0, 1, 3] and wb[0, 3] == 0 and wb[0, 4] == 0


def test_argument_checks():
    lg = np.zeros((2, 4), np.float32)
    for kb, kl in ((5, 2), (2, 3), (2, 0)):
        with pytest.raises(ValueError):
            oracle.route(lg, None, 0.7, kb, kl, False)


# ------------------------------------------------------------------ confidence
def test_token_confidence_closed_forms():
    V = 1000
    uniform = np.full((1, V), 4.2, np.float32)
    assert abs(oracle.token_confidence(uniform)[0] - 1.0 / V) < 1e-9
    onehot = np.zeros((1, V), np.float32)
    onehot[0, 17] = 60.0
    assert oracle.token_confidence(onehot)[0] == pytest.approx(1.0, abs=1e-7)
    a, b = 1.25, -0.5                         # two classes: logistic function of the gap
    two = np.array([[a, b]], np.float32)
    assert oracle.token_confidence(two)[0] == pytest.approx(1 / (1 + np.exp(-(a - b))), rel=1e-6)
    z = wl.make_lm_logits(0, 64, 1024, r=0.25)
    ref = torch.softmax(torch.from_numpy(z).double(), -1).max(-1).values.numpy()
    assert np.abs(oracle.token_confidence(z) - ref).max() < 1e-7


# ------------------------------------------------------------------ dispatch
def test_dispatch_equals_stable_sort():
    g = np.random.default_rng(2)
    T, E, K = 41, 9, 4
    kt = g.choice([2, 4], size=T).astype(np.int32)
    idx = np.full((T, K), -1, np.int32)
    for t in range(T):
        idx[t, :kt[t]] = g.permutation(E)[:kt[t]]
    off, st, sr, inv = oracle.dispatch(idx, kt, E)
    pairs = [(t, j) for t in range(T) for j in range(kt[t])]
    keys = np.array([idx[t, j] for t, j in pairs])
    order = np.argsort(keys, kind="stable")
    P = len(pairs)
    assert off[-1] == P == kt.sum()
    assert st[:P].tolist() == [pairs[i][0] for i in order]
    assert sr[:P].tolist() == [pairs[i][1] for i in order]
    assert (st[P:] == -1).all() and (sr[P:] == -1).all()
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(keys, minlength=E))]))
    # inverse map is a bijection onto [0,P) and consistent
    flat = inv[inv >= 0]
    assert sorted(flat.tolist()) == list(range(P))
    for t, j in pairs:
        p = inv[t, j]
        assert st[p] == t and sr[p] == j and off[idx[t, j]] <= p < off[idx[t, j] + 1]
    for e in range(E):                        # tokens strictly increasing inside a segment
        seg = st[off[e]:off[e + 1]]
        assert (np.diff(seg) > 0).all()
    # empty input
    off0, st0, _, _ = oracle.dispatch(np.zeros((0, K), np.int32), np.zeros((0,), np.int32), E)
    assert (off0 == 0).all() and st0.size == 0


# ------------------------------------------------------------------ expert FFN / combine
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_single_expert_is_dense_mlp(dtype):
    cfg = small_cfg(E=1, k_big=1, k_little=1, shared_I=(), renorm=True, dtype=dtype)
    layer = wl.make_layer(cfg, seed=13)
    res = run_oracle(layer)
    ref = np_swiglu(wl.as_f32(layer.x).astype(np.float64), layer.expert_w[0], cfg.H, cfg.I)
    assert relerr(res["out"], ref) < 1e-12
    # rows given in any order / with repeats
    tok = np.array([5, 0, 5, 36], np.int32)
    y = oracle.swiglu_rows(layer.x, layer.expert_w[0], cfg.I, tok)
    assert relerr(y, ref[tok]) < 1e-12


def test_ffn_zero_cases_and_storage_equivalence():
    cfg = small_cfg(shared_I=())
    layer = wl.make_layer(cfg, seed=17)
    H, I = cfg.H, cfg.I
    blob = layer.expert_w[0].copy()
    blob[I * H:2 * I * H] = 0                   # W_up = 0  ->  y = 0
    assert np.abs(oracle.swiglu_rows(layer.x, blob, I)).max() == 0
    assert np.abs(oracle.swiglu_rows(np.zeros_like(layer.x), layer.expert_w[0], I)).max() == 0
    # the same values stored as bf16 bits or widened to fp32 give identical results
    cfgb = cfg.with_(dtype="bf16")
    lb = wl.make_layer(cfgb, seed=17)
    y16 = oracle.swiglu_rows(lb.x, lb.expert_w[1], I)
    y32 = oracle.swiglu_rows(wl.as_f32(lb.x), wl.as_f32(lb.expert_w[1]), I)
    assert np.array_equal(y16, y32)
    l16 = oracle.gate_logits(lb.x, lb.Wg)
    l32 = oracle.gate_logits(wl.as_f32(lb.x), wl.as_f32(lb.Wg))
    assert np.array_equal(l16, l32)


def test_combine_special_cases():
    cfg = small_cfg(k_big=1, k_little=1, renorm=True, shared_I=())
    layer = wl.make_layer(cfg, seed=19)
    res = run_oracle(layer)
    xf = wl.as_f32(layer.x).astype(np.float64)
    for t in range(cfg.T):                       # k=1 with renorm: out = FFN_idx(x)
        e = res["topk_idx"][t, 0]
        ref = np_swiglu(xf[t:t + 1], layer.expert_w[e], cfg.H, cfg.I)[0]
        assert relerr(res["out"][t], ref) < 1e-12
    # linearity in w, and shared terms are added with weight one
    g = np.random.default_rng(3)
    T, H, K = 5, 7, 3
    y = g.standard_normal((T * K, H))
    inv = g.permutation(T * K).reshape(T, K).astype(np.int32)
    kt = np.array([3, 1, 2, 3, 1], np.int32)
    w = g.random((T, K)).astype(np.float32)
    sh = g.standard_normal((2, T, H))
    out = oracle.combine(y, w, inv, kt, sh, T, H)
    ref = np.zeros((T, H))
    for t in range(T):
        for j in range(kt[t]):
            ref[t] += np.float64(w[t, j]) * y[inv[t, j]]
    ref += sh[0] + sh[1]
    assert relerr(out, ref) < 1e-14
    out2 = oracle.combine(y, 2 * w, inv, kt, None, T, H)
    assert relerr(out2, 2 * (ref - sh[0] - sh[1])) < 1e-14


def test_shared_only_when_routed_weights_vanish():
    cfg = small_cfg(shared_I=(24, 16))
    layer = wl.make_layer(cfg, seed=23)
    for b in layer.expert_w:
        b[2 * cfg.I * cfg.H:] = 0               # W_down = 0 for every routed expert
    res = run_oracle(layer)
    xf = wl.as_f32(layer.x).astype(np.float64)
    ref = sum(np_swiglu(xf, b, cfg.H, Is) for b, Is in zip(layer.shared_w, cfg.shared_I))
    assert relerr(res["out"], ref) < 1e-12


# ------------------------------------------------------------------ workload generator
def test_confidence_generator_hits_fallback_ratio():
    for r in (0.0, 0.11, 0.21, 1.0):
        c = wl.make_confidence(0, 20000, 0.7, r)
        frac = float((~(c > np.float32(0.7))).mean())
        assert abs(frac - r) < 0.01
        assert (c > 0).all() and (c <= 1).all()
    bits = wl.f32_to_bf16_bits(np.array([1.0, 1.00390625, 1.01171875, -2.5], np.float32))
    ref = torch.tensor([1.0, 1.00390625, 1.01171875, -2.5]).bfloat16().view(torch.int16).numpy()
    assert np.array_equal(bits, ref.view(np.uint16))


# ------------------------------------------------------------------ second pass of Alg. 1 at layer level
def test_dispatch_from_equals_stable_sort_of_the_window():
    g = np.random.default_rng(7)
    T, E, K = 53, 11, 6
    kt = g.choice([2, 3, 6], size=T).astype(np.int32)
    idx = np.full((T, K), -1, np.int32)
    for t in range(T):
        idx[t, :kt[t]] = g.permutation(E)[:kt[t]]
    # j_lo = 0 is the plain dispatch
    for a, b in zip(oracle.dispatch_from(idx, kt, 0, E), oracle.dispatch(idx, kt, E)):
        assert np.array_equal(a, b)
    for j_lo in (1, 2, 3, 6, 9):
        off, st, sr, inv = oracle.dispatch_from(idx, kt, j_lo, E)
        pairs = [(t, j) for t in range(T) for j in range(j_lo, kt[t])]
        P = len(pairs)
        assert off[-1] == P == np.maximum(kt - j_lo, 0).sum()
        if P:
            keys = np.array([idx[t, j] for t, j in pairs])
            order = np.argsort(keys, kind="stable")
            assert st[:P].tolist() == [pairs[i][0] for i in order]
            assert sr[:P].tolist() == [pairs[i][1] for i in order]
            assert np.array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(keys, minlength=E))]))
        assert (st[P:] == -1).all() and (sr[P:] == -1).all()
        want = np.full((T, K), -1)
        for p in range(P):
            want[st[p], sr[p]] = p
        assert np.array_equal(inv, want)               # -1 for every rank outside the window


def test_combine_add_is_the_window_of_combine():
    g = np.random.default_rng(8)
    T, H, K, E = 9, 12, 4, 5
    kt = g.choice([2, 4], size=T).astype(np.int32)
    idx = np.full((T, K), -1, np.int32)
    for t in range(T):
        idx[t, :kt[t]] = g.permutation(E)[:kt[t]]
    w = g.random((T, K)).astype(np.float32)
    off, st, sr, inv = oracle.dispatch(idx, kt, E)
    y = g.standard_normal((int(off[-1]), H))
    full = oracle.combine(y, w, inv, kt, None, T, H)
    low = oracle.combine(y, w, inv, np.minimum(kt, 2).astype(np.int32), None, T, H)
    base = g.standard_normal((T, H))
    got = oracle.combine_add(y, w, inv, kt, 2, base)
    assert np.allclose(got, base + (full - low), rtol=1e-12, atol=1e-12)
    # written out by hand for one token
    t = int(np.argmax(kt))
    hand = base[t] + sum(float(w[t, j]) * y[inv[t, j]] for j in range(2, kt[t]))
    assert np.allclose(got[t], hand, rtol=1e-12, atol=1e-14)
    # tokens whose window is empty are untouched, bit for bit
    assert np.array_equal(got[kt <= 2], base[kt <= 2])
    assert np.array_equal(oracle.combine_add(y, w, inv, kt, K, base), base)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("r", [0.0, 0.3, 1.0])
def test_little_pass_plus_fallback_increment_is_the_mixed_layer(dtype, r):
    # Alg. 1: little model on every token, big model again for the rejected ones.  Without
    # renormalisation the two-pass result must be the layer evaluated once with k_t per token,
    # which in turn is pinned to the brute-force dense evaluation above.
    cfg = wl.LayerConfig(name="two_pass", T=23, H=40, E=7, I=24, k_big=4, k_little=2, shared_I=(16,),
                         dtype=dtype, renorm=False, gate_std=0.5, w_std=0.2, fallback_ratio=r)
    layer = wl.make_layer(cfg, seed=11)
    args = (layer.x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I, layer.shared_w, cfg.shared_I)
    mixed = oracle.moe_layer(*args, layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, False)
    never = np.full(cfg.T, np.inf, np.float32)                       # confidence above gamma: nobody falls back
    little = oracle.moe_layer(*args, never, cfg.gamma, cfg.k_big, cfg.k_little, False)
    assert (little["k_t"] == cfg.k_little).all()
    second = oracle.fallback_increment(layer.x, layer.expert_w, cfg.I, little["logits"], layer.conf,
                                       cfg.gamma, cfg.k_big, cfg.k_little, little["out"])
    assert np.array_equal(second["k_t"], mixed["k_t"])
    assert int(second["expert_offsets"][-1]) == int((mixed["k_t"] - cfg.k_little).sum())
    scale = np.abs(mixed["out"]).max()
    assert np.abs(second["out"] - mixed["out"]).max() <= 1e-12 * scale
    # tokens that keep their little result are not touched at all
    keep = mixed["important"] == 0
    assert np.array_equal(second["out"][keep], little["out"][keep])
    # and against the independent dense evaluation
    dense, _, _ = brute_force_layer(layer, layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, False)
    assert np.abs(second["out"] - dense).max() <= 1e-9 * scale


# ------------------------------------------------------------------ Eq. 1 against the numbers the paper prints
def _golden(name):
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_eq1_against_the_papers_threshold_sweep():
    # Table IV gives (r, speedup) pairs of one model.  Eq. 1 fixes their relation: at r = 0 the
    # speedup is T / T_l; every further row then implies a big-model latency T_b / T, which must be
    # positive and below 1 (Sec. III-B: the big pass hides its expert loads behind prefetching, so it
    # is faster than full offloading), and the speedup must fall as r grows.
    rows = [(float(g), float(r), float(s)) for g, r, s in _golden("table4_threshold_sweep.txt")]
    assert rows[0][1] == 0.0
    Tl_over_T = 1.0 / rows[0][2]
    assert abs(oracle.eq1_speedup(1.0, Tl_over_T, 0.7, 0.0) - rows[0][2]) < 1e-12      # r = 0: T_b is irrelevant
    prev = rows[0][2]
    for g, r, s in rows[1:]:
        Tb_over_T = (1.0 / s - Tl_over_T) / r                                            # Eq. 1 solved for T_b / T
        assert 0.0 < Tb_over_T < 1.0, (g, Tb_over_T)
        assert abs(oracle.eq1_speedup(1.0, Tl_over_T, Tb_over_T, r) - s) < 1e-9
        assert s < prev
        prev = s
    # the formula itself, written out once by hand: T = 10, T_l = 5, T_b = 4, r = 0.25 -> 10 / 6
    assert abs(oracle.eq1_speedup(10.0, 5.0, 4.0, 0.25) - 10.0 / 6.0) < 1e-15


def test_eq1_against_the_papers_main_results_and_bench_helper():
    import bench
    for model, task, kl, kb, r, s_little, s_mobile in _golden("table3_main_results.txt"):
        r, s_little, s_mobile = float(r), float(s_little), float(s_mobile)
        assert int(kl) * 2 == int(kb)                                                    # Sec. III-A: the little model uses K/2 experts
        Tl_over_T = 1.0 / s_little
        Tb_over_T = (1.0 / s_mobile - Tl_over_T) / r
        assert 0.0 < Tb_over_T < 1.0, (model, task, Tb_over_T)
        for f in (oracle.eq1_speedup, bench.eq1):                                        # the benchmark's own helper agrees
            assert abs(f(1.0, Tl_over_T, Tb_over_T, r) - s_mobile) < 1e-9
            assert abs(f(1.0, Tl_over_T, Tb_over_T, 0.0) - s_little) < 1e-9
