"""GPU-vs-oracle parity through the C ABI (needs an MI355X; run with ``-m gpu``).

Bars: expert indices, importance flags, k_t and every dispatch array are bit-exact given the
same gate logits; routing weights agree to fp32 rounding; layer outputs agree within 2e-2
maximum relative error (bf16 storage with fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl
from gpu_util import (TOL_OUT, DeviceLayer, out_to_f64, rel_err, run_gpu_layer, run_oracle_layer)

pytestmark = pytest.mark.gpu


def cfg_small(**kw):
    base = dict(name="small", T=37, H=264, E=10, I=136, k_big=4, k_little=2, shared_I=(72,),
                dtype="bf16", renorm=False, gate_std=0.3, w_std=0.1, fallback_ratio=0.3)
    base.update(kw)
    return wl.LayerConfig(**base)


def i32(t):
    return t.cpu().numpy().astype(np.int32)


# ------------------------------------------------------------------ selection stage
@pytest.mark.parametrize("T,E,kb,kl", [(1, 8, 2, 1), (64, 60, 4, 2), (300, 64, 8, 4), (33, 200, 6, 3),
                                       (5, 1, 1, 1), (17, 256, 16, 8)])
@pytest.mark.parametrize("renorm", [False, True])
def test_route_bit_exact_on_given_logits(T, E, kb, kl, renorm):
    g = np.random.default_rng(T * 1000 + E)
    logits = g.standard_normal((T, E)).astype(np.float32)
    if E >= 8:
        logits[0, 3] = logits[0, 5] = logits[0].max() + 1          # tie at the top
        logits[T // 2, :] = 0.5                                      # all equal
        logits[T - 1, 1] = np.nan
        logits[T - 1, 2] = -np.inf
    conf = g.random(T).astype(np.float32)
    conf[0] = 0.7                                                    # equality falls back
    cfg = wl.LayerConfig("r", T=T, H=8, E=E, I=8, k_big=kb, k_little=kl, renorm=renorm)
    c = mm.make_config(cfg)
    b = mm.StepBuffers(cfg)
    b.logits.copy_(torch.from_numpy(logits))
    mm.moe_route(c, None, None, None, torch.from_numpy(conf).cuda(), b.logits, True, b.topk_idx,
                 b.topk_w, b.important, b.k_t)
    torch.cuda.synchronize()
    idx, w, imp, kt = oracle.route(logits, conf, cfg.gamma, kb, kl, renorm)
    assert np.array_equal(i32(b.topk_idx), idx)
    assert np.array_equal(b.important.cpu().numpy(), imp)
    assert np.array_equal(i32(b.k_t), kt)
    assert np.abs(b.topk_w.cpu().numpy() - w).max() <= 2e-6
    # conf = NULL: every token important
    mm.moe_route(c, None, None, None, None, b.logits, True, b.topk_idx, b.topk_w, b.important, b.k_t)
    torch.cuda.synchronize()
    idx2, _, _, _ = oracle.route(logits, None, cfg.gamma, kb, kl, renorm)
    assert np.array_equal(i32(b.topk_idx), idx2) and b.important.cpu().numpy().all()


@pytest.mark.parametrize("dtype,T,H,E", [("bf16", 64, 2048, 60), ("bf16", 300, 264, 10), ("fp32", 64, 256, 8),
                                         ("bf16", 1, 2048, 64), ("fp32", 130, 72, 33)])
def test_gate_logits(dtype, T, H, E):
    cfg = wl.LayerConfig("g", T=T, H=H, E=E, I=8, k_big=1, k_little=1, dtype=dtype, gate_std=0.1,
                         gate_bias_std=1.0)
    layer = wl.make_layer(cfg, seed=2, experts=False)
    ref = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = mm.StepBuffers(cfg)
    x, Wg = mm.to_device(layer.x, cfg), mm.to_device(layer.Wg, cfg)
    mm.moe_route(b.c, x, Wg, torch.from_numpy(layer.gate_bias).cuda(), None, b.logits, False, b.topk_idx,
                 b.topk_w, b.important, b.k_t)
    torch.cuda.synchronize()
    got = b.logits.cpu().numpy()
    # fp32 accumulation of exact bf16 products: error ~ sqrt(H) * 2^-24 * |terms|
    assert np.abs(got - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())


def test_token_confidence():
    z = wl.make_lm_logits(0, 64, 1024, r=0.25)
    conf = torch.empty(64, dtype=torch.float32, device="cuda")
    mm.moe_token_confidence(torch.from_numpy(z).cuda(), 64, 1024, conf)
    torch.cuda.synchronize()
    ref = oracle.token_confidence(z)
    assert np.abs(conf.cpu().numpy() - ref).max() <= 1e-6
    z2 = wl.make_lm_logits(1, 3, 50257, r=0.5)                      # ragged vocabulary size
    conf2 = torch.empty(3, dtype=torch.float32, device="cuda")
    mm.moe_token_confidence(torch.from_numpy(z2).cuda(), 3, 50257, conf2)
    torch.cuda.synchronize()
    assert np.abs(conf2.cpu().numpy() - oracle.token_confidence(z2)).max() <= 1e-6


# ------------------------------------------------------------------ dispatch
@pytest.mark.parametrize("T,E,K", [(1, 8, 2), (64, 60, 4), (256, 64, 8), (257, 64, 8), (2048, 64, 8),
                                   (1000, 7, 3), (40, 256, 16), (0, 8, 2)])
def test_dispatch_bit_exact(T, E, K):
    g = np.random.default_rng(T + E + K)
    kl = max(1, K // 2)
    kt = g.choice([kl, K], size=T).astype(np.int32)
    idx = np.full((T, K), -1, np.int32)
    skew = g.random(E) ** 3 + 1e-3                                   # imbalanced expert loads
    skew /= skew.sum()
    for t in range(T):
        idx[t, :kt[t]] = g.choice(E, size=kt[t], replace=False, p=skew)
    cfg = wl.LayerConfig("d", T=T, H=8, E=E, I=8, k_big=K, k_little=kl)
    b = mm.StepBuffers(cfg)
    if T:
        b.topk_idx.copy_(torch.from_numpy(idx))
        b.k_t.copy_(torch.from_numpy(kt))
    for buf in (b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos):
        buf.fill_(-7)
    mm.moe_dispatch(b.c, b.topk_idx, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos,
                    b.dws, b.dws_bytes)
    torch.cuda.synchronize()
    off, st, sr, inv = oracle.dispatch(idx, kt, E)
    assert np.array_equal(i32(b.expert_offsets), off)
    assert np.array_equal(i32(b.sorted_token), st)
    assert np.array_equal(i32(b.sorted_rank), sr)
    assert np.array_equal(i32(b.inv_pos), inv)


# ------------------------------------------------------------------ whole layer, element by element
def check_layer(cfg, seed=0, conf="layer", tol=TOL_OUT):
    layer = wl.make_layer(cfg, seed=seed)
    dl = DeviceLayer(layer)
    # the oracle's fp32 logits are handed to the GPU path so that selection is bit-comparable
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    cdev = dl.conf if isinstance(conf, str) else (None if conf is None else torch.from_numpy(conf).cuda())
    b = run_gpu_layer(dl, conf=cdev, logits=logits)
    ref = run_oracle_layer(layer, conf=conf, logits=logits)
    assert np.array_equal(i32(b.topk_idx), ref["topk_idx"])
    assert np.array_equal(b.important.cpu().numpy(), ref["important"])
    assert np.array_equal(i32(b.k_t), ref["k_t"])
    assert np.array_equal(i32(b.expert_offsets), ref["expert_offsets"])
    assert np.array_equal(i32(b.sorted_token), ref["sorted_token"])
    assert np.array_equal(i32(b.sorted_rank), ref["sorted_rank"])
    assert np.array_equal(i32(b.inv_pos), ref["inv_pos"])
    P = int(ref["expert_offsets"][-1])
    e_y = rel_err(b.y[:P].cpu().numpy(), ref["y"])
    assert e_y <= tol, f"expert outputs: {e_y}"
    if ref["shared"] is not None:
        # the slabs of shared_out are partial sums; together they are the shared experts' output
        e_s = rel_err(b.shared_out.cpu().numpy().sum(axis=0), ref["shared"].sum(axis=0))
        assert e_s <= tol, f"shared experts: {e_s}"
    e_o = rel_err(out_to_f64(b.out), ref["out"])
    assert e_o <= tol, f"layer output: {e_o}"
    # the GPU's own gate GEMM leads to the same layer within tolerance wherever selection agrees
    b2 = run_gpu_layer(dl, conf=cdev)
    same = (i32(b2.topk_idx) == ref["topk_idx"]).all(axis=1)
    assert same.mean() > 0.9
    assert rel_err(out_to_f64(b2.out)[same], ref["out"][same]) <= tol
    return b, ref


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("r", [0.0, 0.3, 1.0])
def test_small_ragged_layer(dtype, r):
    # H, I not multiples of 16/32, E not a multiple of 16, T with a ragged tail
    check_layer(cfg_small(dtype=dtype, fallback_ratio=r, gate_bias_std=0.5), seed=1,
                tol=TOL_OUT if dtype == "bf16" else 1e-4)


def test_tiny_fp32_config():
    check_layer(wl.CONFIGS["tiny_fp32"], seed=0, tol=1e-4)


def test_tiny_config_in_bf16():
    check_layer(wl.CONFIGS["tiny_fp32"].with_(dtype="bf16"), seed=0)


@pytest.mark.parametrize("T", [1, 8, 32, 64])
def test_fine60_decode_full_size(T):
    check_layer(wl.CONFIGS["fine60_decode"].with_(T=T), seed=0)


def test_many_tokens_per_expert_and_renorm():
    # more than 64 tokens per expert (several token blocks per work item list) and renorm on
    check_layer(cfg_small(T=300, E=4, k_big=3, k_little=1, renorm=True, shared_I=(40, 24)), seed=4)


def test_many_token_blocks_in_the_streaming_kernels():
    # fewer than 256 tokens (streaming kernels) but several token blocks per expert, row-tile
    # counts that are not multiples of 8, K with a partial last chunk
    check_layer(cfg_small(T=200, E=4, k_big=3, k_little=1, shared_I=(40, 24)), seed=5)
    check_layer(cfg_small(T=97, E=6, k_big=4, k_little=2, shared_I=(72,)), seed=6)


def test_all_big_and_all_little_and_null_conf():
    cfg = cfg_small()
    b_big, ref_big = check_layer(cfg, conf=None)
    assert (ref_big["k_t"] == cfg.k_big).all()
    hi = np.ones(cfg.T, np.float32)
    b_lit, ref_lit = check_layer(cfg, conf=hi)
    assert (ref_lit["k_t"] == cfg.k_little).all()


def test_zero_tokens_and_bad_arguments():
    cfg = cfg_small(T=0)
    b = mm.StepBuffers(cfg)
    layer = wl.make_layer(cfg.with_(T=1), seed=0)
    dl = DeviceLayer(layer)
    mm.layer_step(b, b.out, dl.Wg, None, None, dl.table, dl.shared)   # nothing to do, no error
    torch.cuda.synchronize()
    bad = mm.make_config(cfg_small(k_big=4, k_little=5))
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_dispatch_workspace_bytes(bad)      # returns 0 ...
        mm.moe_route(bad, None, None, None, None, b.logits, True, b.topk_idx, b.topk_w, b.important, b.k_t)
    assert ei.value.code == -2
    odd = mm.make_config(cfg_small(H=100))
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_combine(odd, b.y, b.topk_w, b.inv_pos, b.k_t, b.shared_out, b.out)
    assert ei.value.code == -3
    ok = mm.StepBuffers(cfg_small())
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_dispatch(ok.c, ok.topk_idx, ok.k_t, ok.expert_offsets, ok.sorted_token, ok.sorted_rank,
                        ok.inv_pos, ok.dws, 0)
    assert ei.value.code == -6
    # a shared expert blob that is not 16-byte aligned is refused before anything is launched
    one = cfg_small(T=4)
    l1 = DeviceLayer(wl.make_layer(one, seed=0))
    b1 = mm.StepBuffers(one)
    raw = torch.zeros(l1.shared[0].numel() + 8, dtype=l1.shared[0].dtype, device="cuda")
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_expert_ffn(b1.c, l1.x, b1.expert_offsets, b1.sorted_token, None, [raw[1:]], False, True, b1.y,
                          b1.shared_out, b1.fws, b1.fws_bytes)
    assert ei.value.code == -1


def test_null_expert_pointer_skips_expert():
    cfg = cfg_small(shared_I=())
    layer = wl.make_layer(cfg, seed=6)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    ref = run_oracle_layer(layer, logits=logits)
    b = mm.StepBuffers(cfg)
    b.logits.copy_(torch.from_numpy(logits))
    mm.moe_route(b.c, dl.x, dl.Wg, None, dl.conf, b.logits, True, b.topk_idx, b.topk_w, b.important, b.k_t)
    mm.moe_dispatch(b.c, b.topk_idx, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos,
                    b.dws, b.dws_bytes)
    # two waves: even experts first, odd experts second; rows of skipped experts stay untouched
    b.y.fill_(123.0)
    even = dl.table.clone(); even[1::2] = 0
    odd = dl.table.clone(); odd[0::2] = 0
    mm.moe_expert_ffn(b.c, dl.x, b.expert_offsets, b.sorted_token, even, [], True, False, b.y, None,
                      b.fws, b.fws_bytes)
    torch.cuda.synchronize()
    off = ref["expert_offsets"]
    y = b.y.cpu().numpy()
    for e in range(cfg.E):
        seg = y[off[e]:off[e + 1]]
        if e % 2 == 1:
            assert (seg == 123.0).all()
        elif seg.size:
            assert rel_err(seg, ref["y"][off[e]:off[e + 1]]) <= TOL_OUT
    mm.moe_expert_ffn(b.c, dl.x, b.expert_offsets, b.sorted_token, odd, [], True, False, b.y, None,
                      b.fws, b.fws_bytes)
    mm.moe_combine(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, None, b.out)
    torch.cuda.synchronize()
    assert rel_err(out_to_f64(b.out), ref["out"]) <= TOL_OUT


def test_deterministic_across_runs():
    cfg = wl.CONFIGS["fine60_decode"].with_(T=8)
    layer = wl.make_layer(cfg, seed=3)
    dl = DeviceLayer(layer)
    a = run_gpu_layer(dl)
    o1, y1 = a.out.clone(), a.y.clone()
    st1 = a.sorted_token.clone()
    b = run_gpu_layer(dl)
    assert torch.equal(o1.view(torch.int16), b.out.view(torch.int16))
    assert torch.equal(y1, b.y) and torch.equal(st1, b.sorted_token)


# ------------------------------------------------------------------ full-size prefill, sampled tokens
def sampled_tokens(off, st, n_random, seed, T):
    """Tokens to check one by one: for every expert the first and the last row of its segment and
    the rows on both sides of each 128-row tile boundary inside it (where the tiled kernels switch
    tiles and stop computing), plus n_random tokens drawn without replacement."""
    pick = set(int(t) for t in np.random.default_rng(seed).choice(T, size=min(n_random, T), replace=False))
    for e in range(len(off) - 1):
        lo, hi = int(off[e]), int(off[e + 1])
        rows = {lo, hi - 1}
        for edge in range(lo + 128, hi, 128):
            rows.update((edge - 1, edge))
        for m in (31, 32, 63, 64):                        # the 32-row blocks of the last tile
            rows.add(lo + (hi - lo - 1) // 128 * 128 + m)
        pick.update(int(st[p]) for p in rows if lo <= p < hi)
    return np.array(sorted(pick), np.int64)


def check_sampled_prefill(cfg, layer, b, logits, n_random, seed):
    """Index outputs in full and bit for bit; y rows and layer outputs on the sampled tokens."""
    idx, w, imp, kt = oracle.route(logits, layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm)
    off, st, sr, inv = oracle.dispatch(idx, kt, cfg.E)
    assert np.array_equal(i32(b.topk_idx), idx) and np.array_equal(i32(b.k_t), kt)
    assert np.array_equal(b.important.cpu().numpy(), imp)
    assert np.array_equal(i32(b.expert_offsets), off) and np.array_equal(i32(b.sorted_token), st)
    assert np.array_equal(i32(b.sorted_rank), sr) and np.array_equal(i32(b.inv_pos), inv)
    tokens = sampled_tokens(off, st, n_random, seed, cfg.T)
    ref = run_oracle_layer(layer, logits=logits, tokens=tokens)
    e = rel_err(out_to_f64(b.out)[tokens], ref["out"])
    assert e <= TOL_OUT, e
    # expert outputs y (Eq. of Sec. II-A before the weighted sum), row by row: the row of token
    # tokens[i] at rank j sits at inv[tokens[i], j] on the device and at the sub-layer's own
    # inv_pos in the oracle's run over the sampled tokens
    y_gpu = b.y.float().cpu().numpy().astype(np.float64)
    got, want = [], []
    for i, t in enumerate(tokens):
        for j in range(int(kt[t])):
            got.append(y_gpu[inv[t, j]])
            want.append(ref["y"][ref["inv_pos"][i, j]])
    e_y = rel_err(np.stack(got), np.stack(want))
    assert e_y <= TOL_OUT, e_y
    return off, tokens


def test_fine64_prefill_full_size_sampled():
    cfg = wl.CONFIGS["fine64_prefill"]
    layer = wl.make_layer(cfg, seed=0)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = run_gpu_layer(dl, logits=logits)
    off, tokens = check_sampled_prefill(cfg, layer, b, logits, n_random=160, seed=0)
    counts = np.diff(off)
    assert counts.max() > 3 * max(1, counts.min())           # the bias skews the loads
    assert len(tokens) >= 256


def test_coarse8_full_size_sampled_prefill_and_single_token():
    """The 8-expert layer with 14336-wide experts at full size: a 4096-token prefill step (tiled MFMA
    kernels) checked on sampled tokens, and a one-token decode step (streaming kernels)."""
    cfg = wl.CONFIGS["coarse8"]
    layer = wl.make_layer(cfg, seed=0)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    b = run_gpu_layer(dl, logits=logits)
    check_sampled_prefill(cfg, layer, b, logits, n_random=8, seed=1)
    # decode: the first token alone, once little (confident) and once big (not confident)
    one = wl.Layer(cfg.with_(T=1), layer.x[:1], layer.Wg, layer.gate_bias, layer.expert_w, layer.shared_w,
                   layer.conf[:1])
    dl1 = DeviceLayer.__new__(DeviceLayer)
    dl1.__dict__.update(dl.__dict__)
    dl1.cfg, dl1.x = one.cfg, dl.x[:1].contiguous()
    for conf in (np.array([0.99], np.float32), np.array([0.1], np.float32)):
        b1 = run_gpu_layer(dl1, conf=torch.from_numpy(conf).cuda(), logits=logits[:1], T=1)
        r1 = oracle.moe_layer(one.x, one.Wg, one.gate_bias, one.expert_w, cfg.I, [], (), conf, cfg.gamma,
                              cfg.k_big, cfg.k_little, cfg.renorm, logits=logits[:1])
        assert np.array_equal(i32(b1.topk_idx), r1["topk_idx"])
        assert rel_err(out_to_f64(b1.out), r1["out"]) <= TOL_OUT


def test_shared_experts_on_a_side_stream():
    """Shared experts enqueued on a second stream (under the router kernels) give the same layer."""
    cfg = wl.CONFIGS["fine60_decode"].with_(T=8)
    layer = wl.make_layer(cfg, seed=5)
    dl = DeviceLayer(layer)
    logits = oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)
    ref = run_oracle_layer(layer, logits=logits)
    side = torch.cuda.Stream()
    b = mm.StepBuffers(cfg)
    for it in range(3):                                  # repeated steps reuse the buffers and events
        b.logits.copy_(torch.from_numpy(logits))
        mm.layer_step(b, dl.x, dl.Wg, dl.gate_bias, dl.conf, dl.table, dl.shared, logits_given=True,
                      side_stream=side)
        torch.cuda.synchronize()
        assert rel_err(out_to_f64(b.out), ref["out"]) <= TOL_OUT
    plain = run_gpu_layer(dl, logits=logits)
    assert torch.equal(plain.out.view(torch.int16), b.out.view(torch.int16))


# ------------------------------------------------------------------ second pass of Alg. 1 at layer level
@pytest.mark.parametrize("T,E,K,j_lo", [(1, 8, 2, 1), (64, 60, 4, 2), (64, 60, 4, 0), (64, 60, 4, 4), (257, 64, 8, 4),
                                        (2048, 64, 8, 4), (1000, 7, 3, 1), (40, 256, 16, 8)])
def test_dispatch_from_bit_exact(T, E, K, j_lo):
    g = np.random.default_rng(T + E + K + j_lo)
    kl = max(1, K // 2)
    kt = g.choice([kl, K], size=T).astype(np.int32)
    idx = np.full((T, K), -1, np.int32)
    for t in range(T):
        idx[t, :kt[t]] = g.choice(E, size=kt[t], replace=False)
    cfg = wl.LayerConfig("d", T=T, H=8, E=E, I=8, k_big=K, k_little=kl)
    b = mm.StepBuffers(cfg)
    b.topk_idx.copy_(torch.from_numpy(idx))
    b.k_t.copy_(torch.from_numpy(kt))
    for buf in (b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos):
        buf.fill_(-7)
    mm.moe_dispatch_from(b.c, b.topk_idx, b.k_t, j_lo, b.expert_offsets, b.sorted_token, b.sorted_rank,
                         b.inv_pos, b.dws, b.dws_bytes)
    torch.cuda.synchronize()
    off, st, sr, inv = oracle.dispatch_from(idx, kt, j_lo, E)
    assert np.array_equal(i32(b.expert_offsets), off)
    assert np.array_equal(i32(b.sorted_token), st)
    assert np.array_equal(i32(b.sorted_rank), sr)
    assert np.array_equal(i32(b.inv_pos), inv)


@pytest.mark.parametrize("cfg", [
    cfg_small(fallback_ratio=0.3, gate_bias_std=0.5),                          # streaming kernels, ragged sizes
    cfg_small(T=300, E=4, k_big=3, k_little=1, shared_I=(40, 24)),             # tiled kernels
    wl.CONFIGS["fine60_decode"].with_(T=64),                                   # the decode layer at full size
    cfg_small(dtype="fp32", fallback_ratio=0.5),
], ids=["small", "tiled", "fine60_b64", "fp32"])
def test_little_pass_then_fallback_pass(cfg):
    tol = TOL_OUT if cfg.dtype == "bf16" else 1e-4
    layer = wl.make_layer(cfg, seed=3)
    dl = DeviceLayer(layer)
    never = torch.full((cfg.T,), float("inf"), dtype=torch.float32, device="cuda")
    b = mm.StepBuffers(cfg)
    # pass 1: the little model on every token
    mm.layer_step(b, dl.x, dl.Wg, dl.gate_bias, never, dl.table, dl.shared)
    torch.cuda.synchronize()
    logits = b.logits.cpu().numpy()                                            # selection is compared on the GPU's logits
    args = (layer.x, layer.Wg, layer.gate_bias, layer.expert_w, cfg.I, layer.shared_w, cfg.shared_I)
    little = oracle.moe_layer(*args, never.cpu().numpy(), cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm,
                              logits=logits)
    assert np.array_equal(i32(b.k_t), little["k_t"]) and (little["k_t"] == cfg.k_little).all()
    assert np.array_equal(i32(b.topk_idx), little["topk_idx"])
    out_little = out_to_f64(b.out)
    assert rel_err(out_little, little["out"]) <= tol
    # pass 2: the rejected tokens get the ranks k_little .. k_big-1 on top
    mm.fallback_step(b, dl.x, dl.conf, dl.table)
    torch.cuda.synchronize()
    ref = oracle.fallback_increment(layer.x, layer.expert_w, cfg.I, logits, layer.conf, cfg.gamma,
                                    cfg.k_big, cfg.k_little, little["out"])
    for name in ("topk_idx", "k_t", "expert_offsets", "sorted_token", "sorted_rank", "inv_pos"):
        assert np.array_equal(i32(getattr(b, name)), ref[name]), name
    assert np.array_equal(b.important.cpu().numpy(), ref["important"])
    P2 = int(ref["expert_offsets"][-1])
    assert P2 == int((ref["k_t"] - cfg.k_little).sum())
    if P2:
        assert rel_err(b.y[:P2].cpu().numpy(), ref["y"]) <= tol
    out2 = out_to_f64(b.out)
    assert rel_err(out2, ref["out"]) <= tol
    keep = ref["important"] == 0
    assert np.array_equal(out2[keep], out_little[keep])                        # kept tokens are not rewritten
    # the two passes give the one-pass layer with k_t per token
    one = mm.StepBuffers(cfg)
    one.logits.copy_(b.logits)
    mm.layer_step(one, dl.x, dl.Wg, dl.gate_bias, dl.conf, dl.table, dl.shared, logits_given=True)
    torch.cuda.synchronize()
    assert rel_err(out2, out_to_f64(one.out)) <= tol


def test_fallback_pass_argument_checks():
    b = mm.StepBuffers(cfg_small(renorm=True))
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_combine_add(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, 2, b.out)
    assert ei.value.code == -3                                                 # renormalised weights: not additive
    ok = mm.StepBuffers(cfg_small())
    for j_lo in (-1, 5):
        with pytest.raises(mm.MoeError) as ei:
            mm.moe_dispatch_from(ok.c, ok.topk_idx, ok.k_t, j_lo, ok.expert_offsets, ok.sorted_token,
                                 ok.sorted_rank, ok.inv_pos, ok.dws, ok.dws_bytes)
        assert ei.value.code == -1
        with pytest.raises(mm.MoeError) as ei:
            mm.moe_combine_add(ok.c, ok.y, ok.topk_w, ok.inv_pos, ok.k_t, j_lo, ok.out)
        assert ei.value.code == -1


# ------------------------------------------------------------------ kernel switch points and table limits
@pytest.mark.parametrize("T", [255, 256])
def test_layer_on_both_sides_of_the_streaming_tiled_switch(T):
    # 255 tokens run the streaming kernels (8 token blocks per expert), 256 the tiled ones
    check_layer(cfg_small(T=T, E=5, k_big=3, k_little=1, shared_I=(40,)), seed=7)


def test_many_experts_and_largest_top_k():
    # group tables near their limits: 200 routed experts + 4 shared experts, top-16 of them
    check_layer(cfg_small(T=33, E=200, k_big=16, k_little=8, shared_I=(24, 40, 8, 16), I=72), seed=8)
    check_layer(cfg_small(T=3, E=256, k_big=16, k_little=8, shared_I=(), I=40), seed=9)


@pytest.mark.parametrize("dtype,T,E,kb", [("bf16", 40, 60, 4), ("fp32", 40, 60, 4), ("bf16", 64, 256, 16),
                                          ("bf16", 1, 7, 3)])
def test_one_launch_router_equals_the_two_kernels(dtype, T, E, kb):
    """Steps of at most 64 tokens compute router logits and selection in one launch; larger steps use
    the separate logits kernel and the selection kernel.  Same rows in: bit-identical logits and
    selections out, and the selections are the oracle's on those logits."""
    cfg = cfg_small(T=T, E=E, k_big=kb, k_little=max(1, kb // 2), dtype=dtype, gate_bias_std=0.5,
                    fallback_ratio=0.4)
    layer = wl.make_layer(cfg, seed=12, experts=False)
    x, Wg = mm.to_device(layer.x, cfg), mm.to_device(layer.Wg, cfg)
    bias, conf = torch.from_numpy(layer.gate_bias).cuda(), torch.from_numpy(layer.conf).cuda()
    b1 = mm.StepBuffers(cfg)
    mm.moe_route(b1.c, x, Wg, bias, conf, b1.logits, False, b1.topk_idx, b1.topk_w, b1.important, b1.k_t)
    big = cfg.with_(T=100)
    rows = torch.arange(100, device="cuda") % cfg.T
    b2 = mm.StepBuffers(big)
    mm.moe_route(b2.c, x[rows].contiguous(), Wg, bias, conf[rows].contiguous(), b2.logits, False, b2.topk_idx,
                 b2.topk_w, b2.important, b2.k_t)
    torch.cuda.synchronize()
    assert torch.equal(b1.logits, b2.logits[:cfg.T])
    assert torch.equal(b1.topk_idx, b2.topk_idx[:cfg.T]) and torch.equal(b1.topk_w, b2.topk_w[:cfg.T])
    assert torch.equal(b1.k_t, b2.k_t[:cfg.T]) and torch.equal(b1.important, b2.important[:cfg.T])
    idx, w, imp, kt = oracle.route(b1.logits.cpu().numpy(), layer.conf, cfg.gamma, cfg.k_big, cfg.k_little, cfg.renorm)
    assert np.array_equal(i32(b1.topk_idx), idx) and np.array_equal(i32(b1.k_t), kt)
    assert np.array_equal(b1.important.cpu().numpy(), imp)
    np.testing.assert_allclose(b1.topk_w.cpu().numpy(), w, rtol=2e-6, atol=1e-9)
    assert rel_err(b1.logits.cpu().numpy(), oracle.gate_logits(layer.x, layer.Wg, layer.gate_bias)) <= \
        (TOL_OUT if dtype == "bf16" else 1e-4)


def test_plain_read_measurement_aid():
    """The plain streaming-read kernel runs over an odd-sized buffer, leaves ordinary data and its
    sink alone, and refuses a misaligned buffer."""
    buf = torch.arange(3 * 1024 * 1024 + 5, dtype=torch.int32, device="cuda")
    keep = buf.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    mm.moe_profile_plain_read(buf, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep) and int(sink.item()) == 0
    with pytest.raises(mm.MoeError):
        mm.moe_profile_plain_read(buf[1:], sink)
