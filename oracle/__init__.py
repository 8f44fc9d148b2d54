"""CPU oracle of the big-little MoE layer -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``mobile_oracle.cpp`` (plain C++, double arithmetic) plus a
pure-Python model of the expert cache (``cache_model``).  Nothing under this folder is
part of the product: only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import it, and it imports nothing from the HIP package.

Storage conventions: activations and weights are numpy arrays of dtype ``float32`` or
``uint16`` (bf16 bit patterns); the oracle widens them exactly and computes in double.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mobile_oracle.cpp")
_LIB = os.path.join(_HERE, "libmobile_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for name in ("oracle_gate_logits", "oracle_token_confidence", "oracle_route",
                     "oracle_dispatch", "oracle_dispatch_from", "oracle_combine_add", "oracle_swiglu_rows", "oracle_expert_ffn",
                     "oracle_combine", "oracle_num_threads", "oracle_set_num_threads", "oracle_swiglu_rows_w8",
                     "oracle_e4m3_decode", "oracle_swiglu_rows_mx4", "oracle_e2m1_decode", "oracle_e8m0_decode"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError(f"oracle reads uint16 (bf16 bits) or float32 arrays, got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a: np.ndarray, dtype=None) -> np.ndarray:
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what}: bad argument (rc={rc})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads of the loops over independent rows from now on (timing only; results do not change)."""
    _load().oracle_set_num_threads(int(n))


def gate_logits(x: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    x, Wg = _c(x), _c(Wg)
    T, H = x.shape
    E = Wg.shape[0]
    assert Wg.shape[1] == H and _dtype_code(x) == _dtype_code(Wg)
    b = None if bias is None else _c(bias, np.float32)
    out = np.empty((T, E), np.float32)
    _check(_load().oracle_gate_logits(_p(x), _p(Wg), _p(b), T, H, E, _dtype_code(x), _p(out)),
           "gate_logits")
    return out


def token_confidence(lm_logits: np.ndarray) -> np.ndarray:
    z = _c(lm_logits, np.float32)
    T, V = z.shape
    out = np.empty((T,), np.float32)
    _check(_load().oracle_token_confidence(_p(z), T, V, _p(out)), "token_confidence")
    return out


def route(logits: np.ndarray, conf: Optional[np.ndarray], gamma: float, k_big: int,
          k_little: int, renorm: bool):
    """-> (topk_idx int32 [T,K], topk_w float32 [T,K], important uint8 [T], k_t int32 [T])"""
    lg = _c(logits, np.float32)
    T, E = lg.shape
    cf = None if conf is None else _c(conf, np.float32)
    idx = np.empty((T, k_big), np.int32)
    w = np.empty((T, k_big), np.float32)
    imp = np.empty((T,), np.uint8)
    kt = np.empty((T,), np.int32)
    _check(_load().oracle_route(_p(lg), _p(cf), ctypes.c_float(gamma), T, E, k_big, k_little,
                                int(bool(renorm)), _p(idx), _p(w), _p(imp), _p(kt)), "route")
    return idx, w, imp, kt


def dispatch(topk_idx: np.ndarray, k_t: np.ndarray, E: int):
    """-> (expert_offsets [E+1], sorted_token [T*K], sorted_rank [T*K], inv_pos [T,K]) int32"""
    idx = _c(topk_idx, np.int32)
    kt = _c(k_t, np.int32)
    T, K = idx.shape
    off = np.empty((E + 1,), np.int32)
    st = np.empty((T * K,), np.int32)
    sr = np.empty((T * K,), np.int32)
    inv = np.empty((T, K), np.int32)
    _check(_load().oracle_dispatch(_p(idx), _p(kt), T, E, K, _p(off), _p(st), _p(sr), _p(inv)),
           "dispatch")
    return off, st, sr, inv


def w8_blob_bytes(H: int, I: int) -> int:
    """Bytes of an expert with 8-bit weights: 3*H*I E4M3 codes + (2*I + H) fp32 row scales."""
    return 3 * H * I + 4 * (2 * I + H)


def mx4_blob_bytes(H: int, I: int) -> int:
    """Bytes of an expert in MXFP4: 3*H*I codes of 4 bits + one E8M0 scale byte per 32 weights."""
    return 3 * H * I // 2 + 3 * H * I // 32


def e2m1_decode(codes: np.ndarray) -> np.ndarray:
    """Values of E2M1 codes (OCP microscaling 4-bit element; low four bits of each byte) -> float64."""
    c = _c(codes, np.uint8).ravel()
    out = np.empty(c.shape, np.float64)
    _check(_load().oracle_e2m1_decode(_p(c), c.size, _p(out)), "e2m1_decode")
    return out.reshape(np.shape(codes))


def e8m0_decode(scales: np.ndarray) -> np.ndarray:
    """Values of E8M0 scales (OCP microscaling: 2^(b - 127), 255 = NaN) -> float64."""
    c = _c(scales, np.uint8).ravel()
    out = np.empty(c.shape, np.float64)
    _check(_load().oracle_e8m0_decode(_p(c), c.size, _p(out)), "e8m0_decode")
    return out.reshape(np.shape(scales))


def _weight_format(blob: np.ndarray, H: int, I: int) -> int:
    """0: weights in the activations' type; 1: 8-bit codes with row scales; 2: MXFP4.  Byte blobs
    are told apart by their size."""
    if blob.dtype != np.uint8:
        return 0
    w8, mx = blob.size == w8_blob_bytes(H, I), H % 32 == 0 and I % 32 == 0 and blob.size == mx4_blob_bytes(H, I)
    assert w8 != mx, "a byte blob must have the size of the 8-bit or of the MXFP4 layout"
    return 1 if w8 else 2


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Values of E4M3 ("e4m3fn", OCP 8-bit floating point) codes -> float64."""
    c = _c(codes, np.uint8).ravel()
    out = np.empty(c.shape, np.float64)
    _check(_load().oracle_e4m3_decode(_p(c), c.size, _p(out)), "e4m3_decode")
    return out.reshape(np.shape(codes))


def swiglu_rows(x: np.ndarray, blob: np.ndarray, I: int,
                tok: Optional[np.ndarray] = None) -> np.ndarray:
    """One expert (blob = [W_gate I*H | W_up I*H | W_down H*I] flat) on rows ``tok`` of x
    (all rows in order when ``tok`` is None).  A uint8 blob holds 8-bit weights (E4M3 codes in
    the same order, then the fp32 row scales [gate I | up I | down H]) or MXFP4 weights (codes two
    per byte in the same order, then one E8M0 scale per 32 weights), told apart by its size.
    -> float64 [n,H]"""
    x, blob = _c(x), _c(blob)
    T, H = x.shape
    tk = None if tok is None else _c(tok, np.int32)
    n = T if tk is None else tk.shape[0]
    y = np.empty((n, H), np.float64)
    fmt = _weight_format(blob, H, I)
    if fmt == 1:
        _check(_load().oracle_swiglu_rows_w8(_p(x), _dtype_code(x), H, I, _p(blob), _p(tk), n, _p(y)),
               "swiglu_rows_w8")
        return y
    if fmt == 2:
        _check(_load().oracle_swiglu_rows_mx4(_p(x), _dtype_code(x), H, I, _p(blob), _p(tk), n, _p(y)),
               "swiglu_rows_mx4")
        return y
    assert blob.size == 3 * H * I and _dtype_code(blob) == _dtype_code(x)
    _check(_load().oracle_swiglu_rows(_p(x), _dtype_code(x), H, I, _p(blob), _p(tk), n, _p(y)),
           "swiglu_rows")
    return y


def expert_ffn(x: np.ndarray, expert_w: Sequence[np.ndarray], I: int, expert_offsets: np.ndarray,
               sorted_token: np.ndarray) -> np.ndarray:
    """-> float64 [P,H], row p = expert FFN of the pair at dispatch position p"""
    x = _c(x)
    T, H = x.shape
    E = len(expert_w)
    blobs = [_c(b) for b in expert_w]
    w8 = _weight_format(blobs[0], H, I) if blobs else 0
    for b in blobs:
        if w8:
            assert _weight_format(b, H, I) == w8
        else:
            assert b.size == 3 * H * I and _dtype_code(b) == _dtype_code(x)
    ptrs = (ctypes.c_void_p * E)(*[b.ctypes.data for b in blobs])
    off = _c(expert_offsets, np.int32)
    st = _c(sorted_token, np.int32)
    P = int(off[E])
    y = np.zeros((P, H), np.float64)
    _check(_load().oracle_expert_ffn(_p(x), _dtype_code(x), H, I, E, _p(off), _p(st), ptrs, int(w8), _p(y)),
           "expert_ffn")
    return y


def combine(y: np.ndarray, topk_w: np.ndarray, inv_pos: np.ndarray, k_t: np.ndarray,
            shared: Optional[np.ndarray], T: int, H: int) -> np.ndarray:
    """-> float64 [T,H];  shared: float64 [n_shared,T,H] or None"""
    y = _c(y, np.float64)
    w = _c(topk_w, np.float32)
    inv = _c(inv_pos, np.int32)
    kt = _c(k_t, np.int32)
    K = w.shape[1]
    sh = None if shared is None else _c(shared, np.float64)
    ns = 0 if sh is None else sh.shape[0]
    out = np.empty((T, H), np.float64)
    _check(_load().oracle_combine(_p(y), _p(w), _p(inv), _p(kt), _p(sh), ns, T, H, K, _p(out)),
           "combine")
    return out


def dispatch_from(topk_idx: np.ndarray, k_t: np.ndarray, j_lo: int, E: int):
    """Dispatch of the ranks j_lo <= j < k_t[t] only -> same four arrays as dispatch()."""
    idx = _c(topk_idx, np.int32)
    kt = _c(k_t, np.int32)
    T, K = idx.shape
    off = np.empty((E + 1,), np.int32)
    st = np.empty((T * K,), np.int32)
    sr = np.empty((T * K,), np.int32)
    inv = np.empty((T, K), np.int32)
    _check(_load().oracle_dispatch_from(_p(idx), _p(kt), int(j_lo), T, E, K, _p(off), _p(st), _p(sr),
                                        _p(inv)), "dispatch_from")
    return off, st, sr, inv


def combine_add(y: np.ndarray, topk_w: np.ndarray, inv_pos: np.ndarray, k_t: np.ndarray, j_lo: int,
                out: np.ndarray) -> np.ndarray:
    """-> out + sum over the ranks j_lo <= j < k_t[t] (float64 [T,H]); `out` is not modified"""
    y = _c(y, np.float64)
    w = _c(topk_w, np.float32)
    inv = _c(inv_pos, np.int32)
    kt = _c(k_t, np.int32)
    res = np.array(out, dtype=np.float64, order="C", copy=True)
    T, H = res.shape
    _check(_load().oracle_combine_add(_p(y), _p(w), _p(inv), _p(kt), int(j_lo), T, H, w.shape[1], _p(res)),
           "combine_add")
    return res


def fallback_increment(x: np.ndarray, expert_w: Sequence[np.ndarray], I: int, logits: np.ndarray,
                       conf: Optional[np.ndarray], gamma: float, k_big: int, k_little: int,
                       out_little: np.ndarray) -> dict:
    """Second pass of Alg. 1 at layer level: the tokens whose little result is rejected (conf not above
    gamma) get the big model's layer output.  With routing weights that are not renormalised the big
    layer output is the little one plus the experts of ranks k_little .. k_big-1, so only those are
    computed and added to `out_little` (the little pass's layer output, all tokens at k_little)."""
    idx, w, imp, kt = route(logits, conf, gamma, k_big, k_little, False)
    off, st, sr, inv = dispatch_from(idx, kt, k_little, len(expert_w))
    y = expert_ffn(x, expert_w, I, off, st)
    out = combine_add(y, w, inv, kt, k_little, out_little)
    return dict(topk_idx=idx, topk_w=w, important=imp, k_t=kt, expert_offsets=off, sorted_token=st,
                sorted_rank=sr, inv_pos=inv, y=y, out=out)


def moe_layer(x: np.ndarray, Wg: np.ndarray, gate_bias: Optional[np.ndarray],
              expert_w: Sequence[np.ndarray], I: int, shared_w: Sequence[np.ndarray],
              shared_I: Sequence[int], conf: Optional[np.ndarray], gamma: float, k_big: int,
              k_little: int, renorm: bool, logits: Optional[np.ndarray] = None) -> dict:
    """The whole layer, step by step (Sec. II-A selection + execution, Alg. 1 flagging)."""
    x = _c(x)
    T, H = x.shape
    E = len(expert_w)
    if logits is None:
        logits = gate_logits(x, Wg, gate_bias)
    idx, w, imp, kt = route(logits, conf, gamma, k_big, k_little, renorm)
    off, st, sr, inv = dispatch(idx, kt, E)
    y = expert_ffn(x, expert_w, I, off, st)
    shared = None
    if len(shared_w):
        shared = np.stack([swiglu_rows(x, b, Is) for b, Is in zip(shared_w, shared_I)])
    out = combine(y, w, inv, kt, shared, T, H)
    return dict(logits=logits, topk_idx=idx, topk_w=w, important=imp, k_t=kt, expert_offsets=off,
                sorted_token=st, sorted_rank=sr, inv_pos=inv, y=y, shared=shared, out=out)


def eq1_speedup(T: float, T_l: float, T_b: float, r: float) -> float:
    """Estimated speedup of Eq. 1 (Sec. III-B): a token costs the little model's latency T_l, and with
    probability r (the fallback ratio) the big model's latency T_b on top; T is the latency of the
    full model without the method."""
    return T / (T_l + r * T_b)


# ----------------------------------------------------------------------------- Alg. 1 as a loop
def alg1_generate(little_model, big_model, prompt: Sequence[int], gamma: float, eos: int,
                  max_new: int):
    """The inference loop of Alg. 1 (Sec. III-A) for one sequence.

    little_model(y) -> (p, h): distribution over the next token after the tokens y, and the router
    states h of that pass; big_model(y, h) -> p.  While the last token is not <eos>: run the little
    model; if its largest probability exceeds gamma keep its token, otherwise drop it and take the
    big model's.  Readings where the paper is silent: "sample" is the most probable token (lowest id
    among equals), and at most max_new tokens are generated.
    Returns (y, from_big) with one flag per generated token."""
    y = [int(t) for t in prompt]
    from_big = []
    while y[-1] != eos and len(from_big) < max_new:
        p_s, h_s = little_model(y)
        p_s = np.asarray(p_s, np.float64)
        if float(p_s.max()) > gamma:
            y.append(int(np.argmax(p_s)))
            from_big.append(False)
        else:
            p_l = np.asarray(big_model(y, h_s), np.float64)
            y.append(int(np.argmax(p_l)))
            from_big.append(True)
    return y, from_big


def _round_to_storage(a: np.ndarray, like: np.ndarray) -> np.ndarray:
    """Rounds double values to the storage type of `like` (float32, or bf16 bits in uint16, both
    round-to-nearest-even): activations between two layers are stored in the layer's dtype."""
    f = np.asarray(a, np.float64).astype(np.float32)
    if like.dtype == np.float32:
        return f
    bits = f.view(np.uint32).astype(np.uint64)
    bits = bits + 0x7FFF + ((bits >> 16) & 1)
    return (bits >> 16).astype(np.uint16)


def rms_normalize(x: np.ndarray) -> np.ndarray:
    """Rows of a stored activation divided by sqrt(mean of squares + 1e-6), stored in the same type."""
    x = _c(x)
    if x.dtype == np.uint16:
        f = (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        f = x.astype(np.float64)
    y = f / np.sqrt((f * f).mean(axis=1, keepdims=True) + 1e-6)
    return _round_to_storage(y, x)


def toy_lm_next(embed: np.ndarray, layers: Sequence[dict], head: np.ndarray, tokens: np.ndarray,
                big: np.ndarray, gamma: float, k_big: int, k_little: int, renorm: bool,
                norm: bool = False) -> dict:
    """One decoding step of a tiny attention-free language model built from MoE layers: embedding
    row of each token, the layers one after the other (a layer's output, rounded to the storage
    type, is the next layer's input), output head, softmax.  big[t] says whether token t runs the
    big model (k_big experts in every layer) or the little one (k_little), Sec. III-A.  With `norm`
    every layer's stored output row is divided by sqrt(mean of its squares + 1e-6) and stored again
    (a SwiGLU layer is quadratic in its input, so a deep stack without it collapses or blows up).
    Each entry of `layers` holds Wg, gate_bias, expert_w, I, shared_w, shared_I.
    Returns p [T,V] (double), lm_logits [T,V] (float32), conf [T], router logits per layer."""
    tokens = np.asarray(tokens, np.int64)
    big = np.asarray(big, bool)
    # Alg. 1 sends a token to the big model when its confidence does not exceed gamma
    conf = np.where(big, np.float32(-np.inf), np.float32(np.inf)).astype(np.float32)
    x = np.ascontiguousarray(embed[tokens])
    h = []
    for ly in layers:
        r = moe_layer(x, ly["Wg"], ly["gate_bias"], ly["expert_w"], ly["I"], ly["shared_w"], ly["shared_I"],
                      conf, gamma, k_big, k_little, renorm)
        h.append(r["logits"])
        x = _round_to_storage(r["out"], embed)
        if norm:
            x = rms_normalize(x)
    z = gate_logits(x, head, None)
    zz = z.astype(np.float64)
    e = np.exp(zz - zz.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    return dict(p=p, lm_logits=z, conf=token_confidence(z), router_logits=h, x_last=x)
