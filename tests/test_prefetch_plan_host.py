"""The library's prefetch plan unit (csrc/prefetch_plan.cpp: plain host C++, no HIP) without a GPU,
built with -fsanitize=address,undefined: its request lists against the oracle's selection on the
same router logits (Sec. III-B: the rejected pass's router outputs name the big pass's experts),
with ties, NaN and infinities, and its schedule against the statement of the rule (at distance d
the list of layer j is requested when layer j - d is about to run, or at the start of the pass)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_12357_amd", "csrc")


@pytest.fixture(scope="module")
def plan_bin(tmp_path_factory):
    cxx = shutil.which(os.environ.get("CXX", "g++"))
    if cxx is None:
        pytest.skip("no host C++ compiler")
    out = str(tmp_path_factory.mktemp("plan") / "prefetch_plan_check")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-Werror", "-I", CSRC,
           os.path.join(ROOT, "tests", "host", "prefetch_plan_check.cpp"), os.path.join(CSRC, "prefetch_plan.cpp"),
           "-o", out]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return out


def run_plan(binary, logits, k, rejected, points=()):
    L, T, E = logits.shape
    bits = logits.astype(np.float32).view(np.uint32).ravel()
    text = f"{L} {E} {k} {T} {len(rejected)}\n" + " ".join(map(str, rejected)) + "\n" + \
           " ".join(f"{b:x}" for b in bits) + "\n" + "".join(f"{l} {d}\n" for l, d in points)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([binary], input=text, capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    lines = r.stdout.strip().splitlines()
    lists = [[int(v) for v in ln.split()[1:]] for ln in lines[1:1 + L]]
    due = [[int(v) for v in ln.split()[1:]] for ln in lines[1 + L:]]
    return lines[0], lists, due


def expected_lists(logits, k, rejected):
    """The oracle's big-mode selection of the rejected tokens, rank by rank, each expert once."""
    out = []
    for l in range(logits.shape[0]):
        idx = oracle.route(logits[l][rejected], None, 0.5, k, max(1, k // 2), False)[0]
        seen = []
        for j in range(k):
            for e in idx[:, j]:
                if int(e) not in seen:
                    seen.append(int(e))
        out.append(seen)
    return out


def test_request_lists_equal_the_oracles_selection(plan_bin):
    rng = np.random.default_rng(5)
    for case in range(12):
        L, T, E = int(rng.integers(1, 6)), int(rng.integers(1, 20)), int(rng.choice([3, 8, 60, 64, 256]))
        k = int(rng.integers(1, min(E, 8) + 1))
        logits = rng.standard_normal((L, T, E)).astype(np.float32)
        if case % 3 == 0:
            logits = np.round(logits * 2) / 2                    # many equal logits: the lowest id wins
        if case % 4 == 1:
            logits[rng.random(logits.shape) < 0.1] = np.nan      # NaN counts as -infinity
            logits[rng.random(logits.shape) < 0.05] = -np.inf
            logits[rng.random(logits.shape) < 0.02] = np.inf
        n = int(rng.integers(1, T + 1))
        rejected = sorted(rng.choice(T, size=n, replace=False).tolist())
        status, lists, _ = run_plan(plan_bin, logits, k, rejected)
        assert status == "ok"
        assert lists == expected_lists(logits, k, rejected), case


def test_a_row_of_equal_logits_and_a_row_of_nan(plan_bin):
    logits = np.zeros((1, 2, 6), np.float32)
    logits[0, 1] = np.nan
    _, lists, _ = run_plan(plan_bin, logits, 3, [0, 1])
    assert lists == [[0, 1, 2]]                                  # both rows: ids 0, 1, 2 in this order


def test_no_rejection_and_bad_token(plan_bin):
    logits = np.zeros((2, 3, 4), np.float32)
    status, lists, _ = run_plan(plan_bin, logits, 2, [])
    assert status == "ok" and lists == [[], []]
    status, lists, _ = run_plan(plan_bin, logits, 2, [3])
    assert status == "bad" and lists == [[], []]


def test_schedule(plan_bin):
    """Over one pass (start, then every layer in order) each layer's list is requested exactly once
    for d >= 1, never later than d layers before its own turn, and never for d = 0."""
    for L in (1, 4, 7):
        logits = np.zeros((L, 1, 4), np.float32)
        for d in range(0, L + 3):
            points = [(-1, d)] + [(l, d) for l in range(L)]
            _, _, due = run_plan(plan_bin, logits, 1, [0], points)
            when = {}
            for (layer, _), ls in zip(points, due):
                for j in ls:
                    assert j not in when
                    when[j] = layer
            if d == 0:
                assert when == {}
                continue
            assert sorted(when) == list(range(L))
            for j, layer in when.items():
                assert layer == max(-1, j - d)
