"""The library's cache policy unit (csrc/cache_policy.cpp: plain host C++, no HIP) replayed without
a GPU, built with -fsanitize=address,undefined, against the host-only model of the oracle: random
DEMAND / PREFETCH traces (slots, counts, copy order, occupancy after every call), the hand-worked
traces, the error returns (which must leave the state untouched) and the wave order."""
import os
import random
import shutil
import subprocess

import pytest

from oracle.cache_model import DEMAND, PREFETCH, CacheModel
from test_cache_model import HAND_TRACES, random_history

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_12357_amd", "csrc")


@pytest.fixture(scope="module")
def replay_bin(tmp_path_factory):
    cxx = shutil.which(os.environ.get("CXX", "g++"))
    if cxx is None:
        pytest.skip("no host C++ compiler")
    out = str(tmp_path_factory.mktemp("policy") / "cache_policy_replay")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-Werror", "-I", CSRC,
           os.path.join(ROOT, "tests", "host", "cache_policy_replay.cpp"), os.path.join(CSRC, "cache_policy.cpp"),
           "-o", out]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return out


def replay(binary, E, n_slots, lines):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1")
    env.pop("LD_PRELOAD", None)                 # the sanitizer runtime wants to be the first library
    r = subprocess.run([binary], input=f"{E} {n_slots}\n" + "\n".join(lines) + "\n", capture_output=True, text=True,
                       env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    return r.stdout.strip().splitlines()


def call_line(ids, mode, limit):
    return " ".join(map(str, [mode, len(ids), -1 if limit is None else limit, *ids]))


def parse(line):
    rc, slots, counts, copies, occ = [p.split() for p in line.split("|")]
    return (int(rc[0]), [int(v) for v in slots], tuple(int(v) for v in counts),
            [tuple(int(v) for v in c.split(":")) for c in copies], [int(v) for v in occ])


def test_random_traces_equal_the_model(replay_bin):
    for seed in range(10):
        rnd = random.Random(500 + seed)
        E, n_slots = rnd.choice([(12, 3), (64, 16), (9, 8), (256, 24), (5, 1)])
        hist = random_history(rnd, E, n_slots, 300)
        out = replay(replay_bin, E, n_slots, [call_line(*h) for h in hist])
        assert len(out) == len(hist)
        m = CacheModel(E, n_slots)
        for i, ((ids, mode, limit), line) in enumerate(zip(hist, out)):
            before = list(m.slot_expert)
            slots, hits, misses, dropped = m.fetch(ids, mode, limit) if mode == PREFETCH else m.fetch(ids, mode)
            rc, g_slots, g_counts, g_copies, g_occ = parse(line)
            assert rc == 0
            assert g_slots == list(slots) and g_counts == (hits, misses, dropped), (seed, i)
            assert g_occ == list(m.slot_expert), (seed, i)
            # the copies are exactly the experts that were not resident before and are now, each into
            # its slot; DEMAND issues them in ascending expert id, PREFETCH in the caller's order
            loaded = [(e, s) for e, s in zip(ids, slots) if s >= 0 and e not in before]
            assert g_copies == (sorted(loaded) if mode == DEMAND else loaded), (seed, i)


def test_hand_traces(replay_bin):
    for E, n_slots, calls in HAND_TRACES:
        out = replay(replay_bin, E, n_slots, [call_line(c[0], c[1], c[2]) for c in calls])
        for c, line in zip(calls, out):
            rc, slots, counts, _, occ = parse(line)
            assert rc == 0 and slots == c[3] and counts == c[4] and occ == c[5]


def test_errors_change_nothing_and_wave_order(replay_bin):
    lines = [call_line([3, 1], DEMAND, None),           # ok: 1 -> slot 0, 3 -> slot 1
             call_line([0, 1, 2], DEMAND, None),        # more than the 2 slots
             call_line([1, 1], DEMAND, None),           # named twice
             call_line([6], PREFETCH, None),            # id out of range
             call_line([-1], DEMAND, None),
             "7 0 -1",                                  # unknown mode
             call_line([], PREFETCH, None),
             "w 4 0 1 3 5",                             # residents (1, 3) first, then 0, 5
             call_line([1, 5], DEMAND, None)]           # the state is what the first call left
    out = replay(replay_bin, 6, 2, lines)
    assert parse(out[0])[:3] == (0, [1, 0], (0, 2, 0))
    assert [parse(l)[0] for l in out[1:6]] == [3, 2, 1, 1, 4]
    assert all(parse(l)[4] == [1, 3] for l in out[1:7])
    assert out[7].split() == ["order", "1", "3", "0", "5"]
    assert parse(out[8]) == (0, [0, 1], (1, 1, 0), [(5, 1)], [1, 5])
