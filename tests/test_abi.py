"""The C-ABI library loads and exports what include/rt.h declares; host-only entry points behave (no GPU)."""
import os
import re

import numpy as np
import pytest

from paper_2604_21215_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "rt.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(rt_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.load()
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(binding.EXPORTS)
    assert L.rt_version() >= 100


def test_status_strings_and_null_context():
    L = binding.load()
    assert L.rt_status_string(0) == b"RT_OK"
    assert L.rt_status_string(2) == b"RT_ERR_UNSUPPORTED"
    assert L.rt_last_error(None) == b"no context"
    assert L.rt_destroy(None) == 0
    assert L.rt_workspace_bytes(None) == 0
    assert L.rt_create(None, None) == binding.RT_ERR_INVALID_ARG


def test_paper_examples_in_the_driver_schedule():
    ev = {e[0]: e for e in binding.rt_schedule_events(8, 1)}
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "schedule_examples.txt")) if l[0] != "#"]
    for t, P, u, v, s, e in (tuple(int(a) for a in r) for r in rows):
        assert ev[t] == (t, P, u, v, s)


@pytest.mark.parametrize("N,p_min", [(1, 1), (2, 1), (7, 1), (100, 1), (100, 4), (257, 32), (300, 64), (1000, 32), (64, 64)])
def test_driver_schedule_plus_direct_window_covers_every_pair_once(N, p_min):
    ev = binding.rt_schedule_events(N, p_min)
    cover = np.zeros((N + 1, N + 1), dtype=np.int32)
    per_level_slots = {}
    for (t, P, u, v, s) in ev:
        assert P >= p_min and t % P == 0 and (t // P) % 2 == 1 and u == t + 1 and v == min(t + P, N) and s == t - P + 1
        cover[u:v + 1, s:t + 1] += 1
        lvl = P.bit_length() - 1
        for q in range(u, v + 1):
            slot = binding.rt_partial_slot(lvl, q)
            assert 0 <= slot < (N + 1) // 2
            assert slot not in per_level_slots.setdefault(lvl, set())      # written once
            per_level_slots[lvl].add(slot)
    for i in range(1, N + 1):                                               # direct window of query i
        w = (i - 1) % p_min
        cover[i, i - w:i] += 1
    for i in range(1, N + 1):
        assert (cover[i, 1:i] == 1).all() and (cover[i, i:] == 0).all()
    # a query takes a tile at a level exactly when that bit of (i-1) is set
    for i in range(1, N + 1):
        for lvl in range(0, 12):
            has = binding.rt_partial_slot(lvl, i) >= 0
            assert has == bool(((i - 1) >> lvl) & 1)


def test_schedule_rejects_bad_arguments():
    L = binding.load()
    assert L.rt_schedule_events(0, 32, None, 0) == -1
    assert L.rt_schedule_events(16, 3, None, 0) == -1
    assert L.rt_partial_slot(-1, 4) == -1
    assert L.rt_partial_slot(2, 0) == -1


@pytest.mark.parametrize("N,p_min", [(1, 32), (2, 32), (33, 32), (34, 32), (100, 32), (257, 32), (300, 64), (1000, 32), (129, 128)])
def test_shifted_schedule_of_the_persistent_engine_covers_every_pair_once(N, p_min):
    """Query i: newest key i-1 directly, window and stored partials from the bits of c = i-2."""
    ev = binding.rt_schedule_events_shifted(N, p_min)
    cover = np.zeros((N + 2, N + 2), dtype=np.int32)
    slots = {}
    for (t, P, u, v, s) in ev:
        assert P >= p_min and t % P == 0 and (t // P) % 2 == 1 and s == t - P + 1
        assert u == t + 2 and v == min(t + P + 1, N) and u <= v
        cover[u:v + 1, s:t + 1] += 1
        lvl = P.bit_length() - 1
        for q in range(u, v + 1):
            slot = binding.rt_partial_slot(lvl, q - 1)          # stored under c + 1 = q - 1 (1-based)
            assert 0 <= slot < (N + 1) // 2 and slot not in slots.setdefault(lvl, set())
            slots[lvl].add(slot)
    for i in range(1, N + 1):
        if i >= 2:
            cover[i, i - 1] += 1                                 # newest key
            c = i - 2
            w = c % p_min
            cover[i, c - w + 1:c + 1] += 1                       # direct window
    for i in range(1, N + 1):
        assert (cover[i, 1:i] == 1).all() and (cover[i, i:] == 0).all(), i


@pytest.mark.parametrize("N,p_min,chunk", [(1, 32, 64), (40, 32, 64), (100, 32, 32), (130, 4, 16), (300, 32, 64), (1000, 32, 128),
                                           (257, 64, 64), (75, 8, 32)])
def test_chunked_schedule_of_the_layer_wavefront_engine_covers_every_pair_once(N, p_min, chunk):
    """Blocks below the chunk as in the driver schedule, one tile over all earlier keys per chunk, direct window below
    p_min; every event's queries lie in the chunk that starts right after the event's last key."""
    ev = binding.rt_schedule_events_chunked(N, p_min, chunk)
    cover = np.zeros((N + 1, N + 1), dtype=np.int32)
    n_far = 0
    for (t, P, u, v, s) in ev:
        assert u == t + 1 and u <= v <= N
        if s == 1 and P == t and t % chunk == 0:            # far tile
            assert v == min(t + chunk, N)
            n_far += 1
        else:
            assert p_min <= P < chunk and t % P == 0 and (t // P) % 2 == 1 and v == min(t + P, N) and s == t - P + 1
        assert (u - 1) // chunk == (v - 1) // chunk        # one chunk, known when the layer enters it
        assert (u - 1) // chunk == t // chunk or t % chunk == 0
        cover[u:v + 1, s:t + 1] += 1
    assert n_far == (N - 1) // chunk
    for i in range(1, N + 1):
        w = (i - 1) % p_min
        cover[i, i - w:i] += 1
    for i in range(1, N + 1):
        assert (cover[i, 1:i] == 1).all() and (cover[i, i:] == 0).all(), i
    assert binding.load().rt_schedule_events_chunked(16, 32, 16, None, 0) == -1     # chunk < p_min
    assert binding.load().rt_schedule_events_chunked(16, 4, 24, None, 0) == -1      # not a power of two


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on exactly one GPU: --gpus N with N > 1 ends with a message and a non-zero status before anything
    touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
