"""The host side of the library (planner, argument checks of every entry point) under AddressSanitizer and
UndefinedBehaviorSanitizer: tests/sanitize/host_check.cpp is linked with the library's own sources, host code
instrumented, and run on seeded planner inputs (outputs compared with the oracle, every buffer sized exactly) and
on a battery of calls each entry point must refuse before launching anything.  No GPU needed."""
import os
import subprocess

import numpy as np
import pytest

import vlc_synth as syn
from oracle import vlc_oracle as orc
from paper_2512_12977_amd.runner import segments_of
from helpers import plan_steps, counts_for

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def host_check():
    from paper_2512_12977_amd.build import build_host_check
    return build_host_check()


def run(exe, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe, *args], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, "sanitizer build failed or reported:\n" + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_refused_calls_under_sanitizers(host_check):
    out = run(host_check, "errors").splitlines()
    codes = [int(v) for v in out[0].split()[1:]]
    N, S, D, I, W, F = 1, 2, 3, 4, 5, 7      # NULL, SHAPE, DTYPE, INDEX, WORKSPACE, INFEASIBLE
    want = [N, S, S, S, S,                    # rate planners: NULL table, L = 0, G > 500, negative budgets
            F, I, S, S, N, S, S, F, N, S,     # index builders: rising rate, overlap, k > 500, cap, no k, caps, rising, budget
            D, S, N, 0, S,                    # gather: dtype, 6-byte rows, NULL, no rows, misaligned
            S, S, N, S, N, S,                 # rope shift: D = 96, negative count, NULL delta, base; job table NULL / misaligned
            I, N,                             # scatter: more rows than cache, NULL v
            S, N, 0,                          # attention: Hq % Hkv, NULL lengths, no rows
            1, 1, 1, 0, N,                    # workspace queries (as booleans), layout ok, layout NULL
            F, N, N, S, W, N, S,              # layer: n > n_in, NULL lists, NULL weights, alias, workspace, events, flag
            S, W, W, 0,                       # first token: H, workspace; no-alloc: beyond the array, no requests
            S, W,                             # mean squared error: n = 0, workspace
            N, S]                             # MFMA probe: NULL, waves per SIMD
    assert codes == want


def planner_input(path, sens, budget, segs, k, explicit, cap):
    L, G1 = sens.shape
    with open(path, "w") as f:
        f.write("%d %d %d\n" % (L, G1 - 1, budget))
        f.write(" ".join(repr(float(v)) for v in sens.ravel()) + "\n")
        f.write("%d\n" % len(segs))
        for s in segs:
            f.write("%d %d %d %d %d %d %d\n" % (s.start, s.length, s.is_image, s.pos, s.old_pos, s.cache_row, s.kv_start))
        sel = k if k is not None else explicit
        f.write("%d %d\n%s\n" % (1 if k is not None else 0, cap, " ".join(str(int(v)) for v in sel)))


@pytest.mark.parametrize("name", ["c1", "c3", "c2"])
def test_planner_under_sanitizers_equals_oracle(host_check, name, tmp_path):
    wl = syn.make_workload(name)
    L = wl.shape.L
    k, explicit = plan_steps(wl)
    segs = segments_of(wl.requests)
    sens = syn.sensitivity_table(L, 150, 1)
    if name == "c2":
        sens[0] = sens[0, 0]                  # flat first layer: the run-based greedy's case
    budget = orc.budget_steps_from_mean_rate(500, L)
    cap = wl.total_slots                       # the exact number of rows a layer can have at most
    path = str(tmp_path / "in.txt")
    planner_input(path, sens, budget, segs, k, explicit, cap)
    lines = run(host_check, "planner", path).splitlines()
    it = iter(lines)

    def ints(line):
        return [int(v) for v in line.split()]

    head = next(it).split()
    assert head[0] == "rates" and int(head[1]) == 0
    np.testing.assert_array_equal([int(v) for v in head[2:]], orc.plan_layer_rates(sens, budget))
    head = next(it).split()
    assert head[0] == "blocks" and int(head[1]) == 0
    np.testing.assert_array_equal([int(v) for v in head[2:]], orc.plan_layer_rates_blocks(sens, budget))
    assert next(it).split() == ["indices", "0"]
    got = []
    for l in range(L):
        n = int(next(it).split()[1])
        arrs = [ints(next(it)) for _ in range(5)]
        assert all(len(a) == n for a in arrs)
        got.append(arrs)
    assert next(it).split() == ["next", "0"]
    nxt = [ints(next(it)) for _ in range(L)]
    assert next(it).split() == ["reuse", "0"]
    reuse = []
    for l in range(L):
        m = int(next(it).split()[1])
        arrs = [ints(next(it)) for _ in range(3)]
        assert all(len(a) == m for a in arrs)
        reuse.append(arrs)
    assert next(it).split() == ["budget", "0", str(orc.budget_steps_from_mean_rate(500, L))]
    for l in range(L):
        slots, src, dst, delta = [], [], [], []
        for req in wl.requests:
            counts = counts_for(req, k, explicit, l)
            slots.append(req.kv_start + orc.select_slots(req.segments, counts))
            rs, rr, ro = orc.reused_slots(req.segments, counts)
            src.append(rr)
            dst.append(req.kv_start + rs)
            delta.append(req.pos_start + rs - ro)
        slots = np.concatenate(slots)
        np.testing.assert_array_equal(got[l][0], slots)
        np.testing.assert_array_equal(reuse[l][0], np.concatenate(src))
        np.testing.assert_array_equal(reuse[l][1], np.concatenate(dst))
        np.testing.assert_array_equal(reuse[l][2], np.concatenate(delta))
        if l + 1 < L:
            below = np.concatenate([req.kv_start + orc.select_slots(req.segments, counts_for(req, k, explicit, l + 1))
                                    for req in wl.requests])
            at = np.searchsorted(below, slots)
            hit = (at < len(below)) & (below[np.minimum(at, len(below) - 1)] == slots)
            np.testing.assert_array_equal(nxt[l], np.where(hit, at, -1))
        else:
            assert set(nxt[l]) <= {-1}
