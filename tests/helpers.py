"""Shared by the GPU parity tests: oracle-side reference results for a workload."""
import numpy as np

import vlc_synth as syn
from oracle import vlc_oracle as orc


def plan_steps(wl):
    """(k per layer or None, explicit count per layer or None) for a workload, from the ORACLE planner."""
    L = wl.shape.L
    if wl.plan == "static":
        return np.full(L, wl.static_k, dtype=np.int32), None
    if wl.plan == "explicit":
        return None, np.full(L, wl.explicit_counts, dtype=np.int32)
    sens = syn.sensitivity_table(L, orc.PLANNER_G, 1)
    return orc.plan_layer_rates(sens, orc.budget_steps_from_mean_rate(wl.budget_bp, L)), None


def counts_for(req, k, explicit, l):
    return orc.image_counts(req.segments, k=None if k is None else int(k[l]),
                            explicit=None if explicit is None else int(explicit[l]))


def tolerance(dtype):
    """abs(g - o) <= atol + rtol * abs(o): 2e-2 / 1e-2 for bf16 storage, 1e-5 for fp32."""
    return (2e-2, 1e-2) if dtype == "bf16" else (1e-5, 1e-5)


def assert_close(got, want, dtype, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    atol, rtol = tolerance(dtype)
    err = np.abs(got - want)
    bound = atol + rtol * np.abs(want)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s got %r want %r (max abs err %.3e)"
                             % (what, int(bad.sum()), bad.size, i, got[i], want[i], err.max()))
    return float(err.max())
