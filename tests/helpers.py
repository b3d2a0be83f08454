"""Shared by the tests: fixture paths and the comparison of a GPU run with the oracle."""

import os

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def hostcheck_library():
    """The host runtime linked with the byte-less device double, loaded.  tests/test_host_mutants.py points
    MW_HOSTCHECK_UNDER_TEST at a deliberately broken build to see that these tests notice."""
    import ctypes

    from paper_2407_08980_amd import build as mwbuild

    return ctypes.CDLL(os.environ.get("MW_HOSTCHECK_UNDER_TEST") or mwbuild.fresh_hostcheck())


def golden(name):
    return os.path.join(ROOT, "tests", "golden", name)


def read_kv(path):
    """Parse a golden text fixture: '#' comments, then 'key: value' lines (keys may repeat)."""
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            out.setdefault(key.strip(), []).append(val.strip())
    return out


def compare_runs(trace, orun, grun, require_checks=True):
    """GPU run vs oracle run of the same trace.

    Statuses must agree for every posting op.  Snapshots of buffers last written
    by a completed all-reduce are held to the summation tolerance; every other
    snapshot is compared byte for byte.  Returns a small report dict."""
    import oracle

    assert set(orun.status) == set(grun.status)
    bad = [(i, trace.ops[i].kind, orun.status[i], grun.status[i]) for i in sorted(orun.status)
           if orun.status[i] != grun.status[i]]
    assert not bad, f"status mismatches (index, kind, oracle, gpu): {bad[:10]} (+{max(0, len(bad) - 10)} more)"
    n_exact = n_tol = 0
    worst = 0.0
    for idx, ref in orun.snapshots.items():
        if ref is None:
            continue
        got = grun.snapshots[idx]
        assert got.shape == ref.shape, f"snapshot {idx}: size differs"
        if idx in orun.reduce_ref:
            s, sabs, count, dtype = orun.reduce_ref[idx]
            ok, w = oracle.allreduce_within_tolerance(got, s, sabs, count, dtype)
            worst = max(worst, w)
            assert ok, f"all-reduce snapshot {idx} ({dtype}, {count} elements): worst ratio {w:.3e}"
            n_tol += 1
        else:
            if not np.array_equal(got, ref):
                diff = np.flatnonzero(got != ref)
                raise AssertionError(
                    f"snapshot {idx} (buffer {trace.ops[idx].buf}): {diff.size} bytes differ, first at {diff[0]}")
            n_exact += 1
    if require_checks:
        assert n_exact + n_tol > 0, "trace had no data checks"
    return {"exact": n_exact, "toleranced": n_tol, "worst_allreduce_ratio": worst}
