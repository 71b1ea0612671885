"""Helpers of the GPU parity tests: contexts on both sides from one workload description and
element-by-element comparison.  The oracle side never sees anything the GPU computed."""
import numpy as np

import workloads
from oracle import capi

SEED = bytes(range(64, 80))


def both(k, rule=0, seed=SEED, digits=None, lam=None):
    """(GPU context, oracle) for the first k primes; lam: explicit label lengths of the primes"""
    from paper_2302_06361_amd import Context
    primes = workloads.PRIMES[:k]
    digits = list(digits or workloads.DIGITS[k])
    return Context(primes, seed, digits, rule, lam=lam), capi.Oracle(primes, digits, seed, rule, lam=lam)


def upload_bundle(ctx, arrays):
    from paper_2302_06361_amd import Labels
    n = arrays[0].shape[0]
    t = Labels(ctx, n)
    for i, a in enumerate(arrays):
        t.from_numpy(i, a)
    return t


def assert_bundle_equal(gpu_labels, ref_arrays, what=""):
    for i, a in enumerate(ref_arrays):
        got = gpu_labels.to_numpy(i)
        bad = np.argwhere(got != a)
        assert bad.size == 0, "%s residue %d: %d digits differ, first at %s" % (what, i, len(bad), bad[:1].tolist())
        assert gpu_labels.pad_is_zero(i), "%s residue %d: pad digits not zero" % (what, i)


def assert_tables_equal(gpu_tables, ref, what=""):
    got = gpu_tables.cpu().numpy()
    assert got.size == ref.size, (what, got.size, ref.size)
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, "%s: %d table bytes differ, first at %d" % (what, bad.size, bad[0])
