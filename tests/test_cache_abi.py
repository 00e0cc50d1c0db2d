"""Host-only checks of the Cache-Reuse part of the C ABI: exported symbols, argument errors
before any launch, and the cost accounting (pure host arithmetic) against the oracle."""
import ctypes
import math
import os
import re

import numpy as np

import paper_2509_22323_amd as ra
from oracle import cache_oracle as co
from paper_2509_22323_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "rapid_cache.h")).read()
A = 0x10000          # fake aligned "device" addresses: never dereferenced


def test_header_and_library_agree():
    declared = re.findall(r"RAPID_API\s+[\w\s\*]+?\b(rapid_\w+)\s*\(", HEADER)
    assert set(declared) == set(binding.CACHE_EXPORTS)
    ra.library()
    lib = ctypes.CDLL(ra.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_argument_errors_come_before_any_launch():
    lib = ra.library()
    S = ra.STATUS
    for f in (lib.rapid_cache_store, lib.rapid_cache_reuse):
        assert f(None, A, A, 1, 8, None, None) == S["RAPID_ERR_NULL"]
        assert f(A, None, A, 1, 8, None, None) == S["RAPID_ERR_NULL"]
        assert f(A, A, None, 1, 8, None, None) == S["RAPID_ERR_NULL"]
        assert f(A, A, A, 0, 8, None, None) == S["RAPID_ERR_SHAPE"]
        assert f(A, A, A, 1, 0, None, None) == S["RAPID_ERR_SHAPE"]
        assert f(A, A, A, 70000, 8, None, None) == S["RAPID_ERR_SHAPE"]
        assert f(A, A, A, 2, 1 << 40, None, None) == S["RAPID_ERR_SHAPE"]
        assert f(A + 1, A, A, 1, 8, None, None) == S["RAPID_ERR_ALIGN"]
        assert f(A, A, A + 3, 1, 8, None, None) == S["RAPID_ERR_ALIGN"]


def test_equivalent_steps_match_the_oracle():
    rng = np.random.default_rng(11)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        ac = rng.integers(0, 2, size=n).tolist()
        asp = rng.integers(0, 4, size=n).tolist()
        cc, cs = co.step_costs(ac, asp)
        want_exact, want_k = co.equivalent_steps(cc, cs)
        got_exact, got_k = ra.rapid_equivalent_steps(cc, cs)
        assert got_k == want_k and abs(got_exact - want_exact) < 1e-12
    assert ra.rapid_equivalent_steps([0.5], [0.0]) == (0.5, 1)
    assert ra.rapid_equivalent_steps([0.0, 0.0, 0.5], [0.0, 0.0, 0.0])[1] == 3
    assert ra.rapid_equivalent_steps([], []) == (0.0, 1)
    lib = ra.library()
    two = (ctypes.c_double * 2)(0.0, 1.5)
    ok = (ctypes.c_double * 2)(0.0, 0.0)
    assert lib.rapid_equivalent_steps(two, ok, 2, None) == ra.STATUS["RAPID_ERR_SHAPE"]
    assert lib.rapid_equivalent_steps(None, ok, 2, None) == ra.STATUS["RAPID_ERR_NULL"]
    assert lib.rapid_equivalent_steps(ok, ok, -1, None) == ra.STATUS["RAPID_ERR_SHAPE"]


def test_reward_matches_the_oracle():
    for K in (1, 3, 8, 15, 28):
        for q, d in ((0.8, 0.3), (-0.2, 0.9), (1.25, 0.0)):
            assert abs(ra.rapid_reward(q, d, K) - co.reward(q, d, K)) < 1e-13
            assert abs(ra.rapid_reward(q, d, K, lam=0.9, omega=0.5) - co.reward(q, d, K, lam=0.9, omega=0.5)) < 1e-13
    assert math.isnan(ra.rapid_reward(1.0, 1.0, 0))
