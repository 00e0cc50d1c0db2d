"""Pins of the Cache-Reuse / cost-accounting oracle against what the paper and arithmetic fix
(RAPID^3 Sec. 3.2 Level-2, Eq. 3; Sec. 3.3 reward; App. hyper-parameter table)."""
import re
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from oracle import cache_oracle as co


def bits(*vals):
    """bf16 bit patterns of values that ARE bf16 numbers (checked)."""
    a = np.array(vals, dtype=np.float32)
    b = (a.view(np.uint32) >> 16).astype(np.uint16)
    assert (co.bf16_to_f64(b) == a.astype(np.float64)).all(), "test value is not a bf16 number"
    return b


def exact_bf16(fr: Fraction) -> int:
    """Brute force: the bf16 bit pattern nearest to an exact rational, ties to even, found by
    scanning the neighbouring bit patterns of the correctly-signed magnitude."""
    sign = 0x8000 if fr < 0 else 0
    mag = abs(fr)
    if mag == 0:
        return sign
    lo, hi = 0, 0x7F80                                     # +0 .. +inf, monotone in value
    val = lambda p: Fraction(float(co.bf16_to_f64(np.array([p], np.uint16))[0])) if p < 0x7F80 else None
    while hi - lo > 1:                                     # largest pattern with value <= mag
        mid = (lo + hi) // 2
        if val(mid) <= mag:
            lo = mid
        else:
            hi = mid
    below, above = val(lo), (val(lo + 1) if lo + 1 < 0x7F80 else Fraction(2) ** 128)
    if mag - below < above - mag or (mag - below == above - mag and lo % 2 == 0):
        return sign | lo
    return sign | (lo + 1)


# ---------------------------------------------------------------- rounding
def test_rounding_hand_cases():
    one = 1.0
    cases = [
        (one + 2.0 ** -8, 1.0),                            # tie between 1 and 1+2^-7: even is 1
        (one + 2.0 ** -7 + 2.0 ** -8, one + 2.0 ** -6),    # tie: even mantissa is 2
        (one + 2.0 ** -8 + 2.0 ** -30, one + 2.0 ** -7),   # just above the tie
        (one + 2.0 ** -8 - 2.0 ** -30, 1.0),               # just below
        (2.0 ** -133, 2.0 ** -133),                        # smallest subnormal stays
        (2.0 ** -134, 0.0),                                # tie with 0: even is 0
        (1.5 * 2.0 ** -134, 2.0 ** -133),
        (-(one + 2.0 ** -8), -1.0),
        (2.0 ** 128 - 2.0 ** 120, 2.0 ** 128 - 2.0 ** 120),  # largest finite
        (2.0 ** 128 - 2.0 ** 119, np.inf),                 # tie at the top rounds to "even" = infinity
        (2.0 ** 128 - 2.0 ** 119 - 2.0 ** 90, 2.0 ** 128 - 2.0 ** 120),
        (np.inf, np.inf), (-np.inf, -np.inf),
    ]
    for x, want in cases:
        got = co.bf16_to_f64(co.f64_to_bf16(np.array([x])))[0]
        assert got == want, (x, got, want)
    assert np.isnan(co.bf16_to_f64(co.f64_to_bf16(np.array([np.nan])))[0])
    assert co.f64_to_bf16(np.array([-0.0]))[0] == 0x8000


def test_rounding_against_brute_force_and_an_independent_implementation():
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.normal(size=300), rng.normal(size=100) * 1e-39, rng.normal(size=100) * 1e38,
                        rng.integers(-512, 512, size=200) * 2.0 ** -9])           # many exact ties
    got = co.f64_to_bf16(x)
    want = np.array([exact_bf16(Fraction(float(v))) for v in x], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)
    f32 = rng.normal(size=4096).astype(np.float32) * np.float32(3.0)
    np.testing.assert_array_equal(co.f64_to_bf16(f32.astype(np.float64)), wl.f32_to_bf16_bits(f32))


# ---------------------------------------------------------------- residual operations
def test_store_and_reuse_exact_cases():
    o, x = bits(1.5, 1.0, -2.0, 1.0), bits(1.0, 1.5, 0.5, 2.0 ** -9)
    np.testing.assert_array_equal(co.cache_store(o, x), bits(0.5, -0.5, -2.5, 1.0))   # 1 - 2^-9: tie -> 1
    np.testing.assert_array_equal(co.cache_reuse(bits(1.0, 1.0, 256.0), bits(0.5, 2.0 ** -8, 1.0)),
                                  bits(1.5, 1.0, 256.0))                              # 257 ties to 256
    rng = np.random.default_rng(3)
    x = wl.f32_to_bf16_bits(rng.normal(size=2000).astype(np.float32))
    o = wl.f32_to_bf16_bits(rng.normal(size=2000).astype(np.float32))
    zero = np.zeros_like(x)
    np.testing.assert_array_equal(co.cache_store(o, zero), o)                 # X = 0: Delta = O
    np.testing.assert_array_equal(co.cache_reuse(x, zero), x)                 # Delta = 0: O = X
    assert (co.cache_store(x, x) == 0).all()                                  # G(X) = X: Delta = +0
    # brute force on exact rationals
    d = co.cache_store(o, x)
    xf, of = co.bf16_to_f64(x), co.bf16_to_f64(o)
    want = np.array([exact_bf16(Fraction(float(a)) - Fraction(float(b))) for a, b in zip(of, xf)], np.uint16)
    np.testing.assert_array_equal(d, want)
    # a reusing step right after the update gives the generator's output back to within the
    # two roundings (each at most half a unit in the last place of its own result)
    back = co.bf16_to_f64(co.cache_reuse(x, d))
    ulp = lambda v: np.maximum(2.0 ** (np.frexp(np.abs(v))[1] - 8), 2.0 ** -133)
    assert (np.abs(back - of) <= 0.5 * ulp(co.bf16_to_f64(d)) + 0.5 * ulp(back) + 1e-300).all()


def test_image_wise_reuse_leaves_other_samples_alone():
    rng = np.random.default_rng(5)
    x = wl.f32_to_bf16_bits(rng.normal(size=(3, 40)).astype(np.float32))
    d = wl.f32_to_bf16_bits(rng.normal(size=(3, 40)).astype(np.float32))
    out0 = np.full((3, 40), 0x1234, np.uint16)
    out = co.cache_reuse_batch(x, d, out0, [1, 0, 1])
    assert (out[1] == 0x1234).all()
    np.testing.assert_array_equal(out[[0, 2]], co.cache_reuse(x[[0, 2]], d[[0, 2]]))


# ---------------------------------------------------------------- cost accounting
def test_equivalent_steps_worked_examples():
    # 28 plain steps cost 28
    assert co.equivalent_steps([0.0] * 28, [0.0] * 28) == (28.0, 28)
    # 5 full, 4 cached (each costs 1 - 0.95), 3 with the first sparse candidate (1 - 0.05)
    cc, cs = co.step_costs([0] * 5 + [1] * 4 + [0] * 3, [0] * 5 + [3] * 4 + [1] * 3)
    assert cs[5:9] == [0.0] * 4                            # sparse policy inactive on cached steps
    k, kr = co.equivalent_steps(cc, cs)
    assert abs(k - (5 + 4 * 0.05 + 3 * 0.95)) < 1e-12 and kr == 8
    # both reductions on one step multiply
    k, _ = co.equivalent_steps([0.95], [0.10])
    assert abs(k - 0.05 * 0.90) < 1e-15
    # ties away from zero, never below one
    assert co.equivalent_steps([0.5], [0.0])[1] == 1
    assert co.equivalent_steps([0.0, 0.0, 0.5], [0.0] * 3)[1] == 3
    assert co.equivalent_steps([0.95], [0.0])[1] == 1
    assert co.C_SPARSE == (0.0, 0.05, 0.07, 0.10) and co.C_CACHE == 0.95 and co.LAMBDA == 0.97 and co.OMEGA == 1.0


def paper_reward_constants():
    """tests/golden/reward_constants.txt: the values the paper prints (its citation is in the file)."""
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "reward_constants.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *rest = line.split()
                vals[name] = [float(x) for x in rest]
    return vals


def test_constants_are_the_ones_the_paper_prints():
    g = paper_reward_constants()
    assert [co.LAMBDA] == g["lambda"] and [co.OMEGA] == g["omega"] and [co.C_CACHE] == g["C_cache"]
    assert list(co.C_SPARSE) == [0.0] + g["C_sparse"]         # action 0 is dense: no reduction
    # the product side: defaults of the reward entry point's binding
    import inspect
    import paper_2509_22323_amd.binding as binding
    sig = inspect.signature(binding.rapid_reward)
    assert [sig.parameters["lam"].default] == g["lambda"] and [sig.parameters["omega"].default] == g["omega"]
    # a step that reuses the cache costs 1 - C_cache; with the printed values 28 plain steps weigh
    # as much as 560 cached ones
    k, _ = co.equivalent_steps(*co.step_costs([1] * 560, [0] * 560))
    assert abs(k - 28.0) < 1e-9


def test_reward_is_the_geometric_series():
    q, d = 0.8, 0.3
    for K in (1, 2, 8, 16, 28):
        closed = (q + 1.0 * d) * (1 - 0.97 ** K) / (K * (1 - 0.97))
        assert abs(co.reward(q, d, K) - closed) < 1e-12
    assert co.reward(q, d, 1) == q + d
    assert all(co.reward(q, d, K + 1) < co.reward(q, d, K) for K in range(1, 40))   # cost is penalised
    assert abs(co.reward(q, d, 5, lam=0.5, omega=2.0) - (q + 2 * d) * (1 + .5 + .25 + .125 + .0625) / 5) < 1e-15


# ---------------------------------------------------------------- the pins can fail
MUTANTS = [
    ("ties_half_up", "np.rint(", "np.floor(0.5 + "),
    ("no_subnormals", "np.maximum(e - 8, -133)", "(e - 8)"),
    ("seven_bits", "np.maximum(e - 8, -133)", "np.maximum(e - 7, -133)"),
    ("delta_sign", "bf16_to_f64(o_bits) - bf16_to_f64(x_bits)", "bf16_to_f64(x_bits) - bf16_to_f64(o_bits)"),
    ("reuse_subtracts", "bf16_to_f64(x_bits) + bf16_to_f64(delta_bits)", "bf16_to_f64(x_bits) - bf16_to_f64(delta_bits)"),
    ("costs_add", "k += (1.0 - a) * (1.0 - b)", "k += (1.0 - a) + (1.0 - b) - 1.0"),
    ("round_to_even", "int(np.floor(k + 0.5))", "int(np.rint(k))"),
    ("sparse_active_when_cached", "cs.append(0.0 if ac else C_SPARSE[asp])", "cs.append(C_SPARSE[asp])"),
    ("decay_reversed", "lam ** (K - k)", "lam ** (-(K - k))"),
    ("no_mean", "return s / K", "return s"),
]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(monkeypatch, name, find, repl):
    import inspect
    import types
    src = inspect.getsource(co)
    assert src.count(find) >= 1
    mod = types.ModuleType("cache_oracle_mutant")
    exec(compile(src.replace(find, repl), "cache_oracle_mutant", "exec"), mod.__dict__)
    caught = 0
    for test in (test_rounding_hand_cases, test_rounding_against_brute_force_and_an_independent_implementation,
                 test_store_and_reuse_exact_cases, test_equivalent_steps_worked_examples,
                 test_reward_is_the_geometric_series):
        monkeypatch.setitem(globals(), "co", mod)
        try:
            test()
        except AssertionError:
            caught += 1
        finally:
            monkeypatch.setitem(globals(), "co", co)
    assert caught, f"mutant {name} survived every pin"
    assert re.sub(r"\s", "", src) != re.sub(r"\s", "", src.replace(find, repl))
