"""The scripted action traces (input generator; counts as in the paper's appendix on the
distribution of learned strategies) and the cost accounting of a trace."""
import paper_2509_22323_amd as ra
import workloads as wl
from oracle import cache_oracle as co


def test_traces_have_the_reported_statistics():
    for seed in range(200):
        t = wl.action_trace(seed)
        n_cached = sum(a for a, _ in t)
        n_sparse = sum(1 for a, s in t if s > 0)
        assert 12 <= len(t) <= 16 and 4 <= n_cached <= 8 and 2 <= n_sparse <= 4
        assert t[0][0] == 0                                    # nothing to reuse at the first step
        assert all(s == 0 for a, s in t if a == 1)             # sparse policy inactive on cached steps
        assert all(0 <= s <= 3 for _, s in t)
    assert wl.action_trace(5) == wl.action_trace(5) and wl.action_trace(5) != wl.action_trace(6)


def test_equivalent_steps_of_a_trace():
    t = wl.action_trace(3, n_steps=14, n_cached=6, n_sparse=3)
    cc, cs = co.step_costs([a for a, _ in t], [s for _, s in t])
    exact, k = ra.rapid_equivalent_steps(cc, cs)
    # 5 full steps, 6 cached at 0.05, 3 sparse between 0.90 and 0.95
    assert 5 + 6 * 0.05 + 3 * 0.90 <= exact <= 5 + 6 * 0.05 + 3 * 0.95
    assert k == co.equivalent_steps(cc, cs)[1] == 8
