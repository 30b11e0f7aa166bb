"""Pins of the oracle's sampling budget (Section 3.7): what the rule must satisfy whatever the
generator -- sizes, membership, uniformity of the kept subset and of the fill, determinism, the
generator being a bijection (so priorities never tie) -- and brute force on small cases."""
import numpy as np

from oracle import slide_oracle as so


def test_mix_is_a_bijection_on_a_window_and_mixes():
    x = np.arange(1 << 16, dtype=np.uint64)
    y = so.sample_mix(x)
    assert np.unique(y).size == x.size and y.max() <= 0xFFFFFFFF
    assert int(so.sample_mix(np.uint64(0))) == 0                 # the finaliser fixes zero
    bits = np.unpackbits(y.astype(">u4").view(np.uint8)).reshape(-1, 32).mean(0)
    assert np.all(np.abs(bits - 0.5) < 0.02)                     # every output bit is balanced
    flip = so.sample_mix(x ^ np.uint64(1)) ^ y                   # one input bit flips about half of the output bits
    assert abs(np.unpackbits(flip.astype(">u4").view(np.uint8)).mean() - 0.5) < 0.01


def test_over_budget_keeps_exactly_budget_candidates_uniformly():
    N, budget = 5000, 10
    cand = np.arange(100, 160)                                    # 60 candidates, 3 of them labels
    labels = np.array([100, 130, 4000])
    counts = np.zeros(N)
    trials = 3000
    for s in range(trials):
        kept = so.apply_budget(cand, labels, N, budget, False, seed=7, step=1 + s, sample=s % 5)
        assert kept.size == budget and np.all(np.diff(kept) > 0)
        assert np.all(np.isin(kept, cand)) and not np.any(np.isin(kept, labels))
        counts[kept] += 1
    pool = np.setdiff1d(cand, labels)
    p = counts[pool] / trials                                     # each of the 58 kept with probability 10/58
    assert abs(p.mean() - budget / pool.size) < 1e-9
    sd = np.sqrt(p.mean() * (1 - p.mean()) / trials)
    assert np.all(np.abs(p - p.mean()) < 5 * sd)
    # brute force: the kept ones are those of smallest priority
    base = so.sample_base(7, 1, 0)
    pr = so.sample_prio(base, pool)
    assert np.array_equal(so.apply_budget(cand, labels, N, budget, False, 7, 1, 0), np.sort(pool[np.argsort(pr)[:budget]]))
    assert np.unique(pr).size == pr.size


def test_under_budget_fill_and_stop_options():
    N, budget = 300, 40
    cand = np.array([5, 9, 77, 200])
    labels = np.array([9, 250])
    assert np.array_equal(so.apply_budget(cand, labels, N, budget, False, 3, 2, 1), np.array([5, 77, 200]))
    hist = np.zeros(N)
    for s in range(2000):
        got = so.apply_budget(cand, labels, N, budget, True, 3, 2 + s, 1)
        assert got.size == budget and np.all(np.diff(got) > 0) and got.min() >= 0 and got.max() < N
        assert np.all(np.isin([5, 77, 200], got)) and not np.any(np.isin(labels, got))
        hist[got] += 1
    free = np.setdiff1d(np.arange(N), np.concatenate([cand, labels]))
    p = hist[free] / 2000                                         # the 37 filled ones are uniform over the rest
    assert np.all(np.abs(p - 37 / free.size) < 5 * np.sqrt(p.mean() * (1 - p.mean()) / 2000))
    # sequential definition, brute force
    base = so.sample_base(3, 2, 1)
    present, need, d = set([5, 77, 200, 9, 250]), budget - 3, 0
    while need:
        j = int(so.sample_draw(base, d, N)); d += 1
        if j not in present:
            present.add(j); need -= 1
    assert np.array_equal(so.apply_budget(cand, labels, N, budget, True, 3, 2, 1),
                          np.array(sorted(present - {9, 250})))
    # a budget that cannot be met stops after 4*budget + 64 draws
    tiny = so.apply_budget(np.arange(3), np.array([], dtype=np.int64), 5, 50, True, 1, 1, 0)
    assert np.array_equal(tiny, np.arange(5))
    d = so.sample_draw(so.sample_base(1, 1, 0), np.arange(100000), 1000)
    assert d.min() == 0 and d.max() == 999 and abs(np.bincount(d).std() - 10) < 1.5


def test_same_inputs_same_sets_and_steps_differ():
    cand = np.arange(1000)
    a = so.apply_budget(cand, [], 5000, 50, False, 11, 4, 2)
    assert np.array_equal(a, so.apply_budget(cand, [], 5000, 50, False, 11, 4, 2))
    assert not np.array_equal(a, so.apply_budget(cand, [], 5000, 50, False, 11, 5, 2))
    assert not np.array_equal(a, so.apply_budget(cand, [], 5000, 50, False, 11, 4, 3))
    assert not np.array_equal(a, so.apply_budget(cand, [], 5000, 50, False, 12, 4, 2))
