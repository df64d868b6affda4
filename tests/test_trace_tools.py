"""The stack-distance trace profiler and generator of Sec. 4.2 (Alg. 1 and Alg. 2), used as a seeded
input generator.  Pinned by what the section and the definitions fix: a hand-worked trace, the
special cases (all-distinct ids, a cyclic trace, immediate re-use), the round trip the section is
about (a generated trace's own profile reproduces p), and the two implementations (plain lists /
Fenwick tree in C) agreeing exactly when driven by the same random numbers."""
import numpy as np
import pytest

from workloads import gen, trace


def test_profile_of_a_hand_worked_trace():
    # ids:      a  b  a  a  c  b        stack (top first) before the access
    # distance: 0  0  2  1  0  3        [] [a] [b,a] [a,b] [a,b] [c,a,b]
    tr = [7, 9, 7, 7, 4, 9]
    for u, p in (trace.profile_trace_py(tr), trace.profile_trace(np.array(tr))):
        assert list(u) == [7, 9, 4]
        assert np.allclose(p, [3 / 6, 1 / 6, 1 / 6, 1 / 6])


def test_all_distinct_ids_have_only_the_infinite_distance():
    tr = np.random.default_rng(0).permutation(500)
    u, p = trace.profile_trace(tr)
    assert np.array_equal(u, tr) and p.shape == (1,) and p[0] == 1.0


def test_cyclic_trace_reuses_at_the_number_of_ids():
    m, reps = 37, 6
    tr = np.tile(np.arange(m), reps)
    u, p = trace.profile_trace(tr)
    assert np.array_equal(u, np.arange(m))
    want = np.zeros(m + 1)
    want[0], want[m] = m / tr.size, (tr.size - m) / tr.size
    assert np.allclose(p, want)


def test_profile_counts_sum_to_one_and_c_agrees_with_the_list_version():
    rng = np.random.default_rng(3)
    for m, n in ((5, 200), (50, 400), (300, 700), (1, 9)):
        tr = rng.integers(0, m, size=n)
        u1, p1 = trace.profile_trace_py(tr.tolist())
        u2, p2 = trace.profile_trace(tr, m)
        assert list(u2) == u1 and np.array_equal(p1, p2)
        assert abs(p2.sum() - 1.0) < 1e-12
        assert len(u2) == len(np.unique(tr)) and abs(p2[0] * n - len(u2)) < 1e-9


def test_generator_special_cases():
    u = [11, 22, 33, 44]
    # only first-time accesses: the ids come out in order
    assert trace.generate_trace_py(u, np.array([1.0]), [0.3, 0.9, 0.1, 0.5]) == u
    assert list(trace.generate_trace(np.array(u), np.array([1.0]), np.array([0.3, 0.9, 0.1, 0.5]))) == u
    # one first-time access, then always the id used just before
    p = np.array([0.01, 0.99])
    r = np.array([0.0] + [0.5] * 7)
    assert trace.generate_trace_py(u, p, r) == [11] * 8
    assert list(trace.generate_trace(np.array(u), p, r)) == [11] * 8
    # distance 2 alternates between the two most recent ids once two exist
    p = np.array([0.5, 0.0, 0.5])
    r = np.array([0.0, 0.0] + [0.99] * 6)       # two new ids, then always distance 2
    assert list(trace.generate_trace(np.array(u), p, r)) == [11, 22, 11, 22, 11, 22, 11, 22]
    # once every id has been seen, distance 0 leaves the support
    out = trace.generate_trace(np.array([5, 6]), np.array([0.9, 0.1]), np.array([0.0, 0.0, 0.0, 0.0]))
    assert list(out[:2]) == [5, 6] and set(out[2:]) <= {5, 6}


def test_c_generator_equals_the_list_version_on_the_same_random_numbers():
    rng = np.random.default_rng(5)
    for m, n0, n in ((8, 300, 500), (60, 2000, 1500), (400, 3000, 2500)):
        orig = (rng.zipf(1.3, size=n0) - 1) % m
        u, p = trace.profile_trace(orig, m)
        r = rng.random(n)
        for min_new in (0.0, 0.05):
            a = trace.generate_trace_py(u.tolist(), p, r.tolist(), min_new)
            b = trace.generate_trace(u, p, r, min_new)
            assert a == list(b)


def test_round_trip_reproduces_the_distance_distribution():
    """The property Sec. 4.2 is about: the profile of a trace generated from (u, p) is p again.  With few
    unique ids in a long trace p[0] is small, the generator needs most of the trace to meet every id, and
    until then it can only draw the distances that exist yet: the section's remedy (first-time accesses
    get a minimum probability while unseen ids remain) shortens that phase, and the distributions then
    lie on each other."""
    rng = np.random.default_rng(7)
    m, n = 5000, 400_000
    cdf = np.cumsum(np.arange(1, m + 1, dtype=np.float64) ** -1.1)
    orig = np.searchsorted(cdf / cdf[-1], rng.random(n))
    u, p = trace.profile_trace(orig, m)
    dist = {}
    for min_new in (0.0, 0.25):
        synth = trace.generate_trace(u, p, rng.random(n), min_new)
        u2, p2 = trace.profile_trace(synth, m)
        assert np.array_equal(u2, u[:len(u2)])          # new ids are taken from the front of u, in order
        k = max(len(p), len(p2))
        c1 = np.cumsum(np.pad(p, (0, k - len(p))))
        c2 = np.cumsum(np.pad(p2, (0, k - len(p2))))
        dist[min_new] = np.abs(c1 - c2).max()           # distance of the two cumulative distributions
        if min_new > 0:
            for depth in (1, 8, 64, 512):               # same share of short re-use distances (what a cache sees)
                assert abs(p[1:depth + 1].sum() - p2[1:depth + 1].sum()) < 0.01
    assert dist[0.25] < 0.01 and dist[0.25] < dist[0.0]


def test_locality_workload_batches_are_valid_and_seeded():
    w = gen.locality_workload(3, 1.05)
    import dataclasses
    w = dataclasses.replace(w, K=2, B=64, rows=("fixed", 20000))
    a, b = gen.make_batch(w), gen.make_batch(w)
    assert np.array_equal(a.indices, b.indices)
    assert a.indices.min() >= 0 and a.indices.max() < 20000
    assert len(a.indices) == a.nnz
    # more skew in the original trace -> more re-use in the generated one
    hi = gen.make_batch(dataclasses.replace(w, dist=("trace", 1.4)))
    assert len(np.unique(hi.indices_of(0))) < len(np.unique(a.indices_of(0)))
