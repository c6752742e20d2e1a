"""Wavefront sample scheduler (Sec. 3.4, Algorithm 1): pins of the oracle, then the host C++ against the oracle.
No GPU is needed: the scheduler is host code."""
import itertools
import os

import pytest

from oracle import scheduler as S
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scheduler_example_tuples.txt")


def paper_example():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    return [tuple(float(x) for x in r) for r in rows]


def random_samples(seed, n, p_text=0.4, post=False):
    """Seeded VLM-like mix: a text-only sample has no work in front of the critical section."""
    u = wl.uniform(seed, "sched", n * 6).reshape(n, 6).tolist()
    out = []
    for r in u:
        text = r[0] < p_text
        vit = 0.0 if text else 0.05 + 0.6 * r[1]
        llm = 0.5 + r[2]
        tail = 0.2 * r[3] if post else 0.0
        out.append((vit, llm, tail, 2.0 * tail, 2.0 * llm, 0.0 if text else 2.0 * vit))
    return out


# ---------------------------------------------------------------- the oracle against the paper and the mathematics
def test_paper_example_critical_section_never_waits():
    ex = paper_example()
    assert ex[0] == (0.1, 1.0, 0.0, 0.0, 2.0, 0.2) and len(ex) == 4
    for interleave in (True, False):
        given = S.simulate(ex, [0, 1, 2, 3], interleave)
        assert given["critical_idle"] == pytest.approx(0.1)            # the first sample's encoder forward is exposed
        order = S.schedule(ex, interleave)
        got = S.simulate(ex, order, interleave)
        # Sec. 3.4: under the algorithm's order the critical (LLM) section is never stalled by the ViT section
        assert got["critical_idle"] == pytest.approx(0.0, abs=1e-12)
        assert got["makespan"] == pytest.approx(sum(s[1] + s[4] for s in ex))   # = the critical section's own work
        assert ex[order[0]][0] == 0.0                                       # a text-only sample opens the schedule
        assert got["makespan"] == pytest.approx(S.brute_force_best(ex, interleave))


def test_closed_forms():
    one = [(0.3, 1.0, 0.2, 0.4, 2.0, 0.6)]
    for il in (True, False):
        assert S.makespan(one, [0], il) == pytest.approx(sum(one[0]))      # a single sample is a pure chain
        # only critical work: any order, the sum
        crit = [(0, 1.0, 0, 0, 2.0, 0), (0, 0.5, 0, 0, 1.0, 0), (0, 2.0, 0, 0, 0.1, 0)]
        for perm in itertools.permutations(range(3)):
            assert S.makespan(crit, list(perm), il) == pytest.approx(6.6)
    # two samples, sample by sample, worked by hand: PRE forwards end at 0.5 and 0.7; critical: 0.5..1.5 f, ..3.5 b,
    # 3.5..4.5 f, ..6.5 b; PRE backwards: 3.5..4.0 and 6.5..6.8
    two = [(0.5, 1.0, 0, 0, 2.0, 0.5), (0.2, 1.0, 0, 0, 2.0, 0.3)]
    r = S.simulate(two, [0, 1], True)
    assert r["makespan"] == pytest.approx(6.8) and r["critical_idle"] == pytest.approx(0.5)
    # all forwards then all backwards: critical f 0.5..1.5, 1.5..2.5, b 2.5..4.5, 4.5..6.5; PRE b 4.5..5.0, 6.5..6.8
    assert S.simulate(two, [0, 1], False)["makespan"] == pytest.approx(6.8)
    # work behind the critical section delays its backward: f 0..1, POST 1..1.6, b 1.6..3.6
    tail = [(0, 1.0, 0.2, 0.4, 2.0, 0)]
    assert S.makespan(tail, [0], True) == pytest.approx(3.6)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("interleave", [True, False])
def test_invariants_and_greedy_gap(seed, interleave):
    n = 4 + seed % 4
    sm = random_samples(seed, n, post=seed % 2 == 1)
    order = S.schedule(sm, interleave)
    assert sorted(order) == list(range(n))
    got = S.simulate(sm, order, interleave)
    lower = max(sum(s[1] + s[4] for s in sm), sum(s[0] + s[5] for s in sm), sum(s[2] + s[3] for s in sm))
    assert got["makespan"] >= lower - 1e-12
    assert got["critical_busy"] == pytest.approx(sum(s[1] + s[4] for s in sm))
    best = S.brute_force_best(sm, interleave)
    assert best - 1e-12 <= got["makespan"] <= 1.05 * best                    # greedy insertion stays near the optimum
    # a planted mistake must show: dropping the pre-critical backward changes the makespan of an encoder-last order
    enc_last = sorted(range(n), key=lambda i: sm[i][5])
    if sm[enc_last[-1]][5] > 0:
        no_bwd = [s[:5] + (0.0,) for s in sm]
        assert S.makespan(no_bwd, enc_last, interleave) < S.makespan(sm, enc_last, interleave)


# ---------------------------------------------------------------- the host C++ against the oracle
@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("interleave", [True, False])
def test_library_matches_oracle(seed, interleave):
    n = [1, 2, 3, 5, 8, 13, 24, 40][seed]
    sm = random_samples(100 + seed, n, post=seed % 3 == 0)
    order, mk = B.schedule_samples(sm, interleave)
    assert order == S.schedule(sm, interleave)                               # same decisions, ties included
    assert mk == pytest.approx(S.makespan(sm, order, interleave), rel=1e-12)
    for perm_seed in range(3):
        perm = wl.randint(seed * 10 + perm_seed, "perm", n, 0, 1 << 30, "cpu").argsort().tolist()
        m, idle = B.schedule_makespan(sm, perm, interleave)
        ref = S.simulate(sm, perm, interleave)
        assert m == pytest.approx(ref["makespan"], rel=1e-12)
        assert idle == pytest.approx(ref["critical_idle"], abs=1e-9)


def test_library_paper_example_and_errors():
    ex = paper_example()
    order, mk = B.schedule_samples(ex)
    assert mk == pytest.approx(12.0) and B.schedule_makespan(ex, order)[1] == pytest.approx(0.0, abs=1e-12)
    assert B.schedule_samples([]) == ([], 0.0)
    with pytest.raises(RuntimeError):
        B.schedule_makespan(ex, [0, 1, 1, 2])                                # not a permutation
    with pytest.raises(RuntimeError):
        B.schedule_samples([(0.1, -1.0, 0, 0, 2, 0)])                        # negative time
    with pytest.raises(RuntimeError):
        B.schedule_samples([(float("nan"), 1.0, 0, 0, 2, 0)])
