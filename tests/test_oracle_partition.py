"""Pins for the oracle's chunker and rung selector (Sec. III-B/C, IV-B/C): invariants,
limit cases with known answers, hand-worked examples, and a brute-force comparison with an
independent restatement of the rule in rational arithmetic."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from conftest import read_golden

INF_Q = 1 << 21


def chunks_of(res):
    return list(zip(res["chunk_start"].tolist(), res["chunk_len"].tolist(),
                    res["chunk_sum"].tolist()))


def restated_partition(q, l_min, l_max, theta, delta):
    """Independent restatement: enumerate the admissible ends of the open chunk as a set and
    take the smallest one at which a test fires, in exact rational means."""
    T = len(q)
    if T == 0:
        return []
    if T < l_min:
        return [(0, T, sum(q))]

    def rec(p):
        if p == T:
            return []
        ends = [e for e in range(p + l_min, min(p + l_max, T) + 1)
                if T - e == 0 or T - e >= l_min]
        chosen = ends[-1]
        for e in ends:
            if e == T:
                chosen = e
                break
            n = e - p
            mean = Fraction(sum(q[p:e]), n)
            if mean >= theta or q[e] >= theta or abs(q[e] - mean) > delta:
                chosen = e
                break
        return [(p, chosen - p, sum(q[p:chosen]))] + rec(chosen)

    return rec(0)


def test_golden_w1(oracle):
    g = read_golden("partition_w1.txt")
    st_, res = oracle.partition(g["q"], [0, len(g["q"])], g["l_min"][0], g["l_max"][0],
                                g["theta_q"][0], g["delta_q"][0])
    assert st_ == 0
    assert res["chunk_start"].tolist() == g["chunk_start"]
    assert res["chunk_len"].tolist() == g["chunk_len"]
    assert res["chunk_sum"].tolist() == g["chunk_sum"]
    assert res["chunk_offsets"].tolist() == [0, 4]
    ri = oracle.select(res["chunk_sum"], res["chunk_len"], g["tau_q"])
    assert ri.tolist() == g["rank_idx"]
    assert [[4, 8, 16][k] for k in ri] == g["ranks"]


def test_golden_w1b(oracle):
    g = read_golden("partition_w1b.txt")
    st_, res = oracle.partition(g["q"], [0, len(g["q"])], g["l_min"][0], g["l_max"][0],
                                g["theta_q"][0], g["delta_q"][0])
    assert st_ == 0
    assert res["chunk_start"].tolist() == g["chunk_start"]
    assert res["chunk_len"].tolist() == g["chunk_len"]
    assert res["chunk_sum"].tolist() == g["chunk_sum"]


@pytest.mark.parametrize("T,want", [(23, [8, 8, 7]), (18, [8, 6, 4]), (8, [8]), (9, [5, 4]),
                                    (3, [3]), (4, [4]), (12, [8, 4]), (11, [7, 4])])
def test_tests_disabled_gives_max_length_chunks(oracle, T, want):
    q = np.arange(T) % 5
    st_, res = oracle.partition(q, [0, T], 4, 8, INF_Q, INF_Q)
    assert st_ == 0
    assert res["chunk_len"].tolist() == want
    assert sum(want) == T


def test_all_hard_gives_min_length_chunks(oracle):
    for T in (16, 19, 23, 40):
        q = np.full(T, 50)
        st_, res = oracle.partition(q, [0, T], 4, 8, 10, INF_Q)
        lens = res["chunk_len"].tolist()
        assert sum(lens) == T
        assert all(n == 4 for n in lens[:-1])
        assert 4 <= lens[-1] <= 7


def test_easy_long_hard_short(oracle):
    q = np.concatenate([np.full(64, 2), np.full(64, 40), np.full(64, 2)])
    st_, res = oracle.partition(q, [0, 192], 4, 32, 30, 10)
    c = chunks_of(res)
    easy = [n for (s, n, _) in c if s + n <= 64 or s >= 128]
    hard = [n for (s, n, _) in c if s >= 64 and s + n <= 128]
    assert max(hard) <= 4 and min(easy) >= 16


def test_brute_force_small(oracle):
    # every q in {0,1,2}^T for T <= 9, plus random longer ones, against the restatement
    cases = [(2, 3, 2, 1), (2, 4, 1, 0), (3, 5, 2, 1), (1, 2, 1, 1), (2, 3, 1 << 21, 1 << 21)]
    for l_min, l_max, th, de in cases:
        for T in range(0, 10):
            for q in itertools.product((0, 1, 2), repeat=T):
                st_, res = oracle.partition(list(q), [0, T], l_min, l_max, th, de)
                assert st_ == 0
                assert chunks_of(res) == restated_partition(list(q), l_min, l_max, th, de)


def test_brute_force_random_longer(oracle):
    rng = np.random.RandomState(5)
    for _ in range(300):
        T = int(rng.randint(1, 60))
        l_min = int(rng.randint(1, 6))
        l_max = int(rng.randint(2 * l_min - 1, 2 * l_min + 9))
        l_max = max(l_max, l_min)
        q = rng.randint(0, 30, size=T).tolist()
        th, de = int(rng.randint(5, 30)), int(rng.randint(1, 15))
        st_, res = oracle.partition(q, [0, T], l_min, l_max, th, de)
        assert st_ == 0
        assert chunks_of(res) == restated_partition(q, l_min, l_max, th, de)


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(0, 12000), min_size=0, max_size=300), st.integers(1, 12),
       st.integers(0, 30), st.integers(0, 12000), st.integers(0, 12000))
def test_invariants_cover_and_bounds(q, l_min, extra, th, de):
    import oracle
    l_max = 2 * l_min - 1 + extra
    T = len(q)
    st_, res = oracle.partition(q, [0, T], l_min, l_max, th, de)
    assert st_ == 0
    starts, lens, sums = res["chunk_start"], res["chunk_len"], res["chunk_sum"]
    assert int(lens.sum()) == T
    pos = 0
    for s, n, sm in zip(starts, lens, sums):
        assert s == pos and n >= 1
        assert sm == sum(q[s:s + n])
        pos += n
    if T >= l_min:
        assert all(l_min <= n <= l_max for n in lens)
    elif T > 0:
        assert lens.tolist() == [T]
    # determinism
    st2, res2 = oracle.partition(q, [0, T], l_min, l_max, th, de)
    assert chunks_of(res) == chunks_of(res2)


def test_batch_independence(oracle):
    rng = np.random.RandomState(9)
    lens = [0, 37, 5, 128, 2, 64]
    qs = [rng.randint(0, 9000, size=n) for n in lens]
    so = np.concatenate([[0], np.cumsum(lens)])
    st_, res = oracle.partition(np.concatenate(qs), so, 4, 16, 6000, 2500)
    assert st_ == 0
    co = res["chunk_offsets"]
    for b, qb in enumerate(qs):
        _, rb = oracle.partition(qb, [0, len(qb)], 4, 16, 6000, 2500)
        sl = slice(co[b], co[b + 1])
        assert (res["chunk_start"][sl] - so[b]).tolist() == rb["chunk_start"].tolist()
        assert res["chunk_len"][sl].tolist() == rb["chunk_len"].tolist()
        assert res["chunk_sum"][sl].tolist() == rb["chunk_sum"].tolist()
    assert co[1] == 0 and co[-1] == len(res["chunk_len"])


def test_argument_errors_and_capacity(oracle):
    q = np.ones(40, dtype=np.int32)
    assert oracle.partition(q, [0, 40], 0, 4, 1, 1)[0] == oracle.reference.ERR_INVALID
    assert oracle.partition(q, [0, 40], 5, 4, 1, 1)[0] == oracle.reference.ERR_INVALID
    assert oracle.partition(q, [0, 40], 4, 6, 1, 1)[0] == oracle.reference.ERR_INFEASIBLE
    st_, res = oracle.partition(q, [0, 40], 4, 8, 0, INF_Q, cap=3)
    assert st_ == oracle.reference.ERR_CAPACITY
    assert res["chunk_offsets"][-1] == 10 and len(res["chunk_len"]) == 3


def test_select_properties(oracle):
    tau = [300, 600, 900]
    lens = np.array([10, 10, 10, 10, 7, 1], dtype=np.int32)
    sums = np.array([2999, 3000, 6000, 9000 - 1, 7 * 900, 0], dtype=np.int64)
    assert oracle.select(sums, lens, tau).tolist() == [0, 1, 2, 2, 3, 0]
    # K = 1: always rung 0
    assert oracle.select(sums, lens, []).tolist() == [0] * 6
    # monotone in the mean
    rng = np.random.RandomState(3)
    n = rng.randint(1, 50, size=200).astype(np.int32)
    s = (rng.randint(0, 1200, size=200) * n).astype(np.int64)
    k = oracle.select(s, n, tau)
    order = np.argsort(s / n, kind="stable")
    assert np.all(np.diff(k[order]) >= 0)
    want = [int(m >= 300) + int(m >= 600) + int(m >= 900) for m in (s // n)]
    assert k.tolist() == want
