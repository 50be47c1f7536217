"""Pins for the oracle's composite score (Sec. III-A: n-gram novelty against the recent context and a
positional prior next to the entropy): an independent restatement with sets of tuples, sequences
with known answers, and the weights taken one at a time."""
import numpy as np
import pytest


def restated_novelty(ids, n, window):
    """Positions whose n-gram is in the set of n-grams ending within the `window` positions before."""
    out = []
    for j in range(len(ids)):
        if j < n - 1:
            out.append(1)
            continue
        recent = {tuple(ids[jp - n + 1:jp + 1]) for jp in range(max(n - 1, j - window), j)}
        out.append(0 if tuple(ids[j - n + 1:j + 1]) in recent else 1)
    return out


@pytest.mark.parametrize("n,window,vocab", [(1, 5, 4), (2, 7, 3), (3, 50, 2), (4, 3, 2), (2, 0, 3), (3, 1000, 5)])
def test_novelty_against_set_restatement(oracle, n, window, vocab):
    rng = np.random.RandomState(n * 100 + window)
    lens = [0, 1, 2, 37, 200]
    ids = rng.randint(0, vocab, size=sum(lens)).astype(np.int32)
    so = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    st, _, nov = oracle.compose_scores(np.zeros(len(ids), np.float32), ids, so, n, window, 1.0, 1.0, 0.0, 0.0)
    assert st == 0
    want = []
    for b in range(len(lens)):
        want += restated_novelty(ids[so[b]:so[b + 1]].tolist(), n, window)
    assert nov.tolist() == want


def test_known_sequences(oracle):
    z = np.zeros(12, np.float32)
    # all tokens distinct: everything is new; one repeated token: only the first n positions are new
    _, _, nov = oracle.compose_scores(z, np.arange(12), [0, 12], 3, 100, 0, 1, 0, 0)
    assert nov.tolist() == [1] * 12
    _, _, nov = oracle.compose_scores(z, np.full(12, 7), [0, 12], 3, 100, 0, 1, 0, 0)
    assert nov.tolist() == [1, 1, 1] + [0] * 9
    # period 4, bigrams: after one period plus one token every bigram has been seen ... within the window only
    ids = np.tile([1, 2, 3, 4], 3)
    _, _, nov = oracle.compose_scores(z, ids, [0, 12], 2, 100, 0, 1, 0, 0)
    assert nov.tolist() == [1, 1, 1, 1, 1] + [0] * 7
    _, _, nov = oracle.compose_scores(z, ids, [0, 12], 2, 3, 0, 1, 0, 0)       # window shorter than the period
    assert nov.tolist() == [1] * 12
    # the window does not reach across a sequence start
    _, _, nov = oracle.compose_scores(z, np.full(12, 7), [0, 6, 12], 1, 100, 0, 1, 0, 0)
    assert nov.tolist() == [1, 0, 0, 0, 0, 0] * 2


def test_weights_one_at_a_time_and_prior_ramp(oracle):
    rng = np.random.RandomState(2)
    h = rng.rand(10).astype(np.float32) * 5
    ids = rng.randint(0, 3, 10)
    _, s, _ = oracle.compose_scores(h, ids, [0, 10], 2, 4, 2.5, 0, 0, 8)
    np.testing.assert_allclose(s, 2.5 * h.astype(np.float64), rtol=1e-15)
    _, s, nov = oracle.compose_scores(h, ids, [0, 10], 2, 4, 0, 3.0, 0, 8)
    np.testing.assert_allclose(s, 3.0 * nov, rtol=1e-15)
    _, s, _ = oracle.compose_scores(h, ids, [0, 4, 10], 2, 4, 0, 0, 4.0, 8)    # restarts with every sequence
    np.testing.assert_allclose(s, 4.0 * np.array([1, 7 / 8, 6 / 8, 5 / 8, 1, 7 / 8, 6 / 8, 5 / 8, 4 / 8, 3 / 8]), rtol=1e-15)
    _, s, _ = oracle.compose_scores(h, ids, [0, 10], 2, 4, 0, 0, 4.0, 3)      # clipped at 0 from position 3 on
    np.testing.assert_allclose(s, 4.0 * np.array([1, 2 / 3, 1 / 3] + [0] * 7), rtol=1e-15, atol=1e-15)
    _, s, _ = oracle.compose_scores(h, ids, [0, 10], 2, 4, 0, 0, 4.0, 0)      # no prior
    assert not s.any()
    # rows outside every sequence keep the entropy term only
    _, s, nov = oracle.compose_scores(h, ids, [2, 6], 1, 4, 1.0, 10.0, 10.0, 5)
    np.testing.assert_allclose(s[[0, 1, 6, 7, 8, 9]], h[[0, 1, 6, 7, 8, 9]].astype(np.float64))
    assert nov[[0, 1, 6, 7, 8, 9]].tolist() == [0] * 6
    assert oracle.compose_scores(h, ids, [0, 10], 0, 4, 1, 1, 1, 1)[0] == oracle.reference.ERR_INVALID
