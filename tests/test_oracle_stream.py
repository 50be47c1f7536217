"""Pins for the oracle's decode-step form (Sec. III-A/B: estimator and chunker run while decoding;
Sec. III-F: scheduler state kept between steps) and for the layer on rows that bring their own gate.

The step function is tied to the batch chunker and selector, which have their own pins (brute force,
hand-worked fixtures): fed token by token it must place the same boundaries wherever the end of the
sequence cannot matter, end every chunk on the rung the batch selector gives that chunk, and on
scores that are constant inside every chunk reproduce the batch layer's output token for token.  The
gated layer is pinned by a float64 library matmul of the textbook formula."""
import numpy as np
import pytest

INF_Q = 1 << 21


def run_stream(oracle, q, l_min, l_max, theta, delta, taus, ranks, scales, w):
    """Feed one sequence token by token.  Returns closed chunks [(start, len, sum)], per-token gates
    and the rung in force at every token."""
    st = oracle.StreamState(1)
    chunks, gates, rungs = [], [], []
    for t, qt in enumerate(q):
        code, out = oracle.stream_step(st, [qt], l_min, l_max, theta, delta, taus, ranks, scales, w)
        assert code == 0
        if out["closed_len"][0]:
            n = int(out["closed_len"][0])
            chunks.append((t - n, n, int(out["closed_sum"][0])))
        gates.append((int(out["r_cur"][0]), float(out["g_cur"][0]), int(out["r_prev"][0]), float(out["g_prev"][0])))
        rungs.append(int(st.k_cur[0]))
        assert st.pos[0] == t + 1
    return chunks, gates, rungs, st


LADDER = ([4, 8, 16], [4.0, 2.0, 1.0])
TAUS = [3000, 6000]


@pytest.mark.parametrize("seed", range(6))
def test_boundaries_match_the_batch_chunker_away_from_the_end(oracle, seed):
    rng = np.random.RandomState(seed)
    l_min, l_max = [(4, 9), (8, 64), (3, 5), (16, 40), (1, 1), (5, 30)][seed]
    T = 700
    # spans of three difficulty levels with noise, as in the workloads
    q = np.concatenate([rng.choice([1500, 5000, 9000]) + rng.randint(-400, 400, size=rng.randint(5, 60))
                        for _ in range(60)])[:T].astype(np.int32)
    theta, delta = 8000, 2500
    code, tab = oracle.partition(q, [0, T], l_min, l_max, theta, delta)
    assert code == 0
    batch = list(zip(tab["chunk_start"].tolist(), tab["chunk_len"].tolist(), tab["chunk_sum"].tolist()))
    chunks, _, rungs, _ = run_stream(oracle, q, l_min, l_max, theta, delta, TAUS, *LADDER, 2)
    safe = [c for c in batch if c[0] + l_max <= T - l_min]
    assert len(safe) > 5
    assert chunks[:len(safe)] == safe
    # the rung in force at the last token of a chunk is the batch selector's rung for that chunk
    want = oracle.select([c[2] for c in safe], [c[1] for c in safe], TAUS)
    got = [rungs[s + n - 1] for s, n, _ in safe]
    assert got == want.tolist()


def test_all_easy_and_all_hard_limits(oracle):
    # nothing fires: every chunk runs to L_max; everything hard: every chunk is L_min long
    for q0, want_len in ((100, 12), (9000, 4)):
        q = np.full(100, q0, np.int32)
        chunks, _, _, st = run_stream(oracle, q, 4, 12, 8000, INF_Q, TAUS, *LADDER, 0)
        assert all(n == want_len for _, n, _ in chunks)
        assert len(chunks) == (100 - 1) // want_len          # the open chunk is not reported
        assert st.n[0] == 100 - len(chunks) * want_len and st.chunks[0] == len(chunks)


def test_sequences_are_independent_and_state_is_all_there_is(oracle):
    rng = np.random.RandomState(3)
    q = rng.randint(0, 10000, size=(5, 300)).astype(np.int32)
    args = (6, 20, 8000, 2500, TAUS, *LADDER, 3)
    # batch of 5 sequences step by step == each sequence alone
    st = oracle.StreamState(5)
    rec = []
    for t in range(300):
        code, out = oracle.stream_step(st, q[:, t], *args)
        assert code == 0
        rec.append({k: v.copy() for k, v in out.items()})
    for b in range(5):
        _, gates, _, st1 = run_stream(oracle, q[b], *args)
        for t in range(300):
            assert gates[t] == (rec[t]["r_cur"][b], rec[t]["g_cur"][b], rec[t]["r_prev"][b], rec[t]["g_prev"][b])
        assert (st1.n[0], st1.sum[0], st1.k_cur[0], st1.k_prev[0], st1.chunks[0]) == \
               (st.n[b], st.sum[b], st.k_cur[b], st.k_prev[b], st.chunks[b])


def test_cross_fade_weights_hand_worked(oracle):
    # L_min = 3, L_max = 5, w = 2, scores 1000 x3 then 7000 x3; the jump fires the deviation test when
    # token 3 arrives (|7000 - 1000| > 500).  Rungs 0 then 2 of ladder r = (4, 8, 16), s = (4, 2, 1).
    # Tokens 3 and 4 open the second chunk: lambda = 1/3, 2/3.
    q = [1000, 1000, 1000, 7000, 7000, 7000]
    chunks, gates, rungs, _ = run_stream(oracle, q, 3, 5, INF_Q, 500, TAUS, *LADDER, 2)
    assert chunks == [(0, 3, 3000)]
    assert rungs == [0, 0, 0, 2, 2, 2]
    assert gates[0] == gates[1] == gates[2] == (4, 4.0, 0, 0.0)
    r_cur, g_cur, r_prev, g_prev = gates[3]
    assert (r_cur, r_prev) == (16, 4) and g_cur == pytest.approx(1.0 / 3) and g_prev == pytest.approx(4.0 * 2 / 3)
    r_cur, g_cur, r_prev, g_prev = gates[4]
    assert (r_cur, r_prev) == (16, 4) and g_cur == pytest.approx(2.0 / 3) and g_prev == pytest.approx(4.0 / 3)
    assert gates[5] == (16, 1.0, 0, 0.0)


def test_piecewise_constant_scores_reproduce_the_batch_layer(oracle):
    """When the score is constant inside every chunk the running mean equals the chunk mean, so the
    step form picks the batch form's rung at every token and the two layers agree row for row."""
    rng = np.random.RandomState(11)
    l_min, l_max, w = 4, 10, 3
    levels = [1000, 4000, 7000]
    q = np.concatenate([np.full(rng.randint(l_min, l_max + 1), levels[i % 3], np.int32) for i in range(14)])
    T = len(q)
    theta, delta = INF_Q, 500                       # a change of level fires the deviation test at once
    ranks, scales = [2, 5, 7], [3.0, 1.5, 0.5]
    code, tab = oracle.partition(q, [0, T], l_min, l_max, theta, delta)
    ri = oracle.select(tab["chunk_sum"], tab["chunk_len"], TAUS)
    _, gates, _, _ = run_stream(oracle, q, l_min, l_max, theta, delta, TAUS, ranks, scales, w)
    d_in, d_out, r_max = 12, 9, 7
    x = rng.randn(T, d_in).astype(np.float32)
    Wm, A, Bm = (rng.randn(*s).astype(np.float32) for s in ((d_in, d_out), (d_in, r_max), (r_max, d_out)))
    y_batch = oracle.linear(x, Wm, A, Bm, ranks, scales, w, [0, T], tab["chunk_offsets"], tab["chunk_start"],
                            tab["chunk_len"], ri)
    g = np.array(gates, dtype=np.float64)
    y_step = oracle.gated_linear(x, Wm, A, Bm, g[:, 0], g[:, 1], g[:, 2], g[:, 3])
    safe = T - l_min - l_max                        # rows the end of the sequence cannot touch
    assert safe > 40
    np.testing.assert_allclose(y_step[:safe], y_batch[:safe], rtol=1e-12, atol=1e-12)


def test_gated_linear_is_the_textbook_formula(oracle):
    rng = np.random.RandomState(5)
    n, d_in, d_out, r_max = 17, 20, 13, 6
    x = rng.randn(n, d_in).astype(np.float32)
    Wm, A, Bm = (rng.randn(*s).astype(np.float32) for s in ((d_in, d_out), (d_in, r_max), (r_max, d_out)))
    r_cur = rng.randint(0, r_max + 1, n)
    r_prev = rng.randint(0, r_max + 1, n)
    g_cur, g_prev = rng.rand(n), rng.rand(n)
    y = oracle.gated_linear(x, Wm, A, Bm, r_cur, g_cur, r_prev, g_prev)
    xd, Wd, Ad, Bd = (a.astype(np.float64) for a in (x, Wm, A, Bm))
    for t in range(n):
        want = xd[t] @ Wd + g_cur[t] * (xd[t] @ Ad[:, :r_cur[t]]) @ Bd[:r_cur[t]] \
            + g_prev[t] * (xd[t] @ Ad[:, :r_prev[t]]) @ Bd[:r_prev[t]]
        np.testing.assert_allclose(y[t], want, rtol=1e-12, atol=1e-12)
    with pytest.raises(ValueError):
        oracle.gated_linear(x, Wm, A, Bm, r_cur + r_max + 1, g_cur, r_prev, g_prev)


def test_argument_errors(oracle):
    st = oracle.StreamState(1)
    assert oracle.stream_step(st, [5], 4, 6, 1, 1, TAUS, *LADDER, 0)[0] == oracle.reference.ERR_INFEASIBLE
    assert oracle.stream_step(st, [5], 0, 6, 1, 1, TAUS, *LADDER, 0)[0] == oracle.reference.ERR_INVALID
    assert st.pos[0] == 0
