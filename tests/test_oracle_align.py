"""Pins for the oracle's budget of high-capacity chunks (Sec. III-B), its percentile buckets and
micro-batches (Sec. III-G, IV-F) and its chunker with boundaries aligned inside a bucket
(Sec. III-G): hand-worked cases, reductions to the plain chunker, invariants, and independent
restatements with numpy's sort and Python integers."""
import numpy as np
import pytest

from test_oracle_partition import restated_partition

INF_Q = 1 << 21


def ragged(rng, n_seqs, t_lo, t_hi, levels=(300, 1500, 4000)):
    lens = rng.integers(t_lo, t_hi + 1, n_seqs)
    so = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q = np.empty(so[-1], np.int32)
    for s in range(n_seqs):
        # spans of one difficulty level each, like the workloads' score series
        t, T = 0, lens[s]
        while t < T:
            n = int(rng.integers(3, 40))
            lvl = levels[int(rng.integers(0, len(levels)))] * (0.5 + s / n_seqs)
            q[so[s] + t: so[s] + min(t + n, T)] = np.clip(rng.normal(lvl, 100, min(n, T - t)), 0, 1 << 20)
            t += n
    return q, so


# ---------------------------------------------------------------- budget of high-capacity chunks

def test_budget_hand_worked(oracle):
    # two sequences; rungs asked for, k_high = 2, budget 2: the third and later askers drop to rung 1
    ranks = [2, 0, 3, 1, 2, 3,   3, 1, 0]
    st, out, asked = oracle.limit_high(ranks, [0, 6, 9], 2, 2)
    assert st == 0
    assert out.tolist() == [2, 0, 3, 1, 1, 1,   3, 1, 0]
    assert asked.tolist() == [4, 1]


def test_budget_limits(oracle):
    rng = np.random.default_rng(5)
    ranks = rng.integers(0, 4, 200).astype(np.int32)
    co = np.array([0, 50, 50, 120, 200], np.int32)
    # a budget no sequence exhausts changes nothing
    st, out, asked = oracle.limit_high(ranks, co, 3, 1000)
    assert st == 0 and out.tolist() == ranks.tolist()
    assert asked.tolist() == [int((ranks[a:b] >= 3).sum()) for a, b in zip(co[:-1], co[1:])]
    # budget 0: every rung is capped below k_high
    st, out, _ = oracle.limit_high(ranks, co, 2, 0)
    assert out.tolist() == np.minimum(ranks, 1).tolist()
    # k_high above the ladder: nothing asks
    st, out, asked = oracle.limit_high(ranks, co, 4, 0)
    assert out.tolist() == ranks.tolist() and asked.tolist() == [0, 0, 0, 0]
    assert oracle.limit_high(ranks, co, 0, 1)[0] != 0
    assert oracle.limit_high(ranks, co, 1, -1)[0] != 0


@pytest.mark.parametrize("seed", range(6))
def test_budget_against_restatement(oracle, seed):
    """Restated with prefix counts: a chunk is lowered iff it asks and at least `budget` earlier
    chunks of its sequence asked."""
    rng = np.random.default_rng(seed)
    K = int(rng.integers(2, 6))
    k_high = int(rng.integers(1, K))
    budget = int(rng.integers(0, 5))
    lens = rng.integers(0, 30, 7)
    co = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ranks = rng.integers(0, K, co[-1]).astype(np.int32)
    st, out, asked = oracle.limit_high(ranks, co, k_high, budget)
    assert st == 0
    for a, b in zip(co[:-1], co[1:]):
        seg = ranks[a:b]
        asks = seg >= k_high
        before = np.cumsum(asks) - asks
        want = np.where(asks & (before >= budget), k_high - 1, seg)
        assert out[a:b].tolist() == want.tolist()
        assert int((out[a:b] >= k_high).sum()) == min(budget, int(asks.sum()))


# ---------------------------------------------------------------- percentile buckets, micro-batches

def test_buckets_hand_worked(oracle):
    # means 10, 40, 20, 30 (lengths 1, 2, 1, 3) and an empty sequence (mean 0)
    so = [0, 1, 3, 4, 7, 7]
    q = [10, 40, 41, 20, 30, 30, 32]
    st, o = oracle.bucket_sequences(q, so, 2, 2)
    assert st == 0
    assert o["seq_sum"].tolist() == [10, 81, 20, 92, 0]
    # ranked: empty(0) < s0(10) < s2(20) < s3(30) < s1(40)
    assert o["order"].tolist() == [4, 0, 2, 3, 1]
    # ranks 0,1,2 | 3,4 with 5 sequences in 2 buckets: floor(rho*2/5)
    assert o["bucket"].tolist() == [0, 1, 0, 1, 0]
    # dealt 4,0 | 3,2 (reversed) | 1
    assert o["micro"].tolist() == [1, 0, 1, 0, 0]


@pytest.mark.parametrize("seed", range(5))
def test_buckets_against_numpy_sort(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 40))
    q, so = ragged(rng, n, 0, 60)
    nb = int(rng.integers(1, 7))
    nm = int(rng.integers(1, 6))
    st, o = oracle.bucket_sequences(q, so, nb, nm)
    assert st == 0
    sums = np.array([int(q[a:b].astype(np.int64).sum()) for a, b in zip(so[:-1], so[1:])])
    lens = np.diff(so)
    means = np.where(lens > 0, sums // np.maximum(lens, 1), 0)
    assert o["seq_sum"].tolist() == sums.tolist()
    order = np.argsort(means, kind="stable")
    assert o["order"].tolist() == order.tolist()
    rho = np.empty(n, np.int64)
    rho[order] = np.arange(n)
    # percentile bins: bucket b holds the ranks in [ceil(b n / nb), ceil((b+1) n / nb))
    for s in range(n):
        b = int(o["bucket"][s])
        assert -(-b * n // nb) <= rho[s] < -(-(b + 1) * n // nb)
    assert np.all(np.diff(o["bucket"][order]) >= 0)
    counts = np.bincount(o["bucket"], minlength=nb)
    assert counts.max() - counts.min() <= 1
    # micro-batches: equal counts within one, total complexity within the spread of the means
    mcount = np.bincount(o["micro"], minlength=nm)
    assert mcount.max() - mcount.min() <= 1
    full_rounds = n // nm * nm
    tot = np.bincount(o["micro"][order[:full_rounds]], weights=means[order[:full_rounds]], minlength=nm)
    assert tot.max() - tot.min() <= means.max() - means.min()


def test_buckets_ties_go_by_index(oracle):
    so = np.arange(0, 7) * 3
    q = np.full(18, 500, np.int32)
    st, o = oracle.bucket_sequences(q, so, 3, 0)
    assert o["order"].tolist() == [0, 1, 2, 3, 4, 5]
    assert o["bucket"].tolist() == [0, 0, 1, 1, 2, 2]


# ---------------------------------------------------------------- aligned chunker

def table(res):
    return (res["chunk_offsets"].tolist(), res["chunk_start"].tolist(), res["chunk_len"].tolist(),
            res["chunk_sum"].tolist())


@pytest.mark.parametrize("seed", range(4))
def test_one_sequence_per_bucket_is_the_plain_chunker(oracle, seed):
    rng = np.random.default_rng(seed)
    q, so = ragged(rng, 6, 0, 200)
    st0, plain = oracle.partition(q, so, 4, 24, 3000, 700)
    perm = rng.permutation(6)
    st1, al = oracle.partition_aligned(q, so, perm, 6, 4, 24, 3000, 700)
    assert st0 == 0 and st1 == 0
    assert table(al) == table(plain)


def test_identical_sequences_keep_their_boundaries(oracle):
    rng = np.random.default_rng(9)
    q1, _ = ragged(rng, 1, 150, 150)
    q = np.tile(q1, 4)
    so = np.arange(5) * 150
    st0, plain = oracle.partition(q, so, 4, 24, 3000, 700)
    st1, al = oracle.partition_aligned(q, so, [0, 1, 0, 1], 2, 4, 24, 3000, 700)
    assert st0 == 0 and st1 == 0 and table(al) == table(plain)


def test_aligned_hand_worked(oracle):
    # one bucket, two sequences of 8 and 5 tokens; L = (2, 4), theta = 100, no deviation test.
    # mean series: floor((a+b)/2) while both run, then a alone
    a = [10, 10, 300, 10, 10, 10, 10, 10]
    b = [11, 20, 100, 10, 10]
    m = [10, 15, 200, 10, 10, 10, 10, 10]
    # chunker on m: [0,2) closes because m[2] >= theta; [2,4): mean 105 >= theta closes at once;
    # [4,8): nothing fires, runs to the end (4 tokens)
    assert restated_partition(m, 2, 4, 100, INF_Q) == [(0, 2, 25), (2, 2, 210), (4, 4, 40)]
    st, al = oracle.partition_aligned(a + b, [0, 8, 13], [0, 0], 1, 2, 4, 100, INF_Q)
    assert st == 0
    assert al["chunk_offsets"].tolist() == [0, 3, 6]
    assert al["chunk_start"].tolist() == [0, 2, 4, 8, 10, 12]
    assert al["chunk_len"].tolist() == [2, 2, 4, 2, 2, 1]          # the short member's last chunk is cut
    assert al["chunk_sum"].tolist() == [20, 310, 40, 31, 110, 10]  # each member's own scores


@pytest.mark.parametrize("seed", range(6))
def test_aligned_against_restatement(oracle, seed):
    """Bucket mean series with Python integers, boundaries from the independent restatement of the
    chunk rule, members cut at their own length."""
    rng = np.random.default_rng(40 + seed)
    n = int(rng.integers(2, 9))
    q, so = ragged(rng, n, 0, 90)
    nb = int(rng.integers(1, 4))
    bucket = rng.integers(0, nb, n)
    l_min, l_max = 3, 11
    theta, delta = 2500, 600
    st, al = oracle.partition_aligned(q, so, bucket, nb, l_min, l_max, theta, delta)
    assert st == 0
    lens = np.diff(so)
    want_off, want = [0], []
    bounds = {}
    for b in range(nb):
        mem = [s for s in range(n) if bucket[s] == b]
        tmax = max([lens[s] for s in mem], default=0)
        m = []
        for t in range(tmax):
            vals = [int(q[so[s] + t]) for s in mem if lens[s] > t]
            m.append(sum(vals) // len(vals))
        bounds[b] = [c[0] for c in restated_partition(m, l_min, l_max, theta, delta)] + [tmax]
    for s in range(n):
        e = bounds[int(bucket[s])]
        for i in range(len(e) - 1):
            if e[i] >= lens[s]:
                break
            hi = min(e[i + 1], lens[s])
            want.append((so[s] + e[i], hi - e[i], int(q[so[s] + e[i]: so[s] + hi].astype(np.int64).sum())))
        want_off.append(len(want))
    assert al["chunk_offsets"].tolist() == want_off
    assert list(zip(al["chunk_start"].tolist(), al["chunk_len"].tolist(), al["chunk_sum"].tolist())) == want
    # every sequence is tiled exactly, and members of a bucket share their boundaries
    for s in range(n):
        a_, b_ = al["chunk_offsets"][s], al["chunk_offsets"][s + 1]
        starts, ls = al["chunk_start"][a_:b_], al["chunk_len"][a_:b_]
        assert ls.sum() == lens[s]
        if b_ > a_:
            assert starts[0] == so[s] and np.all(starts[1:] == starts[:-1] + ls[:-1])


def test_aligned_errors(oracle):
    q = np.arange(20, dtype=np.int32)
    assert oracle.partition_aligned(q, [0, 10, 20], [0, 2], 2, 2, 4, 100, 100)[0] != 0     # bucket out of range
    assert oracle.partition_aligned(q, [0, 10, 20], [0, 1], 2, 3, 4, 100, 100)[0] == 3     # infeasible bounds
    st, al = oracle.partition_aligned(q, [0, 10, 20], [0, 1], 2, 2, 4, 100, 100, cap=3)
    assert st == 4                                                                        # capacity


# ---------------------------------------------------------------- decode step of a batch: aligned, budgeted

LADDER = ([0, 4, 8, 16], [0.0, 4.0, 2.0, 1.0])
TAUS = [1000, 2500, 4200]


def level_scores(rng, n_seqs, T):
    """Equal-length sequences made of spans of one difficulty level each, scaled per sequence."""
    q = np.empty((n_seqs, T), np.int32)
    for s in range(n_seqs):
        row = np.concatenate([rng.choice([600, 2000, 5000]) + rng.randint(-300, 300, size=rng.randint(5, 50))
                              for _ in range(T // 5 + 1)])[:T]
        q[s] = np.clip(row * (0.6 + 0.1 * s), 0, 1 << 20)
    return q


def feed(oracle, q, l_min, l_max, theta, delta, w, bucket=None, n_buckets=0, k_high=1, budget=0, use_budget=False):
    """Feed a batch token by token.  Returns per sequence: closed chunks (start, len, sum), rung in force
    at every token, gates."""
    n_seqs, T = q.shape
    st = oracle.StreamState(n_seqs)
    bst = oracle.BucketState(n_buckets) if bucket is not None else None
    n_high = np.zeros(n_seqs, np.int32) if use_budget else None
    chunks = [[] for _ in range(n_seqs)]
    rungs = np.zeros((n_seqs, T), np.int32)
    gates = []
    for t in range(T):
        code, out = oracle.stream_step_aligned(st, q[:, t], l_min, l_max, theta, delta, TAUS, *LADDER, w,
                                               bucket=bucket, bucket_state=bst, k_high=k_high, budget=budget,
                                               n_high=n_high)
        assert code == 0
        for s in range(n_seqs):
            n = int(out["closed_len"][s])
            if n:
                chunks[s].append((t - n, n, int(out["closed_sum"][s])))
        rungs[:, t] = st.k_cur
        gates.append({k: v.copy() for k, v in out.items()})
    return chunks, rungs, gates, st, n_high


def test_step_without_buckets_and_budget_is_the_plain_step(oracle):
    rng = np.random.RandomState(1)
    q = level_scores(rng, 4, 300)
    st0 = oracle.StreamState(4)
    st1 = oracle.StreamState(4)
    for t in range(300):
        c0, o0 = oracle.stream_step(st0, q[:, t], 5, 24, 4000, 1200, TAUS, *LADDER, 3)
        c1, o1 = oracle.stream_step_aligned(st1, q[:, t], 5, 24, 4000, 1200, TAUS, *LADDER, 3)
        assert c0 == 0 and c1 == 0
        for k in o0:
            assert o0[k].tolist() == o1[k].tolist(), (t, k)
    for f in ("n", "sum", "k_cur", "k_prev", "chunks", "pos"):
        assert getattr(st0, f).tolist() == getattr(st1, f).tolist()


@pytest.mark.parametrize("seed", range(4))
def test_aligned_budgeted_step_reproduces_the_batch_forms(oracle, seed):
    """Token by token on equal-length sequences: the boundaries of the aligned batch chunker wherever the
    end cannot matter, and at every chunk's last token the rung of select followed by the budget."""
    rng = np.random.RandomState(10 + seed)
    n_seqs, T = 6, 500
    l_min, l_max = [(4, 9), (8, 40), (3, 5), (6, 30)][seed]
    theta, delta, k_high, budget = 4500, 1300, 2, [0, 1, 3, 5][seed]
    q = level_scores(rng, n_seqs, T)
    bucket = np.array([0, 1, 0, 2, 1, 0], np.int32)
    so = np.arange(n_seqs + 1) * T
    code, tab = oracle.partition_aligned(q.ravel(), so, bucket, 3, l_min, l_max, theta, delta)
    assert code == 0
    ranks = oracle.select(tab["chunk_sum"], tab["chunk_len"], TAUS)
    code, limited, _ = oracle.limit_high(ranks, tab["chunk_offsets"], k_high, budget)
    assert code == 0
    chunks, rungs, _, _, n_high = feed(oracle, q, l_min, l_max, theta, delta, 2, bucket, 3, k_high, budget, True)
    lowered = 0
    for s in range(n_seqs):
        a, b = tab["chunk_offsets"][s], tab["chunk_offsets"][s + 1]
        batch = [(int(tab["chunk_start"][c]) - s * T, int(tab["chunk_len"][c]), int(tab["chunk_sum"][c]), int(limited[c]),
                  int(ranks[c])) for c in range(a, b)]
        safe = [c for c in batch if c[0] + l_max <= T - l_min]
        assert len(safe) > 5
        assert chunks[s][:len(safe)] == [c[:3] for c in safe]
        assert [int(rungs[s, c[0] + c[1] - 1]) for c in safe] == [c[3] for c in safe]
        lowered += sum(1 for c in safe if c[3] != c[4])
        assert n_high[s] >= sum(1 for c in safe if c[4] >= k_high)
    if budget < 5:
        assert lowered > 0          # the budget did bite somewhere


def test_members_of_a_bucket_close_together(oracle):
    rng = np.random.RandomState(5)
    q = level_scores(rng, 5, 200)
    bucket = np.array([1, 0, 1, 1, 0], np.int32)
    chunks, _, _, _, _ = feed(oracle, q, 4, 16, 4500, 1300, 0, bucket, 2)
    for members in ([0, 2, 3], [1, 4]):
        first = [(c[0], c[1]) for c in chunks[members[0]]]
        for s in members[1:]:
            assert [(c[0], c[1]) for c in chunks[s]] == first
    assert [(c[0], c[1]) for c in chunks[0]] != [(c[0], c[1]) for c in chunks[1]]


def test_aligned_step_hand_worked(oracle):
    # one bucket of two sequences, L = (2, 4), theta = 100, no deviation test, rungs at means 50 / 150 / 250,
    # k_high = 2 with a budget of one chunk
    a = [10, 10, 300, 10, 10, 10]
    b = [11, 20, 300, 300, 10, 10]
    # means 10, 15, 300, 155, 10, 10: [0,2) closes in front of t=2 (its mean token is hard); [2,4): bucket mean
    # (300 + 155) / 2 >= 100 closes in front of t=4
    st = oracle.StreamState(2)
    bst = oracle.BucketState(1)
    n_high = np.zeros(2, np.int32)
    closed, rung = [], []
    for t in range(6):
        code, out = oracle.stream_step_aligned(st, [a[t], b[t]], 2, 4, 100, INF_Q, [50, 150, 250], *LADDER, 0,
                                               bucket=[0, 0], bucket_state=bst, k_high=2, budget=1, n_high=n_high)
        assert code == 0
        closed.append(out["closed_len"].tolist())
        rung.append(st.k_cur.tolist())
    assert closed == [[0, 0], [0, 0], [2, 2], [0, 0], [2, 2], [0, 0]]
    # sequence a: chunk [2,4) has means 300, 155 -> rungs 3, 2 (first asker, kept); chunk [4,6): mean 10 -> 0
    # sequence b: chunk [2,4) means 300, 300 -> 3, 3 (kept, it is the first asker)
    assert [r[0] for r in rung] == [0, 0, 3, 2, 0, 0]
    assert [r[1] for r in rung] == [0, 0, 3, 3, 0, 0]
    assert n_high.tolist() == [1, 1]
    # a further hard chunk is now over budget in both sequences: lowered to rung 1
    for t in range(2):
        code, out = oracle.stream_step_aligned(st, [400, 400], 2, 4, 100, INF_Q, [50, 150, 250], *LADDER, 0,
                                               bucket=[0, 0], bucket_state=bst, k_high=2, budget=1, n_high=n_high)
        assert st.k_cur.tolist() == [1, 1]
        assert out["r_cur"].tolist() == [4, 4] and out["g_cur"].tolist() == [4.0, 4.0]


def test_aligned_step_errors(oracle):
    st = oracle.StreamState(2)
    bst = oracle.BucketState(2)
    assert oracle.stream_step_aligned(st, [1, 2], 2, 4, 100, 100, TAUS, *LADDER, 0, bucket=[0, 2],
                                      bucket_state=bst)[0] != 0
    assert oracle.stream_step_aligned(st, [1, 2], 2, 4, 100, 100, TAUS, *LADDER, 0, k_high=0, budget=1,
                                      n_high=np.zeros(2, np.int32))[0] != 0
    assert oracle.stream_step_aligned(st, [1, 2], 3, 4, 100, 100, TAUS, *LADDER, 0)[0] == 3


# ---------------------------------------------------------------- the integer means are floors

def test_sequence_mean_is_a_floor(oracle):
    # sums 10 and 8 over 4 tokens: floors 2 and 2 tie and go by index; rounded up or to nearest the first would be 3
    st, o = oracle.bucket_sequences([3, 3, 2, 2, 2, 2, 2, 2], [0, 4, 8], 2, 0)
    assert st == 0 and o["seq_sum"].tolist() == [10, 8]
    assert o["order"].tolist() == [0, 1] and o["bucket"].tolist() == [0, 1]


def test_bucket_mean_series_is_a_floor(oracle):
    # members score 10 and 11 at position 2, theta = 11: the mean floor(21 / 2) = 10 stays below it, so nothing closes the
    # first chunk before L_max; rounded to nearest the mean would be 11 and close it in front of position 2
    a = [0, 0, 10, 0, 0, 0, 0, 0]
    b = [0, 0, 11, 0, 0, 0, 0, 0]
    st, al = oracle.partition_aligned(a + b, [0, 8, 16], [0, 0], 1, 2, 4, 11, INF_Q)
    assert st == 0
    assert al["chunk_len"].tolist() == [4, 4, 4, 4]
    # with 12 in place of 11 the floor reaches theta and the chunk is closed there: [0,2), then [2,6) (nothing fires,
    # L_max), then the tail [6,8)
    b[2] = 12
    st, al = oracle.partition_aligned(a + b, [0, 8, 16], [0, 0], 1, 2, 4, 11, INF_Q)
    assert al["chunk_len"].tolist() == [2, 4, 2, 2, 4, 2]


def test_bucket_mean_of_a_step_is_a_floor(oracle):
    st = oracle.StreamState(2)
    bst = oracle.BucketState(1)
    closed = []
    for q in ([0, 0], [0, 0], [10, 11], [0, 0], [0, 0], [10, 12]):
        code, out = oracle.stream_step_aligned(st, q, 2, 8, 11, INF_Q, TAUS, *LADDER, 0, bucket=[0, 0], bucket_state=bst)
        assert code == 0
        closed.append(out["closed_len"].tolist())
    # (10 + 11) // 2 = 10 < theta: no close; (10 + 12) // 2 = 11 >= theta: the five tokens so far are closed
    assert closed == [[0, 0], [0, 0], [0, 0], [0, 0], [0, 0], [5, 5]]
