"""GPU parity of cwl_select_ranks_budget, cwl_bucket_sequences and cwl_partition_chunks_aligned
against the CPU oracle: integer work, so every output must match bit for bit when both sides start
from the same fp32 scores."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from helpers import assert_tables_equal, gpu_table_to_host
from paper_2601_21109_amd import binding as B
from test_gpu_partition import synth_scores

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def scores_by_sequence(seq_lens, vocab, seed):
    """synth_scores with a per-sequence difficulty factor, so that the sequences of a batch differ in
    mean complexity the way prompts of different kinds do."""
    h = synth_scores(seq_lens, vocab, seed)
    rng = np.random.RandomState(seed + 1)
    t = 0
    for n in seq_lens:
        h[t:t + n] *= rng.uniform(0.4, 1.0)
        t += n
    return h.astype(np.float32)


def offsets(seq_lens):
    return np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int32)


CASES = [
    ([128], 8, 64, 1024),
    ([2048] * 8, 32, 512, 32000),
    ([5, 0, 31, 32, 33, 63, 64, 65, 1000, 0, 7, 2047, 4096], 32, 512, 32000),
    ([1] * 40 + [300] * 5, 4, 7, 1024),
    ([977] * 300, 16, 40, 32000),
    ([9000, 100, 100, 100], 16, 256, 32000),
    ([20000, 50, 0, 50, 50], 16, 256, 32000),
    ([4096] * 16, 32, 512, 32000),          # the shapes of the larger workloads, whole
    ([2048] * 32, 32, 512, 32000),
    ([32768], 64, 2048, 128000),
]


@pytest.mark.parametrize("seq_lens,l_min,l_max,vocab", CASES)
@pytest.mark.parametrize("k_high,budget", [(1, 0), (2, 1), (3, 2), (2, 5), (3, 100000), (4, 0)])
def test_budget_matches_oracle(seq_lens, l_min, l_max, vocab, k_high, budget):
    h = scores_by_sequence(seq_lens, vocab, 3)
    so = offsets(seq_lens)
    lnv = math.log(vocab)
    theta, delta, taus = 0.9 * lnv, 0.25 * lnv, [0.3 * lnv, 0.6 * lnv, 0.9 * lnv]
    hd, sod = torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV)
    table = B.partition_chunks(hd, sod, l_min, l_max, theta, delta)
    ri, asked = B.select_ranks_budget(table, taus, 4, k_high, budget)
    plain = B.select_ranks(table, taus, 4)
    torch.cuda.synchronize()
    q, _ = O.quantise(h)
    st, ref = O.partition(q, so, l_min, l_max, O.quantise_threshold(theta), O.quantise_threshold(delta))
    assert st == 0
    ref_ri = O.select(ref["chunk_sum"], ref["chunk_len"], [O.quantise_threshold(t) for t in taus])
    st, lim, ref_asked = O.limit_high(ref_ri, ref["chunk_offsets"], k_high, budget)
    assert st == 0
    n = int(ref["chunk_offsets"][-1])
    assert ri.cpu().numpy()[:n].tolist() == lim.tolist()
    assert asked.cpu().numpy()[:len(seq_lens)].tolist() == ref_asked.tolist()
    if budget >= 100000 or k_high >= 4:
        assert ri.cpu().numpy()[:n].tolist() == plain.cpu().numpy()[:n].tolist()


@pytest.mark.parametrize("seq_lens,l_min,l_max,vocab", CASES + [([3] * 4096, 2, 3, 1024)])
@pytest.mark.parametrize("n_buckets,n_micro", [(1, 1), (2, 3), (4, 2), (7, 5)])
def test_buckets_match_oracle(seq_lens, l_min, l_max, vocab, n_buckets, n_micro):
    h = scores_by_sequence(seq_lens, vocab, 11)
    so = offsets(seq_lens)
    out = B.bucket_sequences(torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV), n_buckets, n_micro)
    torch.cuda.synchronize()
    q, _ = O.quantise(h)
    st, ref = O.bucket_sequences(q, so, n_buckets, n_micro)
    assert st == 0
    n = len(seq_lens)
    for key in ("seq_sum", "order", "bucket", "micro"):
        assert out[key].cpu().numpy()[:n].tolist() == ref[key].tolist(), key


def test_buckets_without_micro_batches():
    seq_lens = [100, 40, 70]
    h = scores_by_sequence(seq_lens, 1024, 2)
    so = offsets(seq_lens)
    out = B.bucket_sequences(torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV), 2)
    torch.cuda.synchronize()
    st, ref = O.bucket_sequences(O.quantise(h)[0], so, 2, 0)
    assert "micro" not in out and out["bucket"].cpu().tolist() == ref["bucket"].tolist()


def run_aligned(h, seq_lens, bucket, n_buckets, l_min, l_max, theta, delta, cap=None):
    so = offsets(seq_lens)
    hd, sod = torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV)
    bd = torch.from_numpy(np.asarray(bucket, np.int32)).to(DEV)
    table = B.partition_chunks_aligned(hd, sod, bd, n_buckets, l_min, l_max, theta, delta, cap=cap)
    torch.cuda.synchronize()
    gpu = gpu_table_to_host(table)
    q, nan_seen = O.quantise(h)
    st, ref = O.partition_aligned(q, so, bucket, n_buckets, l_min, l_max, O.quantise_threshold(theta),
                                  O.quantise_threshold(delta), cap=cap)
    return gpu, ref, st, nan_seen


@pytest.mark.parametrize("seq_lens,l_min,l_max,vocab", CASES)
@pytest.mark.parametrize("n_buckets", [1, 2, 5])
def test_aligned_chunker_matches_oracle(seq_lens, l_min, l_max, vocab, n_buckets):
    h = scores_by_sequence(seq_lens, vocab, 7)
    so = offsets(seq_lens)
    lnv = math.log(vocab)
    # buckets from the library's own percentile call (checked against the oracle above)
    out = B.bucket_sequences(torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV), n_buckets)
    bucket = out["bucket"].cpu().numpy()[:len(seq_lens)]
    gpu, ref, st, _ = run_aligned(h, seq_lens, bucket, n_buckets, l_min, l_max, 0.9 * lnv, 0.25 * lnv)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)


def test_one_sequence_per_bucket_is_the_plain_chunker():
    seq_lens = [700, 0, 333, 2048, 64, 31]
    h = scores_by_sequence(seq_lens, 32000, 5)
    so = offsets(seq_lens)
    lnv = math.log(32000)
    hd, sod = torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV)
    plain = B.partition_chunks(hd, sod, 16, 128, 0.9 * lnv, 0.25 * lnv)
    bd = torch.tensor([3, 1, 5, 0, 2, 4], dtype=torch.int32, device=DEV)
    al = B.partition_chunks_aligned(hd, sod, bd, 6, 16, 128, 0.9 * lnv, 0.25 * lnv)
    torch.cuda.synchronize()
    assert_tables_equal(gpu_table_to_host(al), gpu_table_to_host(plain))


def test_aligned_empty_buckets_and_random_assignment():
    rng = np.random.RandomState(0)
    seq_lens = rng.randint(0, 600, 37).tolist()
    h = scores_by_sequence(seq_lens, 32000, 8)
    bucket = rng.choice([0, 2, 3, 9], 37)            # buckets 1, 4..8 stay empty
    lnv = math.log(32000)
    gpu, ref, st, _ = run_aligned(h, seq_lens, bucket, 10, 8, 64, 0.9 * lnv, 0.25 * lnv)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)


def test_aligned_status_bits():
    seq_lens = [200, 120]
    h = scores_by_sequence(seq_lens, 1024, 4)
    lnv = math.log(1024)
    h[50] = np.nan
    gpu, ref, st, nan_seen = run_aligned(h, seq_lens, [0, 0], 1, 8, 64, 0.9 * lnv, 0.25 * lnv)
    assert nan_seen and gpu["status"] == B.STATUS_NAN_SCORE
    assert_tables_equal(gpu, ref)
    # capacity: the first `cap` chunks are written and the bit is set
    h = scores_by_sequence(seq_lens, 1024, 4)
    gpu, ref, st, _ = run_aligned(h, seq_lens, [0, 1], 2, 8, 64, 0.9 * lnv, 0.25 * lnv, cap=3)
    assert st == O.reference.ERR_CAPACITY and gpu["status"] == B.STATUS_CAPACITY
    assert gpu["chunk_offsets"].tolist() == ref["chunk_offsets"].tolist()
    assert gpu["chunk_start"].tolist() == ref["chunk_start"].tolist()
    assert gpu["chunk_sum"].tolist() == ref["chunk_sum"].tolist()
    # a bucket index out of range is flagged and taken as the nearest bucket
    so = offsets(seq_lens)
    hd, sod = torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV)
    bd = torch.tensor([-3, 7], dtype=torch.int32, device=DEV)
    t = B.partition_chunks_aligned(hd, sod, bd, 2, 8, 64, 0.9 * lnv, 0.25 * lnv)
    torch.cuda.synchronize()
    got = gpu_table_to_host(t)
    assert got["status"] == B.STATUS_BAD_BUCKET
    st, ref = O.partition_aligned(O.quantise(h)[0], so, [0, 1], 2, 8, 64, O.quantise_threshold(0.9 * lnv),
                                  O.quantise_threshold(0.25 * lnv))
    assert_tables_equal(got, ref)


def test_aligned_table_feeds_the_linear():
    """The aligned table is an ordinary chunk table: the projection on it matches the oracle."""
    from helpers import TOL_F32, rel_err, host
    seq_lens = [96, 64, 80]
    h = scores_by_sequence(seq_lens, 1024, 6)
    so = offsets(seq_lens)
    lnv = math.log(1024)
    taus = [0.3 * lnv, 0.6 * lnv, 0.9 * lnv]
    hd, sod = torch.from_numpy(h).to(DEV), torch.from_numpy(so).to(DEV)
    bk = B.bucket_sequences(hd, sod, 2)
    table = B.partition_chunks_aligned(hd, sod, bk["bucket"], 2, 4, 16, 0.9 * lnv, 0.25 * lnv)
    ri, _ = B.select_ranks_budget(table, taus, 4, 3, 2)
    g = torch.Generator(device="cpu").manual_seed(1)
    d_in, d_out, r_max = 64, 48, 16
    x = torch.randn(sum(seq_lens), d_in, generator=g)
    W = torch.randn(d_in, d_out, generator=g) / 8
    A = torch.randn(d_in, r_max, generator=g) / 8
    Bm = torch.randn(r_max, d_out, generator=g) / 4
    ranks, scales = [0, 4, 8, 16], [0.0, 2.0, 1.5, 1.0]
    y = B.chunkwise_lora_linear(x.to(DEV), W.to(DEV), A.to(DEV), Bm.to(DEV), ranks, scales, 2, sod, table, ri)
    torch.cuda.synchronize()
    tab = gpu_table_to_host(table, ri)
    ref = O.linear(x.numpy(), W.numpy(), A.numpy(), Bm.numpy(), ranks, scales, 2, so, tab["chunk_offsets"],
                   tab["chunk_start"], tab["chunk_len"], tab["rank_idx"])
    assert rel_err(host(y), ref) <= TOL_F32


# ---------------------------------------------------------------- decode step of a batch: aligned, budgeted

def gate_fields(gate):
    g = gate.cpu().numpy()
    return g[:, 0].copy(), g[:, 1].copy(), g[:, 2].copy().view(np.float32), g[:, 3].copy().view(np.float32)


@pytest.mark.parametrize("n_seqs,n_buckets,steps,l_min,l_max,w,ladder,k_high,budget", [
    (37, 3, 300, 4, 9, 2, ([4, 8, 16], [4.0, 2.0, 1.0]), 2, 3),
    (300, 7, 120, 8, 64, 4, ([8, 16, 32, 64], [2.0, 1.0, 0.5, 0.25]), 2, 1),
    (64, 1, 200, 3, 40, 3, ([0, 4, 16], [0.0, 2.0, 1.0]), 1, 0),
    (4096, 4096, 12, 2, 4, 1, ([4, 8], [1.0, 0.5]), 1, 2),         # the largest batch the call takes
    (9, 12, 150, 4, 16, 2, ([4, 8, 16], [4.0, 2.0, 1.0]), 2, None),  # empty buckets, no budget
    (50, 0, 150, 4, 16, 2, ([4, 8, 16], [4.0, 2.0, 1.0]), 2, 2),     # no buckets, budget only
    (40, 5, 150, 4, 16, 3, (list(range(0, 256, 16)), [0.0] + [16.0 / r for r in range(16, 256, 16)]), 9, 2),  # 16 rungs
])
def test_aligned_stream_step_matches_oracle(n_seqs, n_buckets, steps, l_min, l_max, w, ladder, k_high, budget):
    ranks, scales = ladder
    K = len(ranks)
    vocab_ln = math.log(32000.0)
    theta, delta = 0.9 * vocab_ln, 0.3 * vocab_ln
    taus = [vocab_ln * f for f in np.linspace(0.3, 0.9, K - 1)] if K > 1 else []
    rng = np.random.RandomState(n_seqs + 1)
    level = rng.choice([0.15, 0.5, 0.95], size=(n_seqs, steps // 10 + 1)).repeat(10, axis=1)[:, :steps]
    h_all = (level * vocab_ln + rng.uniform(-0.4, 0.4, size=(n_seqs, steps))).astype(np.float32)
    use_b = n_buckets > 0
    bucket = rng.randint(0, max(n_buckets, 1), n_seqs).astype(np.int32) if use_b else None
    bucket_d = torch.from_numpy(bucket).to(DEV) if use_b else None
    bst_d = B.bucket_state(n_buckets, DEV) if use_b else None
    n_high_d = torch.zeros(n_seqs, dtype=torch.int32, device=DEV) if budget is not None else None
    state = B.stream_state(n_seqs, DEV)
    dev_out = []
    for t in range(steps):
        h = torch.from_numpy(h_all[:, t].copy()).to(DEV)
        out = B.stream_step_aligned(h, state, l_min, l_max, theta, delta, taus, ranks, scales, w, bucket=bucket_d,
                                    bucket_st=bst_d, k_high=k_high, budget=budget or 0, n_high=n_high_d)
        dev_out.append({k: v.clone() for k, v in out.items()})
    torch.cuda.synchronize()
    ost = O.StreamState(n_seqs)
    obst = O.BucketState(n_buckets) if use_b else None
    o_high = np.zeros(n_seqs, np.int32) if budget is not None else None
    tq = [O.quantise_threshold(t) for t in taus]
    for t in range(steps):
        q, _ = O.quantise(h_all[:, t])
        code, ref = O.stream_step_aligned(ost, q, l_min, l_max, O.quantise_threshold(theta),
                                          O.quantise_threshold(delta), tq, ranks, scales, w, bucket=bucket,
                                          bucket_state=obst, k_high=k_high, budget=budget or 0, n_high=o_high)
        assert code == 0
        r_cur, r_prev, g_cur, g_prev = gate_fields(dev_out[t]["gate"])
        assert np.array_equal(r_cur, ref["r_cur"]) and np.array_equal(r_prev, ref["r_prev"]), t
        assert np.array_equal(dev_out[t]["closed_len"].cpu().numpy(), ref["closed_len"]), t
        assert np.array_equal(dev_out[t]["closed_sum"].cpu().numpy(), ref["closed_sum"]), t
        np.testing.assert_allclose(g_cur, ref["g_cur"], rtol=1e-6, atol=0)
        np.testing.assert_allclose(g_prev, ref["g_prev"], rtol=1e-6, atol=0)
        assert int(dev_out[t]["status_word"].item()) == 0
    f = B.stream_state_fields(state)
    assert np.array_equal(f["n"], ost.n) and np.array_equal(f["sum"], ost.sum)
    assert np.array_equal(f["k_cur"], ost.k_cur) and np.array_equal(f["n_chunks"], ost.chunks)
    if use_b:
        bs = bst_d.cpu().numpy()
        assert np.array_equal(bs[:, 0], obst.sum) and np.array_equal((bs[:, 1] & 0xffffffff).astype(np.int32), obst.n)
    if budget is not None:
        assert np.array_equal(n_high_d.cpu().numpy(), o_high)
    assert ost.chunks.sum() > 0


def test_aligned_stream_step_flags():
    state = B.stream_state(3, DEV)
    bst = B.bucket_state(2, DEV)
    h = torch.tensor([1.0, float("nan"), 2.0], device=DEV)
    bucket = torch.tensor([0, 5, -1], dtype=torch.int32, device=DEV)
    out = B.stream_step_aligned(h, state, 2, 4, math.inf, math.inf, [1.5], [4, 8], [1.0, 0.5], 0, bucket=bucket,
                                bucket_st=bst)
    torch.cuda.synchronize()
    assert int(out["status_word"].item()) == B.STATUS_NAN_SCORE | B.STATUS_BAD_BUCKET
    # buckets taken as 0, 1, 0: bucket 0 sees (1024 + 2048) // 2, bucket 1 the NaN scored as 0
    bs = bst.cpu().numpy()
    assert bs[:, 0].tolist() == [1536, 0] and (bs[:, 1] & 0xffffffff).tolist() == [1, 1]


def test_aligned_degenerate_batches():
    lnv = math.log(1024)
    # no sequences at all
    so = torch.zeros(1, dtype=torch.int32, device=DEV)
    t = B.partition_chunks_aligned(torch.empty(0, device=DEV), so, torch.empty(0, dtype=torch.int32, device=DEV), 3,
                                   4, 16, 0.9 * lnv, 0.25 * lnv)
    torch.cuda.synchronize()
    assert t["chunk_offsets"].cpu().tolist() == [0] and int(t["status_word"].item()) == 0
    # only empty sequences
    gpu, ref, st, _ = run_aligned(np.empty(0, np.float32), [0, 0, 0], [0, 1, 0], 2, 4, 16, 0.9 * lnv, 0.25 * lnv)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)
    assert gpu["chunk_offsets"].tolist() == [0, 0, 0, 0]
    # sequences shorter than l_min, more buckets than sequences
    h = scores_by_sequence([3, 1, 2], 1024, 1)
    gpu, ref, st, _ = run_aligned(h, [3, 1, 2], [4, 4, 0], 6, 4, 16, 0.9 * lnv, 0.25 * lnv)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)


@pytest.mark.parametrize("n_buckets", [1, 64, 4096])
def test_aligned_largest_batch(n_buckets):
    rng = np.random.RandomState(3)
    seq_lens = rng.randint(0, 40, 4096).tolist()
    h = scores_by_sequence(seq_lens, 1024, 12)
    bucket = rng.randint(0, n_buckets, 4096)
    lnv = math.log(1024)
    gpu, ref, st, _ = run_aligned(h, seq_lens, bucket, n_buckets, 3, 9, 0.9 * lnv, 0.25 * lnv)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)


def test_aligned_decode_step_replays_from_a_hip_graph():
    """The bucketed, budgeted scheduler step only enqueues one kernel: captured once, every replay (with eager work
    and synchronisations in between) must leave the same state, gates and counters as the eager call."""
    n_seqs, n_buckets = 24, 3
    ranks, scales = [4, 8, 16], [4.0, 2.0, 1.0]
    lnv = math.log(1500)
    args = (2, 4, 0.9 * lnv, 0.3 * lnv, [0.45 * lnv, 0.9 * lnv], ranks, scales, 2)
    h = torch.empty(n_seqs, dtype=torch.float32, device=DEV)
    bucket = (torch.arange(n_seqs, device=DEV, dtype=torch.int32) % n_buckets).contiguous()
    state, bst = B.stream_state(n_seqs, DEV), B.bucket_state(n_buckets, DEV)
    n_high = torch.zeros(n_seqs, dtype=torch.int32, device=DEV)
    kw = dict(bucket=bucket, bucket_st=bst, k_high=1, budget=2, n_high=n_high)
    out = B.stream_step_aligned(h.zero_(), state, *args, **kw)          # allocates the outputs once, outside the graph

    def reset():
        state.zero_(); bst.zero_(); n_high.zero_()

    def new_scores(i):
        gi = torch.Generator(device=DEV).manual_seed(500 + i)
        h.copy_(torch.rand(n_seqs, generator=gi, device=DEV) * lnv)

    reset()
    eager = []
    for i in range(8):
        new_scores(i)
        B.stream_step_aligned(h, state, *args, out=out, **kw)
        torch.cuda.synchronize()
        eager.append((state.clone(), bst.clone(), n_high.clone(), out["gate"].clone(), out["closed_len"].clone()))
    reset()
    new_scores(0)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.stream_step_aligned(h, state, *args, out=out, **kw)           # warm-up on the capture stream
        reset()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        B.stream_step_aligned(h, state, *args, out=out, **kw)
    for i in range(8):
        new_scores(i)
        graph.replay()
        torch.cuda.synchronize()
        got = (state, bst, n_high, out["gate"], out["closed_len"])
        for a, b in zip(got, eager[i]):
            assert torch.equal(a, b), i
    assert int(n_high.sum().item()) > 0 and int(out["status_word"].item()) == 0
