"""GPU parity of cwl_partition_chunks / cwl_select_ranks against the CPU oracle: the chunk
table must match bit for bit when both sides start from the same fp32 scores."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from helpers import assert_tables_equal, gpu_table_to_host
from paper_2601_21109_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def synth_scores(seq_lens, vocab, seed):
    """Piecewise-constant difficulty levels with noise, like the entropy of the synthetic logits."""
    rng = np.random.RandomState(seed)
    n = int(np.sum(seq_lens))
    h = np.empty(n, dtype=np.float32)
    t = 0
    lnv = math.log(vocab)
    while t < n:
        span = int(rng.randint(8, 200))
        level = rng.choice([0.19, 0.8, 0.985]) * lnv
        h[t:t + span] = level + rng.randn(min(span, n - t)) * 0.03 * lnv
        t += span
    return np.clip(h, 0, None).astype(np.float32)


def run_both(h, seq_lens, l_min, l_max, theta, delta, taus, cap=None):
    so = np.concatenate([[0], np.cumsum(seq_lens)]).astype(np.int32)
    hd = torch.from_numpy(h).to(DEV)
    sod = torch.from_numpy(so).to(DEV)
    table = B.partition_chunks(hd, sod, l_min, l_max, theta, delta, cap=cap)
    ri = B.select_ranks(table, taus, len(taus) + 1)
    torch.cuda.synchronize()
    gpu = gpu_table_to_host(table, ri)
    q, nan_seen = O.quantise(h)
    st, ref = O.partition(q, so, l_min, l_max, O.quantise_threshold(theta), O.quantise_threshold(delta),
                          cap=cap)
    ref["rank_idx"] = O.select(ref["chunk_sum"], ref["chunk_len"], [O.quantise_threshold(t) for t in taus])
    return gpu, ref, st, nan_seen


@pytest.mark.parametrize("seq_lens,l_min,l_max,vocab", [
    ([128], 8, 64, 1024),
    ([2048] * 8, 32, 512, 32000),
    ([32768], 64, 2048, 128000),
    ([5, 0, 31, 32, 33, 63, 64, 65, 1000, 0, 7, 2047, 4096], 32, 512, 32000),
    ([1] * 40 + [300] * 5, 4, 7, 1024),
    ([977] * 300, 16, 40, 32000),
    ([17, 4099, 23], 1, 1, 1024),
    ([4097], 3, 5000, 1024),
    ([9000, 100, 100, 100], 16, 256, 32000),   # short-sequence path, one sequence beyond its LDS
    ([20000, 50, 0, 50, 50], 16, 256, 32000),  # long-sequence path with short sequences in the batch
    ([40000, 300], 64, 2048, 32000),      # longer than the chain walk keeps in LDS
    ([20000, 9], 16, 15000, 32000),       # reach of a start (l_max) larger than the LDS window
])
def test_partition_matches_oracle(seq_lens, l_min, l_max, vocab):
    lnv = math.log(vocab)
    h = synth_scores(seq_lens, vocab, seed=len(seq_lens) * 7 + l_min)
    taus = [np.float32(f * lnv) for f in (0.3, 0.6, 0.9)]
    gpu, ref, st, _ = run_both(h, seq_lens, l_min, l_max, np.float32(0.9 * lnv), np.float32(0.3 * lnv), taus)
    assert st == 0 and gpu["status"] == 0
    assert_tables_equal(gpu, ref)
    lens = gpu["chunk_len"]
    assert int(lens.sum()) == int(np.sum(seq_lens))


def test_tests_disabled_and_all_hard():
    h = synth_scores([5000, 777], 1024, 3)
    gpu, ref, st, _ = run_both(h, [5000, 777], 8, 64, math.inf, math.inf, [1.0])
    assert_tables_equal(gpu, ref)
    assert set(gpu["chunk_len"].tolist()) <= set(range(8, 65)) and gpu["chunk_len"][0] == 64
    gpu, ref, st, _ = run_both(h + 100.0, [5000, 777], 8, 64, 1.0, math.inf, [1.0])
    assert_tables_equal(gpu, ref)
    assert gpu["chunk_len"][0] == 8 and gpu["rank_idx"].min() == 1


def test_threshold_ties_and_exact_grid():
    # scores on the Q10 grid, thresholds exactly on chunk means: ties must go up on both sides
    rng = np.random.RandomState(0)
    h = (rng.randint(0, 8, size=4096) * 0.5).astype(np.float32)
    gpu, ref, _, _ = run_both(h, [4096], 4, 16, 3.0, 1.0, [1.0, 1.75, 2.5])
    assert_tables_equal(gpu, ref)
    assert len(set(gpu["rank_idx"].tolist())) >= 3


def test_capacity_overflow_sets_status():
    h = synth_scores([4096], 1024, 4)
    gpu, ref, st, _ = run_both(h + 100.0, [4096], 8, 64, 1.0, math.inf, [1.0], cap=100)
    assert st == O.reference.ERR_CAPACITY
    assert gpu["status"] & B.STATUS_CAPACITY
    assert gpu["chunk_offsets"].tolist() == ref["chunk_offsets"].tolist() == [0, 512]
    assert gpu["chunk_start"].tolist() == ref["chunk_start"].tolist()
    assert len(gpu["chunk_len"]) == 100


def test_nan_score_and_bad_offsets_set_status():
    h = synth_scores([512], 1024, 5)
    h[77] = np.nan
    gpu, ref, st, nan_seen = run_both(h, [512], 8, 64, 6.0, 2.0, [3.0])
    assert nan_seen and (gpu["status"] & B.STATUS_NAN_SCORE)
    assert_tables_equal(gpu, ref)
    hd = torch.from_numpy(synth_scores([512], 1024, 6)).to(DEV)
    bad = torch.tensor([0, 300, 200, 512], dtype=torch.int32, device=DEV)
    t = B.partition_chunks(hd, bad, 8, 64, 6.0, 2.0)
    torch.cuda.synchronize()
    assert int(t["status_word"].item()) & B.STATUS_BAD_OFFSETS
    short = torch.tensor([0, 300, 500], dtype=torch.int32, device=DEV)
    t = B.partition_chunks(hd, short, 8, 64, 6.0, 2.0)
    assert int(t["status_word"].item()) & B.STATUS_BAD_OFFSETS


def test_no_sequences_and_determinism():
    hd = torch.zeros(0, dtype=torch.float32, device=DEV)
    t = B.partition_chunks(hd, torch.zeros(1, dtype=torch.int32, device=DEV), 4, 8)
    assert t["chunk_offsets"].cpu().tolist() == [0] and int(t["status_word"].item()) == 0
    h = synth_scores([2048] * 8, 32000, 9)
    a, _, _, _ = run_both(h, [2048] * 8, 32, 512, 9.3, 3.1, [3.1, 6.2, 9.3])
    b, _, _, _ = run_both(h, [2048] * 8, 32, 512, 9.3, 3.1, [3.1, 6.2, 9.3])
    assert_tables_equal(a, b)
