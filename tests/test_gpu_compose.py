"""GPU parity of cwl_compose_scores (Sec. III-A: n-gram novelty, positional prior, entropy) against the
CPU oracle: novelty bit-exact, score to fp32 rounding."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2601_21109_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run(h, ids, so, n, window, w_e, w_n, w_p, plen):
    hd = torch.from_numpy(np.asarray(h, np.float32)).to(DEV)
    idd = torch.from_numpy(np.asarray(ids, np.int32)).to(DEV)
    sod = torch.from_numpy(np.asarray(so, np.int32)).to(DEV)
    score, nov = B.compose_scores(hd, idd, sod, n, window, w_e, w_n, w_p, plen)
    torch.cuda.synchronize()
    st, ref, ref_nov = O.compose_scores(h, ids, so, n, window, w_e, w_n, w_p, plen)
    assert st == 0
    assert np.array_equal(nov.cpu().numpy(), ref_nov)
    np.testing.assert_allclose(score.cpu().numpy(), ref, rtol=2e-6, atol=1e-6)
    return ref_nov


@pytest.mark.parametrize("lens,vocab,n,window", [
    ([2048] * 8, 50, 3, 256),            # the 7B-shaped batch, small alphabet so that n-grams repeat
    ([700, 0, 1, 3000, 17], 4, 2, 64),   # ragged, empty and one-token sequences, blocks straddling joins
    ([5000], 3, 8, 4096),                # longest n-gram and window
    ([300, 300], 2, 1, 0),               # no look-back at all
    ([1000], 1000000, 4, 100),           # practically all new
    ([513], 2, 5, 7),
])
def test_compose_matches_oracle(lens, vocab, n, window):
    rng = np.random.RandomState(len(lens) * 31 + n)
    N = int(np.sum(lens))
    h = (rng.rand(N) * 10).astype(np.float32)
    ids = rng.randint(0, vocab, size=N).astype(np.int32)
    so = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    nov = run(h, ids, so, n, window, 1.0, 2.5, 0.75, 300.0)
    assert 0 < nov.sum() <= N


def test_rows_outside_sequences_and_in_place():
    rng = np.random.RandomState(1)
    h = (rng.rand(600) * 3).astype(np.float32)
    ids = rng.randint(0, 3, 600).astype(np.int32)
    run(h, ids, [50, 300, 520], 2, 30, 0.5, 1.0, 1.0, 64.0)
    hd = torch.from_numpy(h).to(DEV)
    score, _ = B.compose_scores(hd, torch.from_numpy(ids).to(DEV), torch.tensor([0, 600], dtype=torch.int32, device=DEV),
                                2, 30, 0.5, 1.0, 1.0, 64.0, out=hd)
    torch.cuda.synchronize()
    _, ref, _ = O.compose_scores(h, ids, [0, 600], 2, 30, 0.5, 1.0, 1.0, 64.0)
    np.testing.assert_allclose(score.cpu().numpy(), ref, rtol=2e-6, atol=1e-6)
    empty, nov = B.compose_scores(torch.empty(0, device=DEV), torch.empty(0, dtype=torch.int32, device=DEV),
                                  torch.zeros(1, dtype=torch.int32, device=DEV), 2, 30)
    assert empty.numel() == 0 and nov.numel() == 0


def test_composite_score_drives_the_chunker():
    """The composite score goes through cwl_partition_chunks like the entropy does: table from the device's
    composite scores equals the oracle's table from the same scores."""
    rng = np.random.RandomState(4)
    T, n_seqs = 1500, 3
    h = (rng.choice([1.0, 5.0, 9.0], size=(n_seqs * T // 50,)).repeat(50) + rng.rand(n_seqs * T) * 0.3).astype(np.float32)
    ids = rng.randint(0, 6, n_seqs * T).astype(np.int32)
    so = np.arange(n_seqs + 1, dtype=np.int32) * T
    hd, idd, sod = (torch.from_numpy(a).to(DEV) for a in (h, ids, so))
    score, _ = B.compose_scores(hd, idd, sod, 3, 128, 1.0, 2.0, 1.0, 200.0)
    tab = B.partition_chunks(score, sod, 16, 128, 9.0, 3.0)
    torch.cuda.synchronize()
    q, _ = O.quantise(score.cpu().numpy())
    st, ref = O.partition(q, so, 16, 128, O.quantise_threshold(9.0), O.quantise_threshold(3.0))
    assert st == 0
    n = int(tab["chunk_offsets"][-1].item())
    assert n == len(ref["chunk_start"])
    assert np.array_equal(tab["chunk_start"][:n].cpu().numpy(), ref["chunk_start"])
    assert np.array_equal(tab["chunk_sum"][:n].cpu().numpy(), ref["chunk_sum"])
