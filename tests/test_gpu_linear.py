"""GPU parity of cwl_chunkwise_lora_linear against the CPU oracle (Sec. III-C / III-D)."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from helpers import TOL_BF16, TOL_F32, gate_matrix, host, rel_err, sample_rows
from paper_2601_21109_amd import binding as B
from paper_2601_21109_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def operands(n, d_in, d_out, r_max, dtype, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    x = torch.randn((n, d_in), generator=g, device=DEV).to(dtype)
    Wm = (torch.randn((d_in, d_out), generator=g, device=DEV) / math.sqrt(d_in)).to(dtype)
    A = (torch.randn((d_in, r_max), generator=g, device=DEV) / math.sqrt(d_in)).to(dtype)
    Bm = (torch.randn((r_max, d_out), generator=g, device=DEV) / math.sqrt(max(r_max, 1))).to(dtype)
    return x, Wm, A, Bm


def run_case(n_seqs, seq_lens, d_in, d_out, ranks, blend_w, dtype, seed, l_min=4, l_max=40,
             alpha=16.0, group_rows=0, packed=False, rows=None, table=None):
    r_max = max(max(ranks), 1) if ranks else 1
    scales = [alpha / r if r > 0 else 0.0 for r in ranks]
    n = int(np.sum(seq_lens))
    x, Wm, A, Bm = operands(n, d_in, d_out, r_max, dtype, seed)
    so, co, cs, cl, ri = table if table is not None else W.random_chunk_table(
        n_seqs, seq_lens, l_min, l_max, len(ranks), seed + 1)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    if packed:
        pw = B.prepack_weights(Wm, A, Bm)
        y = B.chunkwise_lora_linear(x, pw, None, None, ranks, scales, blend_w, sod, tab, rid,
                                    group_rows=group_rows)
    else:
        y = B.chunkwise_lora_linear(x, Wm, A, Bm, ranks, scales, blend_w, sod, tab, rid,
                                    group_rows=group_rows)
    torch.cuda.synchronize()
    ref = O.linear(host(x), host(Wm), host(A), host(Bm), ranks, scales, blend_w, so, co, cs, cl, ri,
                   rows=rows)
    yh = host(y)
    if rows is not None:
        yh = yh[rows]
    return yh, ref, y


def test_fp32_cfg0_shape():
    wl = W.WORKLOADS["cfg0"]
    yh, ref, _ = run_case(1, [128], 256, 256, wl.ladder, wl.blend_w, torch.float32, 1, l_min=8, l_max=64)
    assert rel_err(yh, ref) <= TOL_F32


@pytest.mark.parametrize("n_seqs,seq_lens,d_in,d_out,ranks,w", [
    (1, [77], 100, 72, [3, 12], 2),
    (3, [50, 1, 200], 64, 130, [0, 4, 8, 16], 3),
    (2, [130, 65], 257, 63, [5], 0),
    (1, [64], 16, 16, [0], 2),
    (4, [9, 9, 9, 300], 48, 200, [1, 2, 70], 4),
])
@pytest.mark.parametrize("packed", [False, True])
def test_fp32_shapes(n_seqs, seq_lens, d_in, d_out, ranks, w, packed):
    yh, ref, _ = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.float32, 7, packed=packed)
    assert rel_err(yh, ref) <= TOL_F32


@pytest.mark.parametrize("n_seqs,seq_lens,d_in,d_out,ranks,w", [
    (1, [600], 256, 512, [8, 16, 32, 64], 4),        # ragged row tile
    (3, [300, 41, 700], 512, 520, [8, 16, 32, 64], 4),  # ragged column tile, several sequences
    (2, [256, 256], 1024, 256, [4, 8, 16, 32, 64, 128], 4),   # two stages of the rank part
    (1, [1000], 128, 264, [0, 8, 24, 40], 2),        # rank 0 rung, ranks not multiples of 16
    (1, [511], 192, 1032, [200], 3),                 # single rung, r_max = 200
    (1, [5], 64, 8, [16], 0),                        # tiny
])
@pytest.mark.parametrize("group_rows", [0, 1])
def test_bf16_shapes(n_seqs, seq_lens, d_in, d_out, ranks, w, group_rows):
    yh, ref, _ = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 11, l_min=8,
                          l_max=90, group_rows=group_rows, packed=True)
    assert rel_err(yh, ref) <= TOL_BF16


@pytest.mark.parametrize("d_in,ranks", [(64, [8, 16]), (128, [0, 8, 64]), (192, [100]), (320, [8, 16, 32, 64])])
def test_bf16_more_tiles_than_compute_units(d_in, ranks):
    """297 output tiles of 256 x 256 (ragged in both directions) with very short reduction loops:
    persistent workgroups take one or two tiles each and their loaders cross from one tile into the
    next, and into the rank part, within a few stages."""
    n, d_out = 2100, 8200
    rows = np.unique(np.concatenate([np.arange(0, n, 37), np.arange(250, 262), np.arange(n - 70, n)]))
    yh, ref, _ = run_case(2, [1300, 800], d_in, d_out, ranks, 3, torch.bfloat16, 17, l_min=8, l_max=90,
                          packed=True, rows=rows)
    assert rel_err(yh, ref) <= TOL_BF16


@pytest.mark.parametrize("d_in,ranks,group_rows", [(128, [8, 16, 32, 64], 0), (192, [0, 24, 100], 0),
                                                   (128, [40, 200], 0), (64, [8, 250], 0), (128, [40, 200], 1)])
def test_bf16_tall_inputs(d_in, ranks, group_rows):
    """65536 rows and more (ragged): the shrink runs on 256-row tiles with a rotated walk over the reduction
    dimension, from 192 padded directions up on the persistent kernel with the gate in its epilogue; row
    sample against the oracle."""
    seq_lens = [30000, 35000, 700]
    n = sum(seq_lens)
    rows = np.unique(np.concatenate([np.arange(0, n, 97), np.arange(65530, 65545), np.arange(n - 40, n)]))
    yh, ref, _ = run_case(3, seq_lens, d_in, 264, ranks, 3, torch.bfloat16, 23, l_min=8, l_max=90,
                          packed=True, rows=rows, group_rows=group_rows)
    assert rel_err(yh, ref) <= TOL_BF16


@pytest.mark.parametrize("n_seqs,seq_lens,d_in,d_out,ranks,w", [
    (1, [1], 64, 8, [16], 0),                         # one token, one slice
    (1, [1], 4096, 4096, [8, 16, 32, 64], 4),         # one decode row at the 7B shape
    (8, [1] * 8, 1024, 1032, [8, 16, 32, 64], 4),     # eight one-token sequences, ragged columns
    (3, [9, 1, 7], 512, 72, [0, 4, 70], 3),           # 17 rows, joins inside, padded rank 128, rank-0 rung
    (1, [64], 2048, 264, [8, 64], 2),                 # exactly one row tile of 64
    (2, [40, 25], 704, 520, [200], 4),                # 65 rows: the 128-row tile; 11 stages over several slices
    (4, [32, 32, 32, 32], 4096, 328, [8, 16, 32, 64], 4),   # 128 rows
    (1, [100], 11008, 136, [8, 16, 32, 64], 4),       # long reduction (172 stages)
    (1, [300], 1024, 520, [8, 16, 32, 64], 4),        # three row tiles of 128, ragged
    (3, [200, 12, 300], 512, 264, [0, 24, 100], 3),   # 512 rows: the largest case of this path
])
@pytest.mark.parametrize("packed", [True, False])
def test_bf16_few_rows(n_seqs, seq_lens, d_in, d_out, ranks, w, packed):
    """At most 512 rows: the split-reduction path (partial products + fix-up kernel)."""
    yh, ref, y = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 23, l_min=4, l_max=12,
                          packed=packed)
    assert rel_err(yh, ref) <= TOL_BF16
    _, _, y2 = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 23, l_min=4, l_max=12,
                        packed=packed)
    assert torch.equal(y, y2)                         # slice sums in a fixed order


@pytest.mark.parametrize("n_seqs,seq_lens,d_in,d_out,ranks,w", [
    (1, [1], 4096, 11008, [8, 16, 32, 64], 4),         # one row, wide output (1376 workgroups)
    (1, [1], 8192, 264, [0, 24, 100], 3),              # one row, the longest reduction of the one-row path, padded rank 128
    (1, [1], 11008, 4096, [8, 16, 32, 64], 4),         # one row of a longer reduction: the split-reduction path
    (1, [1], 1344, 8, [200], 0),                       # reduction not a multiple of 512 elements, one column block, padded rank 256
    (1, [2], 4096, 4096, [8, 16, 32, 64], 4),          # two rows of one sequence at the 7B shape
    (2, [2, 1], 4096, 11008, [8, 16, 32, 64], 4),      # three rows, wide output
    (3, [4, 1, 2], 2048, 1032, [4, 8, 200], 3),        # seven rows, padded rank 256, joins with a cross-fade inside
    (1, [8], 4096, 4096, [8, 16, 32, 64], 4),          # eight rows of one sequence: two chunks, a join
    (2, [9, 7], 4096, 4096, [8, 16, 32, 64], 4),       # 16 rows: the last count on 32 x 128 partial-product tiles
    (2, [9, 8], 4096, 4096, [8, 16, 32, 64], 4),       # 17 rows: back on 64 x 64 tiles
    (1, [16], 4096, 8320, [8, 16, 32, 64], 4),         # 16 rows, 66 column tiles of 128: 64 x 64 tiles
])
@pytest.mark.parametrize("packed", [True, False])
def test_bf16_a_handful_of_rows(n_seqs, seq_lens, d_in, d_out, ranks, w, packed):
    """A handful of rows around the one-row path (x A first, then every output column as one dot product over
    [x | uhat] on the vector ALUs; from two rows up, and for reductions beyond 8192 elements, the split-reduction path,
    with tiles of 32 rows x 128 columns up to 16 rows, 8192 columns and a reduction of 4096 elements)."""
    yh, ref, y = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 31, l_min=2, l_max=5,
                          packed=packed)
    assert rel_err(yh, ref) <= TOL_BF16
    _, _, y2 = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 31, l_min=2, l_max=5,
                        packed=packed)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("seed", range(24))
def test_bf16_random_shapes_across_the_launch_plans(seed):
    """Random shapes around the switch points of the launch plan (512 rows, 64 / 128 tiles of 256 x 256,
    slice counts), random ladders and joins, against the oracle."""
    rng = np.random.RandomState(1000 + seed)
    n = int(rng.choice([1, 2, 3, 5, 8, 9, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 700, 1100]))
    d_in = 64 * int(rng.randint(1, 13))
    d_out = 8 * int(rng.randint(1, 90))
    K = int(rng.randint(1, 5))
    ranks = sorted(int(r) for r in rng.choice(np.arange(0, 201), size=K, replace=False))
    n_seqs = int(rng.randint(1, 4))
    cuts = np.sort(rng.randint(0, n + 1, size=n_seqs - 1))
    seq_lens = np.diff(np.concatenate([[0], cuts, [n]])).tolist()
    w = int(rng.randint(0, 5))
    rows = None if n * d_out * d_in <= 6e7 else np.unique(rng.randint(0, n, size=120))
    yh, ref, _ = run_case(n_seqs, seq_lens, d_in, d_out, ranks, w, torch.bfloat16, 2000 + seed, l_min=5, l_max=37,
                          packed=bool(seed % 2), rows=rows)
    assert rel_err(yh, ref) <= TOL_BF16


def test_bf16_few_rows_agree_with_the_large_path():
    """Rows 0..511 of a 513-row call (tiled path) against the same rows as a 512-row call."""
    d_in, d_out, ranks = 1024, 520, [8, 16, 32, 64]
    scales = [16.0 / r for r in ranks]
    x, Wm, A, Bm = operands(513, d_in, d_out, 64, torch.bfloat16, 29)
    pw = B.prepack_weights(Wm, A, Bm)
    ys = []
    for n in (513, 512):
        so, co, cs, cl, ri = W.random_chunk_table(1, [n], 128, 128, len(ranks), 3)
        ri[:] = np.arange(len(ri)) % len(ranks)
        sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
        ys.append(B.chunkwise_lora_linear(x[:n], pw, None, None, ranks, scales, 4, sod, tab, rid)[:512].float())
    torch.cuda.synchronize()
    # both round uhat and y to bf16 once; the sums run in different orders
    assert (ys[0] - ys[1]).abs().max().item() <= 2.0 ** -6 * ys[0].abs().max().item()


@pytest.mark.parametrize("n,d_out", [(1500, 2504), (2000, 3000)])
def test_bf16_mid_sized_grids(n, d_out):
    """60 and 96 tiles of 256 x 256: too few for the persistent kernel, served with 128 x 128 and
    256 x 128 tiles (ragged in both directions, ranks up to two stages of the rank part)."""
    rows = np.unique(np.concatenate([np.arange(0, n, 29), np.arange(250, 262), np.arange(n - 40, n)]))
    yh, ref, _ = run_case(2, [n - 700, 700], 320, d_out, [8, 16, 32, 64, 100], 3, torch.bfloat16, 19, l_min=8,
                          l_max=90, packed=True, rows=rows)
    assert rel_err(yh, ref) <= TOL_BF16


def test_bf16_grouped_rows_give_identical_output():
    args = (3, [300, 41, 700], 512, 520, [8, 16, 32, 64], 4, torch.bfloat16, 5)
    _, _, y0 = run_case(*args, group_rows=0, packed=True, l_min=8, l_max=90)
    _, _, y1 = run_case(*args, group_rows=1, packed=True, l_min=8, l_max=90)
    _, _, y2 = run_case(*args, group_rows=0, packed=False, l_min=8, l_max=90)
    assert torch.equal(y0, y1) and torch.equal(y0, y2)


@pytest.mark.parametrize("dtype,tol", [(torch.float32, TOL_F32), (torch.bfloat16, TOL_BF16)])
def test_special_cases_reduce_to_textbook_lora(dtype, tol):
    n, d_in, d_out, r = 300, 128, 136, 16
    table = (np.array([0, n], np.int32), np.array([0, 1], np.int32), np.array([0], np.int32),
             np.array([n], np.int32), np.array([0], np.int32))
    # one chunk at r_max: y = x W + s (x A) B ; rank 0: y = x W   (float64 library matmul)
    for ranks in ([r], [0]):
        yh, _, _ = run_case(1, [n], d_in, d_out, ranks, 3, dtype, 21, table=table)
        x, Wm, A, Bm = (host(t).astype(np.float64) for t in operands(n, d_in, d_out, max(ranks[0], 1), dtype, 21))
        want = x @ Wm
        if ranks[0]:
            want = want + float(np.float32(16.0 / r)) * (x @ A) @ Bm
        assert rel_err(yh, want) <= tol


def test_uncovered_tokens_and_bad_rank_index_get_base_only():
    n, d_in, d_out = 200, 64, 72
    table = (np.array([0, n], np.int32), np.array([0, 2], np.int32), np.array([0, 100], np.int32),
             np.array([50, 50], np.int32), np.array([0, 9], np.int32))     # rows 50..99 and 150.. uncovered
    x, Wm, A, Bm = operands(n, d_in, d_out, 8, torch.float32, 31)
    sod, tab, rid = B.table_from_host(*table, DEV)
    y = host(B.chunkwise_lora_linear(x, Wm, A, Bm, [8], [2.0], 0, sod, tab, rid))
    xd, Wd, Ad, Bd = (host(t).astype(np.float64) for t in (x, Wm, A, Bm))
    base = xd @ Wd
    full = base + 2.0 * (xd @ Ad) @ Bd
    assert rel_err(y[:50], full[:50]) <= TOL_F32
    assert rel_err(y[50:], base[50:]) <= TOL_F32       # uncovered rows and the chunk with rank_idx 9


@pytest.mark.parametrize("dtype,n,d_in,d_out,ranks", [
    (torch.float32, 300, 256, 264, [4, 8, 16]),
    (torch.bfloat16, 600, 512, 520, [8, 16, 32, 64]),          # mid-size tiles
    (torch.bfloat16, 40, 1024, 264, [8, 16, 32, 64]),          # few-row path
    (torch.bfloat16, 2304, 256, 2048, [0, 24, 100]),           # persistent kernel
])
def test_every_element_is_within_its_own_bound(dtype, n, d_in, d_out, ranks):
    """The tolerance of the other tests divides by max(|ref|, rms(ref)), which is lenient to elements far
    below the RMS (sums with cancellation).  Here every element is held to a bound of its own, without a
    floor: |y - ref| <= rel |ref| + eps * (sum of the magnitudes of the element's terms).  fp32: rel = 1e-5
    and eps = 2^-24 per accumulated term (a plain bound on fp32 summation); bf16: rel = 2^-8, the unit
    roundoff of bf16 (the one rounding of y; attained just above a power of two), and eps = 2^-8 on the
    adapter's terms (the one rounding of the gated shrink output) plus fp32 summation on all terms.  These
    are worst-case bounds of the arithmetic the header states, with no slack added."""
    blend_w, alpha = 3, 16.0
    r_max = max(max(ranks), 1)
    scales = [alpha / r if r else 0.0 for r in ranks]
    x, Wm, A, Bm = operands(n, d_in, d_out, r_max, dtype, 41)
    so, co, cs, cl, ri = W.random_chunk_table(2, [n - n // 3, n // 3], 5, 37, len(ranks), 42)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    y = B.chunkwise_lora_linear(x, B.prepack_weights(Wm, A, Bm), None, None, ranks, scales, blend_w, sod, tab, rid)
    torch.cuda.synchronize()
    xs, Ws, As, Bs = host(x), host(Wm), host(A), host(Bm)
    ref = O.linear(xs, Ws, As, Bs, ranks, scales, blend_w, so, co, cs, cl, ri)
    G = gate_matrix(n, r_max, ranks, scales, blend_w, so, co, cs, cl, ri)
    xd = xs.astype(np.float64)
    mag_base = np.abs(xd) @ np.abs(Ws.astype(np.float64))
    mag_lora = np.abs((xd @ As.astype(np.float64)) * G) @ np.abs(Bs.astype(np.float64))
    assert rel_err(ref, xd @ Ws.astype(np.float64) + ((xd @ As.astype(np.float64)) * G) @ Bs.astype(np.float64)) < 1e-9
    n_terms = d_in + r_max
    if dtype == torch.float32:
        bound = 1e-5 * np.abs(ref) + 2.0 ** -24 * n_terms * (mag_base + mag_lora)
    else:
        bound = 2.0 ** -8 * np.abs(ref) + 2.0 ** -8 * mag_lora + 2.0 ** -24 * n_terms * (mag_base + mag_lora)
    excess = float(np.max(np.abs(host(y).astype(np.float64) - ref) / np.maximum(bound, 1e-300)))
    small = float(np.mean(np.abs(ref) < np.sqrt(np.mean(ref * ref))))
    print(f"per-element error / bound: max {excess:.3f}; {100 * small:.0f} % of the elements lie below the output RMS")
    assert excess <= 1.0, excess
    assert 0.4 < small < 0.9            # most elements are the small ones the floored metric is lenient to


def test_bf16_full_size_q_proj_sampled_rows():
    """The 7B-shaped q_proj at its full size (16384 x 4096 x 4096, ladder {8,16,32,64}), launch
    configuration as benchmarked (packed weights); the oracle checks a row sample."""
    wl = W.WORKLOADS["cfg1"]
    n, d = wl.n_rows, 4096
    x, Wm, A, Bm = W.linear_operands(wl, 0, DEV)
    so, co, cs, cl, ri = W.random_chunk_table(wl.n_seqs, [wl.seq_len] * wl.n_seqs, wl.l_min, wl.l_max,
                                              len(wl.ladder), 99)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    pw = B.prepack_weights(Wm, A, Bm)
    rows = sample_rows(n, cs, cl, wl.blend_w, 96, seed=1, first_chunks=24)
    xs, Ws, As, Bs = host(x), host(Wm), host(A), host(Bm)
    ref = O.linear(xs, Ws, As, Bs, wl.ladder, wl.scales, wl.blend_w, so, co, cs, cl, ri, rows=rows)
    for group_rows in (0, 1):
        y = B.chunkwise_lora_linear(x, pw, None, None, wl.ladder, wl.scales, wl.blend_w, sod, tab, rid,
                                    group_rows=group_rows)
        torch.cuda.synchronize()
        assert rel_err(host(y[torch.from_numpy(rows).to(DEV)]), ref) <= TOL_BF16
        # property that holds at any size: rows are independent, so the first 256 rows of the full
        # launch equal a launch over a prefix of the batch
        if group_rows == 0:
            y_again = B.chunkwise_lora_linear(x, pw, None, None, wl.ladder, wl.scales, wl.blend_w, sod,
                                              tab, rid)
            assert torch.equal(y, y_again)


@pytest.mark.parametrize("dtype,tol", [(torch.float32, TOL_F32), (torch.bfloat16, TOL_BF16)])
@pytest.mark.parametrize("seq_lens", [[40], [300, 212], [2100, 1500, 3000]])
@pytest.mark.parametrize("group_rows", [0, 1])
def test_largest_ladder_and_rank(dtype, tol, seq_lens, group_rows):
    """The limits of the ABI at once: sixteen rungs, the top one at rank 256 (four stages of the rank part in
    the bf16 kernels), on the few-row, the mid-size and the persistent path."""
    ranks = [0] + [16 * k + (8 if k % 2 else 0) for k in range(1, 15)] + [256]
    assert len(ranks) == B.MAX_LADDER and ranks[-1] == B.MAX_RANK and ranks == sorted(ranks)
    n = int(np.sum(seq_lens))
    rows = None if n <= 1000 else np.unique(np.concatenate([np.arange(0, n, 37), np.arange(n - 40, n)]))
    yh, ref, _ = run_case(len(seq_lens), seq_lens, 512, 640, ranks, 5, dtype, 23, l_min=6, l_max=48,
                          group_rows=group_rows, packed=(dtype == torch.bfloat16), rows=rows)
    assert rel_err(yh, ref) <= tol
