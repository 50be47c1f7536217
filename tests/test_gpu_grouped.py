"""GPU parity of the grouped calls (projections that share x: q/k/v, gate/up; Sec. III-C, III-F) against
the CPU oracle, which is called once per projection: every projection must come out as the plain layer on
the prefixes of its own factors."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import TOL_BF16, TOL_F32, host, rel_err, sample_rows
from paper_2601_21109_amd import binding as B
from paper_2601_21109_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def group_operands(n, d_in, d_outs, r_max, dtype, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    mk = lambda shape, std: (torch.randn(shape, generator=g, device=DEV) * std).to(dtype)
    x = mk((n, d_in), 1.0)
    Ws = [mk((d_in, n_out), d_in ** -0.5) for n_out in d_outs]
    As = [mk((d_in, r_max), d_in ** -0.5) for _ in d_outs]
    Bs = [mk((r_max, n_out), r_max ** -0.5) for n_out in d_outs]
    return x, Ws, As, Bs


def check_against_oracle(y, pg, x, Ws, As, Bs, ranks, scales, blend_w, table, rows, tol):
    so, co, cs, cl, ri = table
    xs = host(x if rows is None else x[torch.from_numpy(rows).to(DEV)])
    worst = 0.0
    for yp, Wp, Ap, Bp in zip(pg.split(y), Ws, As, Bs):
        ref = O.linear(xs, host(Wp), host(Ap), host(Bp), ranks, scales, blend_w, so, co, cs, cl, ri, rows=rows,
                       x_compact=rows is not None)
        got = host(yp if rows is None else yp[torch.from_numpy(rows).to(DEV)])
        worst = max(worst, rel_err(got, ref))
    assert worst <= tol, worst


@pytest.mark.parametrize("seq_lens,d_in,d_outs,ranks,w,dtype,tol", [
    ([40], 512, [264, 72, 136], [8, 16, 32, 64], 3, torch.bfloat16, TOL_BF16),            # few-row path, three projections
    ([300, 100], 256, [256, 512], [4, 8, 16, 32, 64, 128], 4, torch.bfloat16, TOL_BF16),   # few-row path, rank 128 x 2
    ([1], 1024, [1024, 1024, 1024], [8, 16, 32, 64], 4, torch.bfloat16, TOL_BF16),         # one decode row
    ([1], 4096, [264, 8, 4096, 72], [0, 24, 100], 0, torch.bfloat16, TOL_BF16),            # one row, four projections, padded rank 128
    ([3, 2], 1024, [264, 8, 72], [0, 24, 100], 2, torch.bfloat16, TOL_BF16),               # five rows, three projections whose columns are not multiples of 16
    ([7, 6], 11008, [136, 520], [8, 16, 32, 64], 4, torch.bfloat16, TOL_BF16),             # thirteen rows, long reduction
    ([700, 500], 256, [520, 264], [0, 24, 100], 3, torch.bfloat16, TOL_BF16),              # mid-size tiles, padded rank 128
    ([2100, 900], 192, [1032, 512, 2056], [8, 16, 32, 64], 4, torch.bfloat16, TOL_BF16),   # persistent kernel per projection
    ([900, 400], 128, [256, 264, 8, 64, 72], [200], 2, torch.bfloat16, TOL_BF16),          # five adapters of 256 padded directions: five shrink passes
    ([40000, 25637], 128, [72, 8, 136], [8, 16, 32, 64], 3, torch.bfloat16, TOL_BF16),     # tall: one shrink of 192 directions on the persistent kernel (ragged rows and columns)
    ([65536], 192, [264, 64, 40], [0, 24, 100], 4, torch.bfloat16, TOL_BF16),              # tall: 384 directions, two column tiles, period 128
    ([77, 50], 100, [72, 33, 5], [3, 12], 2, torch.float32, TOL_F32),                      # fp32
    ([600], 64, [130, 70], [0, 4, 8, 16], 3, torch.float32, TOL_F32),
])
def test_grouped_projections_match_the_oracle_per_projection(seq_lens, d_in, d_outs, ranks, w, dtype, tol):
    n, r_max = int(np.sum(seq_lens)), max(max(ranks), 1)
    scales = [16.0 / r if r else 0.0 for r in ranks]
    x, Ws, As, Bs = group_operands(n, d_in, d_outs, r_max, dtype, 5)
    table = W.random_chunk_table(len(seq_lens), seq_lens, 4, 37, len(ranks), 6)
    sod, tab, rid = B.table_from_host(*table, DEV)
    pg = B.prepack_weights_grouped(Ws, As, Bs)
    y = B.chunkwise_lora_linear_grouped(x, pg, ranks, scales, w, sod, tab, rid)
    torch.cuda.synchronize()
    rows = None if n * d_in * sum(d_outs) <= 2e8 else np.unique(np.concatenate([np.arange(0, n, 31), [n - 1]]))
    check_against_oracle(y, pg, x, Ws, As, Bs, ranks, scales, w, table, rows, tol)
    # every projection also agrees with its own single-projection call; the sums may run in another
    # order (on tall inputs the grouped shrink is another kernel), so in bf16 an entry of the shrink
    # output and then the output element itself can each land on the neighbouring value: two units
    # of 2^-8 .. 2^-7 relative
    for yp, Wp, Ap, Bp in zip(pg.split(y), Ws, As, Bs):
        y1 = B.chunkwise_lora_linear(x, B.prepack_weights(Wp, Ap, Bp), None, None, ranks, scales, w, sod, tab, rid)
        assert rel_err(host(yp), host(y1)) <= (2.0 ** -6 if dtype == torch.bfloat16 else 1e-5)
    y2 = B.chunkwise_lora_linear_grouped(x, pg, ranks, scales, w, sod, tab, rid)
    assert torch.equal(y, y2)


def test_grouped_gated_rows_of_a_decode_step():
    """64 decode rows with their own gate entries through q/k/v at once, against the oracle's gated layer."""
    n, d_in, d_outs, ranks = 64, 1024, [1024, 256, 264], [8, 16, 32, 64]
    scales = [16.0 / r for r in ranks]
    x, Ws, As, Bs = group_operands(n, d_in, d_outs, 64, torch.bfloat16, 9)
    rng = np.random.RandomState(4)
    k_cur, k_prev = rng.randint(0, 4, n), rng.randint(0, 4, n)
    lam = rng.choice([1.0, 0.2, 0.6], size=n).astype(np.float32)
    gate = np.zeros((n, 4), np.int32)
    g_cur = (lam * np.asarray(scales, np.float32)[k_cur]).astype(np.float32)
    g_prev = ((1 - lam) * np.asarray(scales, np.float32)[k_prev]).astype(np.float32)
    gate[:, 0], gate[:, 1] = np.asarray(ranks)[k_cur], np.where(lam < 1, np.asarray(ranks)[k_prev], 0)
    gate[:, 2], gate[:, 3] = g_cur.view(np.int32), np.where(lam < 1, g_prev, 0).astype(np.float32).view(np.int32)
    pg = B.prepack_weights_grouped(Ws, As, Bs)
    y = B.gated_lora_linear_grouped(x, pg, torch.from_numpy(gate).to(DEV), ranks, scales)
    torch.cuda.synchronize()
    gf = gate.view(np.float32)
    for yp, Wp, Ap, Bp in zip(pg.split(y), Ws, As, Bs):
        ref = O.gated_linear(host(x), host(Wp), host(Ap), host(Bp), gate[:, 0], gf[:, 2], gate[:, 1], gf[:, 3])
        assert rel_err(host(yp), ref) <= TOL_BF16


@pytest.mark.parametrize("projs", [(0, 1, 2), (4, 5)])
def test_grouped_full_size_decoder_layer(projs):
    """q/k/v (3 x 4096 -> 4096) and gate/up (2 x 4096 -> 11008) of the 32 x 2048 workload with the ladder
    {4, .., 128} at full size: each projection on its own rungs, row sample against the oracle."""
    wl = W.WORKLOADS["cfg3"]
    ops = [W.linear_operands(wl, p, DEV) for p in projs]
    x = ops[0][0]                                      # the projections of a group read the same x
    Ws, As, Bs = [o[1] for o in ops], [o[2] for o in ops], [o[3] for o in ops]
    table = W.random_chunk_table(wl.n_seqs, [wl.seq_len] * wl.n_seqs, wl.l_min, wl.l_max, len(wl.ladder), 77)
    sod, tab, rid = B.table_from_host(*table, DEV)
    pg = B.prepack_weights_grouped(Ws, As, Bs)
    del ops
    y = B.chunkwise_lora_linear_grouped(x, pg, wl.ladder, wl.scales, wl.blend_w, sod, tab, rid)
    torch.cuda.synchronize()
    rows = sample_rows(wl.n_rows, table[2], table[3], wl.blend_w, 24, seed=3, first_chunks=8)
    check_against_oracle(y, pg, x, Ws, As, Bs, wl.ladder, wl.scales, wl.blend_w, table, rows, TOL_BF16)
