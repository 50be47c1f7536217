"""End-to-end GPU parity of the whole hot path (score -> partition -> select -> linear) against
the CPU oracle, stage by stage and end to end."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import (TOL_BF16, TOL_F32, assert_tables_equal, entropy_err, gpu_table_to_host, host,
                     oracle_table, rel_err, sample_rows)
from paper_2601_21109_amd import binding as B
from paper_2601_21109_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_path(wl, logits, x, Wm, A, Bm, sod, group_rows=0):
    h = B.score_tokens(logits)
    table = B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta())
    ri = B.select_ranks(table, wl.taus(), len(wl.ladder))
    y = B.chunkwise_lora_linear(x, Wm, A, Bm, wl.ladder, wl.scales, wl.blend_w, sod, table, ri,
                                group_rows=group_rows)
    torch.cuda.synchronize()
    return h, table, ri, y


def test_cfg0_end_to_end():
    wl = W.WORKLOADS["cfg0"]
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(DEV)
    logits = W.logits(wl, DEV)
    x, Wm, A, Bm = W.linear_operands(wl, 0, DEV)
    h, table, ri, y = gpu_path(wl, logits, x, Wm, A, Bm, sod)

    # stage 1: entropy
    h_ref = O.entropy(host(logits))
    assert entropy_err(host(h), h_ref, wl.vocab) <= TOL_F32
    # stages 2-3, stage-wise: the oracle starts from the device's own fp32 scores -> bit-exact
    gpu = gpu_table_to_host(table, ri)
    ref = oracle_table(host(h), so, wl)
    assert gpu["status"] == 0
    assert_tables_equal(gpu, ref)
    assert len(set(ref["rank_idx"].tolist())) == 3          # all three rungs are exercised
    # end to end: the oracle's own double-precision scores; codes may differ by one unit on a few
    # tokens, and only such a flip may change the table
    e2e = oracle_table(h_ref.astype(np.float32), so, wl)
    dq = np.abs(e2e["q"].astype(np.int64) - ref["q"].astype(np.int64))
    assert dq.max() <= 1
    if dq.max() == 0:
        assert_tables_equal(gpu, e2e)
    # stage 4
    y_ref = O.linear(host(x), host(Wm), host(A), host(Bm), wl.ladder, wl.scales, wl.blend_w, so,
                     ref["chunk_offsets"], ref["chunk_start"], ref["chunk_len"], ref["rank_idx"])
    assert rel_err(host(y), y_ref) <= TOL_F32


def test_bf16_small_end_to_end():
    wl = W.scaled(W.WORKLOADS["cfg1"], n_seqs=3, seq_len=700, vocab=4096,
                  projections=[("proj", 256, 384)], name="cfg1-small")
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(DEV)
    logits = W.logits(wl, DEV)
    x, Wm, A, Bm = W.linear_operands(wl, 0, DEV)
    for group_rows in (0, 1):
        h, table, ri, y = gpu_path(wl, logits, x, Wm, A, Bm, sod, group_rows)
        assert entropy_err(host(h), O.entropy(host(logits)), wl.vocab) <= TOL_F32
        gpu = gpu_table_to_host(table, ri)
        ref = oracle_table(host(h), so, wl)
        assert_tables_equal(gpu, ref)
        y_ref = O.linear(host(x), host(Wm), host(A), host(Bm), wl.ladder, wl.scales, wl.blend_w, so,
                         ref["chunk_offsets"], ref["chunk_start"], ref["chunk_len"], ref["rank_idx"])
        assert rel_err(host(y), y_ref) <= TOL_BF16


def test_cfg1_full_size_scoring_and_table():
    """The 16384 x 32000 bf16 logits of the 7B-shaped workload at full size: entropy on a row
    sample, chunk table and rungs in full (stage-wise, bit-exact)."""
    wl = W.WORKLOADS["cfg1"]
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(DEV)
    logits = W.logits(wl, DEV)
    h = B.score_tokens(logits)
    table = B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta())
    ri = B.select_ranks(table, wl.taus(), len(wl.ladder))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, wl.n_rows, 61), [wl.n_rows - 1]]))
    sub = host(logits[torch.from_numpy(rows).to(DEV)])
    assert entropy_err(host(h)[rows], O.entropy(sub), wl.vocab) <= TOL_F32
    gpu = gpu_table_to_host(table, ri)
    ref = oracle_table(host(h), so, wl)
    assert gpu["status"] == 0
    assert_tables_equal(gpu, ref)
    lens = gpu["chunk_len"]
    assert lens.min() >= wl.l_min and lens.max() <= wl.l_max and int(lens.sum()) == wl.n_rows
    assert len(set(gpu["rank_idx"].tolist())) >= 3


@pytest.mark.parametrize("n_seqs,seq_len,d_in,d_out,group_rows", [
    (3, 700, 256, 512, 0),        # 128 x 128 tiles, split shrink
    (8, 2048, 512, 1024, 0),      # persistent 256 x 256 kernel
    (2, 200, 256, 320, 0),        # few-row path (partial products + fix-up)
    (8, 2048, 512, 1024, 1),      # rows grouped by rank
    (8, 2048, 512, 1024, 2),      # two-phase form: x A in the chunker's launch, gate + persistent kernel
    (3, 700, 256, 512, 2),        # two-phase form: split shrink behind the chunker
    (2, 200, 256, 320, 2),        # two-phase form on the few-row path (empty first phase)
])
def test_whole_step_replays_from_a_hip_graph(n_seqs, seq_len, d_in, d_out, group_rows):
    """The four calls only enqueue kernels on the caller's stream: a whole step captured once must give, on every
    replay (with eager work and synchronisations in between), the bits of the eager step on the same inputs."""
    vocab, r_max = 2000, 32
    ranks, scales = [8, 16, 32], [2.0, 1.0, 0.5]
    lnv = float(np.log(vocab))
    theta, delta, taus = 0.9 * lnv, 0.25 * lnv, [0.35 * lnv, 0.7 * lnv]
    N = n_seqs * seq_len
    sod = torch.arange(0, N + 1, seq_len, dtype=torch.int32, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(3)
    mk = lambda *s: (torch.randn(s, generator=g, device=DEV) / s[0] ** 0.5).to(torch.bfloat16)
    packed = B.prepack_weights(mk(d_in, d_out), mk(d_in, r_max), mk(r_max, d_out))
    logits = torch.empty((N, vocab), dtype=torch.bfloat16, device=DEV)
    x = torch.empty((N, d_in), dtype=torch.bfloat16, device=DEV)
    h = torch.empty(N, dtype=torch.float32, device=DEV)
    y = torch.empty((N, d_out), dtype=torch.bfloat16, device=DEV)
    ws = B.linear_workspace((N, d_in), torch.bfloat16, d_out, r_max, ranks, scales, 3, DEV)

    def new_inputs(i):
        gi = torch.Generator(device=DEV).manual_seed(40 + i)
        # spans of 50 tokens at one of three temperatures: low, middle and high entropy
        sigma = torch.tensor([0.5, 2.5, 7.0], device=DEV)[torch.randint(0, 3, (N // 50 + 1,), generator=gi, device=DEV)]
        sigma = sigma.repeat_interleave(50)[:N, None]
        logits.copy_((torch.randn((N, vocab), generator=gi, device=DEV) * sigma).to(torch.bfloat16))
        x.copy_(torch.randn((N, d_in), generator=gi, device=DEV).to(torch.bfloat16))

    new_inputs(0)
    table = B.partition_chunks(B.score_tokens(logits, out=h), sod, 8, 64, theta, delta)
    ri = B.select_ranks(table, taus, 3)

    two_phase = group_rows == 2          # (third setting of the parameter: the step in its two-phase form)
    u = B.lora_shrink(x, packed, ranks, scales, 3) if two_phase else None

    def step():
        B.score_tokens(logits, out=h)
        if two_phase:
            B.schedule_chunks(h, sod, 8, 64, theta, delta, taus, 3, out=table, rank_idx=ri,
                              shrink=(x, packed, ranks, scales, 3, u))
            B.chunkwise_lora_linear_shrunk(x, packed, u, ranks, scales, 3, sod, table, ri, out=y, workspace=ws)
            return
        B.partition_chunks(h, sod, 8, 64, theta, delta, out=table)
        B.select_ranks(table, taus, 3, out=ri)
        B.chunkwise_lora_linear(x, packed, None, None, ranks, scales, 3, sod, table, ri, out=y, group_rows=group_rows,
                                workspace=ws)

    eager = []
    for i in range(4):
        new_inputs(i)
        step()
        torch.cuda.synchronize()
        eager.append((y.clone(), table["chunk_start"].clone(), ri.clone(), table["chunk_offsets"].clone()))
    assert len({int(e[3][-1].item()) for e in eager}) > 1      # the inputs do lead to different chunk tables
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                 # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in (2, 0, 3, 1):
        new_inputs(i)
        graph.replay()
        torch.cuda.synchronize()
        assert int(table["status_word"].item()) == 0
        assert torch.equal(table["chunk_offsets"], eager[i][3]), i
        n = int(eager[i][3][-1].item())
        assert torch.equal(table["chunk_start"][:n], eager[i][1][:n]) and torch.equal(ri[:n], eager[i][2][:n]), i
        assert torch.equal(y, eager[i][0]), i
