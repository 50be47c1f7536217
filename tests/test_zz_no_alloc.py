"""The entry point that allocates nothing: cwl_chunkwise_lora_linear_packed_static keeps its scratch
memory in a static device array of the library.  Called through the C ABI (ctypes on the .so) and
compared, bit for bit, with cwl_chunkwise_lora_linear_packed (the same kernels on a caller's
workspace) and, to the bf16 tolerance, with the oracle; two calls in a row, the second on a smaller
input, so that whatever the first call left in the array would show."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as O
from helpers import TOL_BF16, host, rel_err
from paper_2601_21109_amd import binding as B
from paper_2601_21109_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _operands(n, d_in, d_out, r_max, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    mk = lambda shape, std: (torch.randn(shape, generator=g, device=DEV) * std).to(torch.bfloat16)
    return mk((n, d_in), 1.0), mk((d_in, d_out), d_in ** -0.5), mk((d_in, r_max), d_in ** -0.5), \
        mk((r_max, d_out), r_max ** -0.5)


def _both(L, n_seqs, seq_lens, d_in, d_out, ranks, blend_w, seed):
    """One case through both entry points; returns (y_static, y_workspace, oracle rows, row sample)."""
    n, r_max = int(np.sum(seq_lens)), max(ranks)
    scales = [16.0 / r if r else 0.0 for r in ranks]
    x, Wm, A, Bm = _operands(n, d_in, d_out, r_max, seed)
    so, co, cs, cl, ri = W.random_chunk_table(n_seqs, seq_lens, 8, 90, len(ranks), seed + 1)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    pw = B.prepack_weights(Wm, A, Bm)
    y_ws = B.chunkwise_lora_linear(x, pw, None, None, ranks, scales, blend_w, sod, tab, rid)
    y_st = torch.empty_like(y_ws)
    d = B._desc_for(x, d_out, r_max, ranks, scales, blend_w, y_st)
    assert L.cwl_linear_packed_workspace_bytes(d.ref()) <= B.STATIC_SCRATCH_BYTES
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = L.cwl_chunkwise_lora_linear_packed_static(
        d.ref(), B._ptr(x), B._ptr(pw.blob), B._ptr(sod), n_seqs, B._ptr(tab["chunk_offsets"]),
        B._ptr(tab["chunk_start"]), B._ptr(tab["chunk_len"]), B._ptr(rid), tab["cap"], B._ptr(y_st),
        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing taken from torch's allocator either
    rows = np.unique(np.concatenate([np.arange(0, n, max(n // 150, 1)), np.arange(max(n - 20, 0), n)]))
    ref = O.linear(host(x), host(Wm), host(A), host(Bm), ranks, scales, blend_w, so, co, cs, cl, ri, rows=rows)
    return y_st, y_ws, ref, rows


@pytest.mark.parametrize("first,second", [
    # tiled path (gate table, shrink, persistent main kernel), then fewer rows on the same path
    ((3, [900, 300, 1400], 512, 1032, [8, 16, 32, 64], 4), (2, [700, 500], 512, 520, [8, 16, 32, 64], 4)),
    # few-row path (partial products in the scratch array), then a smaller few-row call
    ((2, [200, 180], 1024, 520, [8, 16, 32, 64], 4), (1, [37], 1024, 264, [8, 16, 32, 64], 2)),
    # large then decode-sized: the second call's layout of the array differs from the first's
    ((1, [3000], 256, 768, [0, 24, 100], 3), (4, [1, 1, 1, 1], 256, 768, [0, 24, 100], 3)),
])
def test_static_scratch_entry_matches_workspace_entry(first, second):
    L = B.lib()
    for i, case in enumerate((first, second)):
        y_st, y_ws, ref, rows = _both(L, *case, seed=40 + i)
        assert torch.equal(y_st, y_ws)                       # same kernels, same bits
        assert rel_err(host(y_st)[rows], ref) <= TOL_BF16


def test_static_scratch_rejects_what_does_not_fit():
    L = B.lib()
    n, d = 200000, 64                                        # uhat alone: 200000 x 64 x 2 bytes > 16 MiB
    x = torch.empty((1, d), dtype=torch.bfloat16, device=DEV)
    y = torch.empty((1, 64), dtype=torch.bfloat16, device=DEV)
    dsc = B._desc_for(x, 64, 64, [64], [1.0], 0, y)
    dsc.c.n_rows = n
    assert L.cwl_linear_packed_workspace_bytes(dsc.ref()) > B.STATIC_SCRATCH_BYTES
    P = ctypes.c_void_p
    st = L.cwl_chunkwise_lora_linear_packed_static(dsc.ref(), P(0x10000), P(0x20000), P(0x1000), 1, P(0x1000),
                                                   P(0x1000), P(0x1000), P(0x1000), 8, P(0x30000), None)
    assert st == B.ERR_CAPACITY
