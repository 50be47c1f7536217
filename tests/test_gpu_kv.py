"""GPU parity of the chunk-level KV-cache policy (cwl_kv_quantise_chunks, cwl_kv_dequantise; Sec. III-E /
IV-F) against the CPU oracle: slots, pool sizes, INT8 codes, scales and kept rows bit for bit."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import host
from paper_2601_21109_amd import binding as B
from paper_2601_21109_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_kv(n, width, seed, spread=6.0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    mag = torch.exp((torch.rand((n, 1), generator=g, device=DEV) * 2 - 1) * spread)
    return (torch.randn((n, width), generator=g, device=DEV) * mag).to(torch.bfloat16)


def compare(kv, H, D, k_keep, so, co, cs, cl, ri, **caps):
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    cache = B.kv_quantise_chunks(kv, H, D, k_keep, tab, rid, **caps)
    back = B.kv_dequantise(cache, kv.shape[0])
    torch.cuda.synchronize()
    ref = O.kv_quantise(host(kv), H, D, cs, cl, ri, k_keep)
    nq, nf = ref["codes"].shape[0], ref["kept"].shape[0]
    assert cache["counts"].cpu().tolist() == [nq, nf]
    return cache, back, ref, nq, nf


def assert_cache_equal(cache, back, ref, nq, nf, kv, H, D):
    assert int(cache["status_word"].item()) == 0
    assert cache["slot"].cpu().numpy()[:kv.shape[0]].tolist() == ref["slot"].tolist()
    assert np.array_equal(cache["q_codes"].cpu().numpy()[:nq], ref["codes"])
    assert np.array_equal(cache["q_scale"].cpu().numpy()[:nq].view(np.uint32), ref["scale"].view(np.uint32))
    assert np.array_equal(host(cache["f_pool"])[:nf].view(np.uint32), ref["kept"].view(np.uint32))
    want = O.kv_dequantise(ref["slot"], ref["codes"], ref["scale"], ref["kept"], H, D)
    assert np.array_equal(host(back).view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("H,D", [(2, 64), (4, 128), (32, 128), (8, 256), (1, 512), (3, 32), (16, 512), (5, 64)])
@pytest.mark.parametrize("k_keep", [0, 2, 9])
def test_shapes_and_policies(H, D, k_keep):
    seq_lens = [300, 1, 77, 523]
    n = sum(seq_lens)
    kv = make_kv(n, H * D, 100 + H)
    so, co, cs, cl, ri = W.random_chunk_table(len(seq_lens), seq_lens, 4, 40, 4, 7 + k_keep)
    cache, back, ref, nq, nf = compare(kv, H, D, k_keep, so, co, cs, cl, ri)
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)
    if k_keep == 0:
        assert nq == 0
    if k_keep == 9:
        assert nf == 0


def test_rows_that_no_chunk_covers_and_rungs_outside_the_ladder():
    n, H, D = 400, 2, 64
    kv = make_kv(n, H * D, 3)
    # chunks tile rows 16 .. 367 only; two chunks carry a rung that is no index of the ladder
    cs = np.arange(16, 368, 32, dtype=np.int32)
    cl = np.full(len(cs), 32, dtype=np.int32)
    ri = (np.arange(len(cs)) % 3).astype(np.int32)
    ri[2], ri[5] = -1, 77
    so, co = np.array([0, n], np.int32), np.array([0, len(cs)], np.int32)
    cache, back, ref, nq, nf = compare(kv, H, D, 2, so, co, cs, cl, ri)
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)
    slot = cache["slot"].cpu().numpy()
    assert np.all(slot[:16] == B.KV_SLOT_ABSENT) and np.all(slot[368:] == B.KV_SLOT_ABSENT)
    assert np.all(host(back)[:16] == 0)


def test_non_finite_and_zero_heads():
    n, H, D = 64, 2, 64
    kv = make_kv(n, H * D, 5, spread=1.0)
    kv[0, :64] = 0.0
    kv[1, 3] = float("nan")
    kv[2, 70] = float("inf")
    kv[3, 5] = float("-inf")
    kv[3, 6] = float("nan")
    so, co = np.array([0, n], np.int32), np.array([0, 2], np.int32)
    cs, cl, ri = np.array([0, 32], np.int32), np.array([32, 32], np.int32), np.array([0, 1], np.int32)
    cache, back, ref, nq, nf = compare(kv, H, D, 1, so, co, cs, cl, ri)
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)


def test_strided_rows():
    n, H, D = 200, 4, 64
    big = make_kv(n, 2 * H * D, 9)
    kv = big[:, :H * D]                      # leading dimension twice the row width
    so, co, cs, cl, ri = W.random_chunk_table(2, [120, 80], 4, 40, 3, 11)
    cache, back, ref, nq, nf = compare(kv, H, D, 1, so, co, cs, cl, ri)
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)


def test_pools_too_small():
    """Rows beyond a pool's capacity are not cached and the status word says so; every other row is as before."""
    n, H, D = 500, 2, 64
    kv = make_kv(n, H * D, 13)
    so, co, cs, cl, ri = W.random_chunk_table(1, [n], 4, 40, 4, 17)
    ref = O.kv_quantise(host(kv), H, D, cs, cl, ri, 2)
    nq, nf = ref["codes"].shape[0], ref["kept"].shape[0]
    assert nq > 40 and nf > 40
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    cache = B.kv_quantise_chunks(kv, H, D, 2, tab, rid, cap_q=nq - 30, cap_f=nf - 7)
    torch.cuda.synchronize()
    assert int(cache["status_word"].item()) == B.STATUS_CAPACITY
    assert cache["counts"].cpu().tolist() == [nq, nf]
    slot = cache["slot"].cpu().numpy()
    want = ref["slot"].copy()
    want[(want >= nq - 30)] = B.KV_SLOT_ABSENT
    want[(want < 0) & (want != B.KV_SLOT_ABSENT) & (-1 - want >= nf - 7)] = B.KV_SLOT_ABSENT
    assert slot.tolist() == want.tolist()
    assert np.array_equal(cache["q_codes"].cpu().numpy()[:nq - 30], ref["codes"][:nq - 30])
    assert np.array_equal(host(cache["f_pool"])[:nf - 7], ref["kept"][:nf - 7])
    # the same buffers again with room for everything: the status word is cleared by the call
    cache2 = B.kv_quantise_chunks(kv, H, D, 2, tab, rid)
    torch.cuda.synchronize()
    assert int(cache2["status_word"].item()) == 0


def test_workload_size_on_the_chunkers_table():
    """The benchmarked shape: 16384 rows of 32 heads x 128 (one of K / V of a 7B layer), the chunk table and the
    rungs from the library's own chunker and selector on the workload's scores; every row against the oracle."""
    wl = W.WORKLOADS["cfg1"]
    n, H, D = wl.n_rows, 32, 128
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(DEV)
    sig = torch.from_numpy(np.asarray(W.token_sigmas(wl), dtype=np.float32)).to(DEV)
    # scores at the workload's three entropy levels without materialising 1 GB of logits
    h = (torch.log(torch.tensor(float(wl.vocab))) * torch.where(sig < 1, 0.988, torch.where(sig < 4, 0.81, 0.20))).float().to(DEV)
    tab, ri = B.schedule_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), len(wl.ladder))
    kv = make_kv(n, H * D, 21, spread=2.0)
    cache = B.kv_quantise_chunks(kv, H, D, 2, tab, ri)
    back = B.kv_dequantise(cache, n)
    torch.cuda.synchronize()
    nc = int(tab["chunk_offsets"][-1].item())
    ref = O.kv_quantise(host(kv), H, D, tab["chunk_start"][:nc].cpu().numpy(), tab["chunk_len"][:nc].cpu().numpy(),
                        ri[:nc].cpu().numpy(), 2)
    nq, nf = ref["codes"].shape[0], ref["kept"].shape[0]
    assert nq > 0 and nf > 0 and nq + nf == n
    assert cache["counts"].cpu().tolist() == [nq, nf]
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)


def test_table_of_more_than_4096_chunks():
    """Above 4096 chunks the plan and the slots are two launches instead of one; same results, and the status
    word says when a pool is too small on this path too."""
    n, H, D = 12000, 2, 64
    kv = make_kv(n, H * D, 33)
    so, co, cs, cl, ri = W.random_chunk_table(3, [5000, 1, 6999], 1, 2, 4, 29)
    assert len(cs) > 4096
    cache, back, ref, nq, nf = compare(kv, H, D, 2, so, co, cs, cl, ri)
    assert_cache_equal(cache, back, ref, nq, nf, kv, H, D)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    small = B.kv_quantise_chunks(kv, H, D, 2, tab, rid, cap_q=nq - 1, cap_f=nf)
    torch.cuda.synchronize()
    assert int(small["status_word"].item()) == B.STATUS_CAPACITY
    assert small["counts"].cpu().tolist() == [nq, nf]


def test_argument_errors():
    kv = make_kv(64, 128, 1)
    so, co, cs, cl, ri = W.random_chunk_table(1, [64], 4, 40, 3, 1)
    sod, tab, rid = B.table_from_host(so, co, cs, cl, ri, DEV)
    with pytest.raises(B.CwlError) as e:
        B.kv_quantise_chunks(kv, 8, 16, 1, tab, rid)          # head_dim 16: fewer than four lanes per head
    assert e.value.status == B.ERR_UNSUPPORTED
    with pytest.raises(B.CwlError) as e:
        B.kv_quantise_chunks(kv, 1, 128, -1, tab, rid)
    assert e.value.status == B.ERR_INVALID_ARG


def test_degenerate_tables():
    """No rows; no chunks (every row absent); a table whose capacity cuts the chunk list short."""
    H, D = 2, 64
    kv0 = torch.empty((0, H * D), dtype=torch.bfloat16, device=DEV)
    sod, tab, rid = B.table_from_host(np.array([0, 0], np.int32), np.array([0, 0], np.int32), np.zeros(0, np.int32),
                                      np.zeros(0, np.int32), np.zeros(0, np.int32), DEV)
    c0 = B.kv_quantise_chunks(kv0, H, D, 1, tab, rid)
    torch.cuda.synchronize()
    assert c0["counts"].cpu().tolist() == [0, 0] and int(c0["status_word"].item()) == 0
    kv = make_kv(50, H * D, 1)
    c1 = B.kv_quantise_chunks(kv, H, D, 1, tab, rid)
    back = B.kv_dequantise(c1, 50)
    torch.cuda.synchronize()
    assert np.all(c1["slot"].cpu().numpy()[:50] == B.KV_SLOT_ABSENT) and float(back.float().abs().max()) == 0.0
    # five chunks listed, the table holds three: rows of the last two are not cached
    so, co = np.array([0, 50], np.int32), np.array([0, 5], np.int32)
    cs, cl, ri = np.arange(0, 50, 10, dtype=np.int32), np.full(5, 10, np.int32), np.array([0, 1, 0, 1, 0], np.int32)
    sod, tab, rid = B.table_from_host(so, co, cs[:3], cl[:3], ri[:3], DEV)
    c2 = B.kv_quantise_chunks(kv, H, D, 1, tab, rid)
    torch.cuda.synchronize()
    ref = O.kv_quantise(host(kv), H, D, cs[:3], cl[:3], ri[:3], 1)
    assert c2["slot"].cpu().numpy()[:50].tolist() == ref["slot"].tolist()
    assert c2["counts"].cpu().tolist() == [20, 10]
