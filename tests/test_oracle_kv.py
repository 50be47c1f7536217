"""Pins of the oracle's chunk-level KV-cache policy (Sec. III-E / IV-F): a hand-worked fixture, closed-form
cases (lossless grids, ties, zero heads), the error bound of symmetric INT8, invariances, and the pool layout
against an independent numpy restatement of the slot rule."""
import os

import numpy as np
import pytest

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kv_int8.txt")


def bf16(a, rng=None):
    """Random-free helper: float64 -> exact bf16 values in float32."""
    return O.bf16_round(np.asarray(a, dtype=np.float64)).astype(np.float32)


def read_golden(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = [float(t) for t in v.split()]
    return out


def test_hand_worked_fixture():
    g = read_golden(GOLDEN)
    H, D = int(g["n_heads"][0]), int(g["head_dim"][0])
    kv = np.array(g["kv"], dtype=np.float32).reshape(-1, H * D)
    r = O.kv_quantise(kv, H, D, np.array(g["chunk_start"], dtype=np.int32), np.array(g["chunk_len"], dtype=np.int32),
                      np.array(g["rank_idx"], dtype=np.int32), int(g["k_keep"][0]))
    assert r["slot"].tolist() == [int(v) for v in g["slot"]]
    assert r["codes"].reshape(-1).tolist() == [int(v) for v in g["codes"]]
    assert r["scale"].reshape(-1).tolist() == [float(np.float32(v)) for v in g["scale"]]
    assert r["kept"].reshape(-1).tolist() == g["kept"]
    # the scales in the fixture are 2/127 and 0.25/127 rounded to fp32
    assert float(np.float32(2.0) / np.float32(127.0)) == float(np.float32(g["scale"][0]))
    assert float(np.float32(0.25) / np.float32(127.0)) == float(np.float32(g["scale"][3]))


def one_chunk(kv, H, D, easy=True):
    n = kv.shape[0]
    return O.kv_quantise(kv, H, D, [0], [n], [0], 1 if easy else 0)


def test_integer_grid_is_lossless():
    """Values m * 2^e with |m| <= 127 and one |m| = 127: the factor 127 / amax is 2^-e exactly, the codes are
    the m themselves and code * scale gives the values back."""
    rng = np.random.RandomState(5)
    for e in (-9, -3, 0, 4):
        m = rng.randint(-127, 128, size=(6, 2 * 64)).astype(np.float32)
        m[:, 0] = 127
        m[:, 64] = -127
        kv = m * np.float32(2.0 ** e)
        r = one_chunk(kv, 2, 64)
        assert np.array_equal(r["codes"].astype(np.float32), m)
        assert np.all(r["scale"] == np.float32(2.0 ** e))
        back = O.kv_dequantise(r["slot"], r["codes"], r["scale"], r["kept"], 2, 64)
        assert np.array_equal(back, kv)


def test_error_bound_and_extremes():
    """|x - code * scale| <= scale / 2 (plus fp32 rounding of the product x * factor), the largest element
    maps to +-127, and a head of zeros has scale 0 and codes 0."""
    rng = np.random.RandomState(7)
    kv = bf16(rng.standard_normal((40, 4 * 128)) * np.exp(rng.uniform(-6, 6, size=(40, 1))))
    kv[3, 128:256] = 0.0
    r = one_chunk(kv, 4, 128)
    x = kv.reshape(40, 4, 128).astype(np.float64)
    codes = r["codes"].reshape(40, 4, 128).astype(np.float64)
    sc = r["scale"].astype(np.float64)[:, :, None]
    assert np.all(np.abs(x - codes * sc) <= sc * (0.5 + 1e-5))
    amax = np.abs(x).max(axis=2)
    assert np.allclose(r["scale"], amax / 127.0, rtol=2e-7, atol=0)
    am = np.abs(x).argmax(axis=2)
    top = np.take_along_axis(codes, am[:, :, None], axis=2)[:, :, 0]
    assert np.all(np.abs(top)[amax > 0] == 127)
    assert r["scale"][3, 1] == 0 and np.all(r["codes"].reshape(40, 4, 128)[3, 1] == 0)
    assert np.abs(codes).max() <= 127


def test_sign_symmetry_and_power_of_two_scaling():
    rng = np.random.RandomState(9)
    kv = bf16(rng.standard_normal((12, 2 * 64)))
    a, b, c = one_chunk(kv, 2, 64), one_chunk(-kv, 2, 64), one_chunk(kv * np.float32(8), 2, 64)
    assert np.array_equal(a["codes"], -b["codes"]) and np.array_equal(a["scale"], b["scale"])
    assert np.array_equal(a["codes"], c["codes"]) and np.array_equal(a["scale"] * np.float32(8), c["scale"])


def test_ties_round_to_even():
    # amax = 127 so the factor is exactly 1: halves go to the even neighbour
    kv = np.zeros((1, 64), dtype=np.float32)
    kv[0, :8] = [127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]
    r = one_chunk(kv, 1, 64)
    assert r["codes"][0, :8].tolist() == [127, 0, 2, 2, 0, -2, -2, 126]


def test_nan_and_inf_elements():
    kv = np.zeros((2, 64), dtype=np.float32)
    kv[0, :4] = [1.0, np.nan, -2.0, 0.5]
    kv[1, :3] = [np.inf, 3.0, -np.inf]
    r = one_chunk(kv, 1, 64)
    assert r["codes"][0, :4].tolist() == [64, 0, -127, 32]          # the NaN is ignored by the maximum, code 0
    assert float(r["scale"][0, 0]) == float(np.float32(2.0) / np.float32(127.0))
    assert r["codes"][1, :3].tolist() == [0, 0, 0] and np.isinf(r["scale"][1, 0])   # factor 127 / inf = 0


def slots_restated(n, chunk_start, chunk_len, rank_idx, k_keep):
    """The slot rule written independently: flags per row, then running counts per pool."""
    easy = np.zeros(n, dtype=bool)
    covered = np.zeros(n, dtype=bool)
    order = []
    for s, l, k in zip(chunk_start, chunk_len, rank_idx):
        covered[s:s + l] = True
        easy[s:s + l] = 0 <= k < k_keep
        order.extend(range(s, s + l))
    slot = np.full(n, O.SLOT_ABSENT, dtype=np.int64)
    order = np.array(order, dtype=np.int64)
    e = easy[order]
    slot[order[e]] = np.arange(int(e.sum()))
    slot[order[~e]] = -1 - np.arange(int((~e).sum()))
    return slot, covered


@pytest.mark.parametrize("k_keep", [0, 1, 2, 4])
def test_pools_hold_the_rows_in_table_order(k_keep):
    rng = np.random.RandomState(11 + k_keep)
    n, H, D = 300, 2, 64
    kv = bf16(rng.standard_normal((n, H * D)))
    # chunks that tile [10, 280): the rows before and after are covered by no chunk
    lens, pos = [], 10
    while pos < 280:
        l = min(int(rng.randint(3, 40)), 280 - pos)
        lens.append(l)
        pos += l
    starts = 10 + np.concatenate([[0], np.cumsum(lens)[:-1]])
    ranks = rng.randint(-1, 4, size=len(lens))
    r = O.kv_quantise(kv, H, D, starts, lens, ranks, k_keep)
    slot, covered = slots_restated(n, starts, lens, ranks, k_keep)
    assert r["slot"].astype(np.int64).tolist() == slot.tolist()
    assert np.all(r["slot"][~covered] == O.SLOT_ABSENT)
    kept_rows = np.where(covered & (slot < 0))[0]
    assert np.array_equal(r["kept"], kv[kept_rows])                 # bit for bit, in row order
    assert r["codes"].shape[0] == int((slot >= 0).sum()) and r["kept"].shape[0] == len(kept_rows)
    if k_keep == 0:
        assert r["codes"].shape[0] == 0
    # a quantised row equals the same row quantised alone
    for t in np.where(slot >= 0)[0][:20]:
        alone = one_chunk(kv[t:t + 1], H, D)
        assert np.array_equal(alone["codes"][0], r["codes"][slot[t]]) and np.array_equal(alone["scale"][0], r["scale"][slot[t]])
    back = O.kv_dequantise(r["slot"], r["codes"], r["scale"], r["kept"], H, D)
    assert np.array_equal(back[kept_rows], kv[kept_rows]) and np.all(back[~covered] == 0)


def test_policy_is_monotone_in_k_keep():
    rng = np.random.RandomState(13)
    kv = bf16(rng.standard_normal((64, 64)))
    starts, lens, ranks = [0, 16, 32, 48], [16, 16, 16, 16], [0, 1, 2, 3]
    counts = [O.kv_quantise(kv, 1, 64, starts, lens, ranks, k)["codes"].shape[0] for k in range(6)]
    assert counts == [0, 16, 32, 48, 64, 64]
