"""Pins for the oracle's chunk-segmented LoRA linear (Sec. III-C/D): special cases that reduce
to textbook LoRA via a float64 library matmul, the gate reformulation, and a hand-worked
example.  Shapes are non-square so that a transposed operand fails."""
import numpy as np
import pytest

from conftest import read_golden


def one_chunk_table(n):
    return ([0, n], [0, 1], [0], [n])


def rand_ops(rng, n, d_in, d_out, r):
    x = rng.randn(n, d_in).astype(np.float32)
    W = (rng.randn(d_in, d_out) / np.sqrt(d_in)).astype(np.float32)
    A = (rng.randn(d_in, r) / np.sqrt(d_in)).astype(np.float32)
    B = (rng.randn(r, d_out) / np.sqrt(r)).astype(np.float32)
    return x, W, A, B


def f64(*a):
    return [v.astype(np.float64) for v in a]


def test_golden_w2(oracle):
    g = read_golden("linear_w2.txt")
    W = np.array(g["W"], np.float32).reshape(2, 2)
    A = np.array(g["A"], np.float32).reshape(2, 2)
    B = np.array(g["B"], np.float32).reshape(2, 2)
    x = np.ones((4, 2), np.float32)
    y = oracle.linear(x, W, A, B, g["ranks"], g["scales"], g["blend_w"][0], [0, 4], [0, 2],
                      g["chunk_start"], g["chunk_len"], g["rank_idx"])
    assert np.allclose(y.ravel(), g["y"], rtol=0, atol=1e-12)


def test_full_rank_single_chunk_is_textbook_lora(oracle):
    rng = np.random.RandomState(0)
    n, d_in, d_out, r = 13, 24, 40, 6
    x, W, A, B = rand_ops(rng, n, d_in, d_out, r)
    s = 16.0 / r
    so, co, cs, cl = one_chunk_table(n)
    y = oracle.linear(x, W, A, B, [r], [s], 3, so, co, cs, cl, [0])
    xd, Wd, Ad, Bd = f64(x, W, A, B)
    sd = float(np.float32(s))
    assert np.allclose(y, xd @ Wd + sd * (xd @ Ad) @ Bd, rtol=1e-12, atol=1e-12)
    assert np.allclose(y, xd @ (Wd + sd * Ad @ Bd), rtol=1e-11, atol=1e-11)   # merged weights


def test_rank_zero_is_bare_gemm(oracle):
    rng = np.random.RandomState(1)
    n, d_in, d_out, r = 9, 16, 10, 4
    x, W, A, B = rand_ops(rng, n, d_in, d_out, r)
    so, co, cs, cl = one_chunk_table(n)
    y = oracle.linear(x, W, A, B, [0], [123.0], 2, so, co, cs, cl, [0])
    xd, Wd = f64(x, W)
    assert np.allclose(y, xd @ Wd, rtol=1e-13, atol=1e-13)
    # r_max = 0 adapters
    y0 = oracle.linear(x, W, np.zeros((d_in, 0), np.float32), np.zeros((0, d_out), np.float32),
                       [0], [1.0], 0, so, co, cs, cl, [0])
    assert np.allclose(y0, xd @ Wd, rtol=1e-13, atol=1e-13)


def table3():
    # two sequences: 0..19 (chunks 7, 6, 7) and 20..30 (chunks 5, 6)
    so = [0, 20, 31]
    co = [0, 3, 5]
    cs = [0, 7, 13, 20, 25]
    cl = [7, 6, 7, 5, 6]
    return so, co, cs, cl


def gate_reference(x, W, A, B, ranks, scales, w, so, co, cs, cl, ri):
    """y = x W + ((x A) * G) B with the per-token, per-direction gate built here."""
    xd, Wd, Ad, Bd = f64(x, W, A, B)
    n, r_max = x.shape[0], A.shape[1]
    G = np.zeros((n, r_max))
    for b in range(len(so) - 1):
        for c in range(co[b], co[b + 1]):
            for j in range(cl[c]):
                t = cs[c] + j
                rc, sc = ranks[ri[c]], float(np.float32(scales[ri[c]]))
                if c == co[b] or w == 0 or j >= w:
                    G[t, :rc] += sc
                else:
                    lam = (j + 1) / (w + 1)
                    rp, sp = ranks[ri[c - 1]], float(np.float32(scales[ri[c - 1]]))
                    G[t, :rp] += (1 - lam) * sp
                    G[t, :rc] += lam * sc
    return xd @ Wd + ((xd @ Ad) * G) @ Bd


@pytest.mark.parametrize("w", [0, 1, 3, 5])
def test_gate_identity(oracle, w):
    rng = np.random.RandomState(2 + w)
    d_in, d_out, r = 12, 18, 8
    so, co, cs, cl = table3()
    x, W, A, B = rand_ops(rng, 31, d_in, d_out, r)
    ranks, scales = [0, 2, 5, 8], [9.0, 8.0, 3.2, 2.0]
    ri = [3, 0, 2, 1, 3]
    y = oracle.linear(x, W, A, B, ranks, scales, w, so, co, cs, cl, ri)
    want = gate_reference(x, W, A, B, ranks, scales, w, so, co, cs, cl, ri)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


def test_hard_switch_equals_per_chunk_fixed_rank(oracle):
    rng = np.random.RandomState(7)
    d_in, d_out, r = 10, 14, 6
    so, co, cs, cl = table3()
    x, W, A, B = rand_ops(rng, 31, d_in, d_out, r)
    ranks, scales = [1, 3, 6], [16.0, 16 / 3, 16 / 6]
    ri = [2, 0, 1, 1, 0]
    y = oracle.linear(x, W, A, B, ranks, scales, 0, so, co, cs, cl, ri)
    xd, Wd, Ad, Bd = f64(x, W, A, B)
    for c in range(5):
        rows = slice(cs[c], cs[c] + cl[c])
        rk, s = ranks[ri[c]], float(np.float32(scales[ri[c]]))
        want = xd[rows] @ Wd + s * (xd[rows] @ Ad[:, :rk]) @ Bd[:rk, :]
        assert np.allclose(y[rows], want, rtol=1e-12, atol=1e-12)


def test_blend_weights_and_sequence_starts(oracle):
    rng = np.random.RandomState(8)
    d_in, d_out, r = 6, 5, 4
    so, co, cs, cl = table3()
    x, W, A, B = rand_ops(rng, 31, d_in, d_out, r)
    ranks, scales = [2, 4], [3.0, 1.5]
    ri = [0, 1, 0, 1, 0]
    w = 3
    y = oracle.linear(x, W, A, B, ranks, scales, w, so, co, cs, cl, ri)
    xd, Wd, Ad, Bd = f64(x, W, A, B)
    base = xd @ Wd
    D = [s * (xd @ Ad[:, :rk]) @ Bd[:rk, :] for rk, s in zip(ranks, scales)]
    # token 7 is the first token of chunk 1 (rung 1) after chunk 0 (rung 0): lambda = 1/4
    for j, lam in enumerate([0.25, 0.5, 0.75]):
        t = 7 + j
        assert np.allclose(y[t], base[t] + (1 - lam) * D[0][t] + lam * D[1][t], atol=1e-12)
    assert np.allclose(y[10], base[10] + D[1][10], atol=1e-12)
    # token 20 opens the second sequence: no cross-fade with the previous sequence's last chunk
    assert np.allclose(y[20], base[20] + D[1][20], atol=1e-12)
    assert np.allclose(y[0], base[0] + D[0][0], atol=1e-12)


def test_same_rung_join_is_a_no_op(oracle):
    rng = np.random.RandomState(9)
    so, co, cs, cl = table3()
    x, W, A, B = rand_ops(rng, 31, 8, 9, 4)
    ranks, scales = [2, 4], [3.0, 1.5]
    y_blend = oracle.linear(x, W, A, B, ranks, scales, 4, so, co, cs, cl, [1, 1, 1, 0, 0])
    y_hard = oracle.linear(x, W, A, B, ranks, scales, 0, so, co, cs, cl, [1, 1, 1, 0, 0])
    assert np.allclose(y_blend, y_hard, rtol=1e-13, atol=1e-13)


def test_linearity_in_x_and_row_subset(oracle):
    rng = np.random.RandomState(10)
    so, co, cs, cl = table3()
    x1, W, A, B = rand_ops(rng, 31, 8, 9, 4)
    x2 = rng.randn(31, 8).astype(np.float32)
    ranks, scales, ri = [1, 4], [2.0, 0.5], [0, 1, 1, 0, 1]
    args = (ranks, scales, 2, so, co, cs, cl, ri)
    y1 = oracle.linear(x1, W, A, B, *args)
    y2 = oracle.linear(x2, W, A, B, *args)
    xs = (x1.astype(np.float64) * 2 + x2.astype(np.float64) * 0.5).astype(np.float32)
    exact = np.all(xs.astype(np.float64) == x1.astype(np.float64) * 2 + x2 * 0.5)
    ys = oracle.linear(xs, W, A, B, *args)
    if exact:
        assert np.allclose(ys, 2 * y1 + 0.5 * y2, rtol=1e-10, atol=1e-10)
    rows = [30, 0, 7, 8, 20, 13]
    assert np.array_equal(oracle.linear(x1, W, A, B, *args, rows=rows), y1[rows])


def test_uncovered_token_gets_base_only(oracle):
    rng = np.random.RandomState(11)
    x, W, A, B = rand_ops(rng, 10, 6, 7, 3)
    # chunk table covers rows 0..5 only
    y = oracle.linear(x, W, A, B, [3], [2.0], 0, [0, 10], [0, 1], [0], [6], [0])
    xd, Wd, Ad, Bd = f64(x, W, A, B)
    assert np.allclose(y[6:], (xd @ Wd)[6:], atol=1e-13)
    assert np.allclose(y[:6], (xd @ Wd + 2.0 * (xd @ Ad) @ Bd)[:6], atol=1e-12)


def test_bf16_round_helper(oracle):
    import torch
    v = np.array([1.0, 1.00390625, 1.001953125, 3.14159, -2.71828, 1e-3, 65504.0, 0.0])
    want = torch.tensor(v, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).double().numpy()
    assert np.array_equal(oracle.bf16_round(v), want)


def test_compact_x_equals_full_x(oracle):
    rng = np.random.RandomState(12)
    so, co, cs, cl = table3()
    x, W, A, B = rand_ops(rng, 31, 8, 9, 4)
    args = ([1, 4], [2.0, 0.5], 2, so, co, cs, cl, [0, 1, 1, 0, 1])
    rows = [30, 7, 8, 20, 0]
    full = oracle.linear(x, W, A, B, *args, rows=rows)
    compact = oracle.linear(x[rows], W, A, B, *args, rows=rows, x_compact=True)
    assert np.array_equal(full, compact)
