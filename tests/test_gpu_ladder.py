"""GPU parity of cwl_build_ladder against the CPU oracle (Sec. III-C: the rank ladder comes from one SVD
of the adapter update).  Singular vectors are fixed only up to sign and up to rotation inside equal singular
values, so the comparison is on what is unique: the singular values, every truncated product
A'[:, :k] B'[:k, :], and the defining identities."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import TOL_BF16, TOL_F32, host, rel_err
from paper_2601_21109_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def factors(d_in, d_out, r, seed, dtype, decay=0.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    A = torch.randn(d_in, r, generator=g) / d_in ** 0.5
    Bm = torch.randn(r, d_out, generator=g) / r ** 0.5
    if decay:
        # a trained adapter's spectrum falls off: scale the directions geometrically
        Bm = Bm * torch.pow(torch.tensor(decay), torch.arange(r, dtype=torch.float32))[:, None]
    return A.to(dtype), Bm.to(dtype)


@pytest.mark.parametrize("d_in,d_out,r,decay", [
    (64, 48, 8, 0.0), (257, 130, 16, 0.8), (1000, 300, 64, 0.9), (96, 640, 33, 0.0), (40, 40, 1, 0.0),
    (512, 384, 128, 0.95), (300, 700, 256, 0.97), (31, 7, 5, 0.0), (20, 7, 12, 0.0),
])
def test_ladder_matches_oracle_f32(d_in, d_out, r, decay):
    A, Bm = factors(d_in, d_out, r, r + d_in, torch.float32, decay)
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    rA, rB, rs = O.build_ladder(A.numpy(), Bm.numpy())
    A2, B2, sigma = host(A2).astype(np.float64), host(B2).astype(np.float64), sigma.cpu().numpy()
    assert np.max(np.abs(sigma - rs)) <= TOL_F32 * rs[0]
    W = A.numpy().astype(np.float64) @ Bm.numpy().astype(np.float64)
    assert rel_err(A2 @ B2, W) <= TOL_F32
    # every truncation the selector can pick
    for k in sorted({1, 2, 4, 8, 16, 32, 64, 128, r // 2, r - 1, r} & set(range(1, r + 1))):
        assert rel_err(A2[:, :k] @ B2[:k, :], rA[:, :k] @ rB[:k, :]) <= TOL_F32, k
    # orthogonal directions carrying sqrt(sigma) on each side
    assert np.max(np.abs(A2.T @ A2 - np.diag(rs))) <= 10 * TOL_F32 * rs[0]
    assert np.max(np.abs(B2 @ B2.T - np.diag(rs))) <= 10 * TOL_F32 * rs[0]


def test_ladder_bf16_and_strided_inputs():
    d_in, d_out, r = 320, 256, 32
    A, Bm = factors(d_in, d_out, r, 3, torch.bfloat16, 0.85)
    # inputs as column / row slices of wider buffers
    Abig = torch.zeros(d_in, r + 8, dtype=torch.bfloat16)
    Abig[:, :r] = A
    Bbig = torch.zeros(r, d_out + 16, dtype=torch.bfloat16)
    Bbig[:, :d_out] = Bm
    A2, B2, sigma = B.build_ladder(Abig.to(DEV)[:, :r], Bbig.to(DEV)[:, :d_out])
    torch.cuda.synchronize()
    rA, rB, rs = O.build_ladder(A.float().numpy(), Bm.float().numpy())
    assert A2.dtype == torch.bfloat16 and A2.is_contiguous()
    assert np.max(np.abs(sigma.cpu().numpy() - rs)) <= TOL_F32 * rs[0]        # sigma is not rounded to bf16
    A2, B2 = host(A2).astype(np.float64), host(B2).astype(np.float64)
    # the spectrum has gaps, so every direction is fixed up to one sign shared by its column of A' and its
    # row of B'; after aligning it the factors differ from the oracle's by their one rounding to bf16
    # (2^-9 relative; bar 2^-8, denominators floored at the direction's RMS as in rel_err)
    for k in range(r):
        sign = 1.0 if float(A2[:, k] @ rA[:, k]) >= 0 else -1.0
        assert rel_err(A2[:, k], sign * rA[:, k]) <= 2.0 ** -8, k
        assert rel_err(B2[k], sign * rB[k]) <= 2.0 ** -8, k
    # and the truncated products, now carrying two roundings per term
    for k in (4, 8, 16, 32):
        assert rel_err(A2[:, :k] @ B2[:k, :], rA[:, :k] @ rB[:k, :]) <= 2 * TOL_BF16, k


def test_ladder_rank_deficient_and_zero_update():
    A, Bm = factors(120, 90, 12, 4, torch.float32)
    Bm[7:] = 0                                   # rows a fresh adapter still has at zero
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    rA, rB, rs = O.build_ladder(A.numpy(), Bm.numpy())
    s = sigma.cpu().numpy()
    assert np.all(s[7:] == 0) and np.all(rs[7:] == 0) and np.max(np.abs(s - rs)) <= TOL_F32 * rs[0]
    assert torch.all(A2[:, 7:] == 0) and torch.all(B2[7:] == 0)
    assert rel_err(host(A2).astype(np.float64) @ host(B2).astype(np.float64), rA @ rB) <= TOL_F32
    # duplicated directions in A: the Gram matrix is singular
    A[:, 3] = A[:, 2]
    Bm = factors(120, 90, 12, 5, torch.float32)[1]
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    rA, rB, rs = O.build_ladder(A.numpy(), Bm.numpy())
    assert np.max(np.abs(sigma.cpu().numpy() - rs)) <= TOL_F32 * rs[0] and sigma[-1].item() == 0 == rs[-1]
    assert rel_err(host(A2).astype(np.float64) @ host(B2).astype(np.float64), rA @ rB) <= TOL_F32
    A2, B2, sigma = B.build_ladder(A.to(DEV), torch.zeros(12, 90, device=DEV))
    torch.cuda.synchronize()
    assert torch.all(sigma == 0) and torch.all(A2 == 0) and torch.all(B2 == 0)


def test_ladder_feeds_the_linear():
    """Full rank on the rebuilt factors is the same layer; a lower rung is the best approximation of it."""
    d_in, d_out, r = 128, 96, 16
    A, Bm = factors(d_in, d_out, r, 9, torch.float32, 0.7)
    g = torch.Generator(device="cpu").manual_seed(2)
    x = torch.randn(40, d_in, generator=g)
    W = torch.randn(d_in, d_out, generator=g) / d_in ** 0.5
    A2, B2, _ = B.build_ladder(A.to(DEV), Bm.to(DEV))
    so = torch.tensor([0, 40], dtype=torch.int32, device=DEV)
    tab = B.table_from_host(np.array([0, 40], np.int32), np.array([0, 2], np.int32), np.array([0, 24], np.int32),
                            np.array([24, 16], np.int32), np.array([1, 0], np.int32), DEV)
    sod, table, rid = tab
    y = B.chunkwise_lora_linear(x.to(DEV), W.to(DEV), A2, B2, [4, 16], [1.0, 1.0], 0, sod, table, rid)
    torch.cuda.synchronize()
    rA, rB, _ = O.build_ladder(A.numpy(), Bm.numpy())
    x64, W64 = x.numpy().astype(np.float64), W.numpy().astype(np.float64)
    ref = x64 @ W64
    ref[:24] += x64[:24] @ (A.numpy().astype(np.float64) @ Bm.numpy().astype(np.float64))     # full rank: the original layer
    ref[24:] += x64[24:] @ (rA[:, :4] @ rB[:4, :])                                              # rung of rank 4
    assert rel_err(host(y), ref) <= 2 * TOL_F32


@pytest.mark.parametrize("d_in,d_out,r,dtype", [
    (4096, 4096, 64, torch.float32), (4096, 11008, 128, torch.float32), (8192, 8192, 128, torch.bfloat16),
])
def test_ladder_at_workload_sizes(d_in, d_out, r, dtype):
    """The projections of the workloads with their largest rank.  An SVD of the full product is out of
    reach for a test, so the check is on what fixes the result: the spectrum through the r x r matrix
    (A^T A)(B B^T), whose eigenvalues are sigma^2 (float64 library routine); orthogonal directions carrying
    sqrt(sigma); and A' B' = A B on sampled rows."""
    A, Bm = factors(d_in, d_out, r, 21, dtype, 0.97)
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    tol = TOL_F32 if dtype == torch.float32 else 2.0 ** -8
    A64, B64 = A.float().numpy().astype(np.float64), Bm.float().numpy().astype(np.float64)
    ev = np.sort(np.linalg.eigvals((A64.T @ A64) @ (B64 @ B64.T)).real)[::-1]
    s = sigma.cpu().numpy()
    assert np.all(np.diff(s) <= 0)
    assert np.max(np.abs(s - np.sqrt(np.maximum(ev, 0)))) <= TOL_F32 * s[0]
    A2, B2 = host(A2).astype(np.float64), host(B2).astype(np.float64)
    assert np.max(np.abs(A2.T @ A2 - np.diag(s))) <= 10 * tol * s[0]
    assert np.max(np.abs(B2 @ B2.T - np.diag(s))) <= 10 * tol * s[0]
    rows = np.unique(np.linspace(0, d_in - 1, 97).astype(np.int64))
    assert rel_err(A2[rows] @ B2, A64[rows] @ B64) <= (TOL_F32 if dtype == torch.float32 else 2 * TOL_BF16)


def test_projections_that_share_x_as_one_fused_projection():
    """q/k/v-style projections fused by columns: W = [W0|W1|W2], A = [A0|A1|A2], B block-diagonal, ladder
    rebuilt on the fused update.  At full rank the fused layer is the three layers side by side."""
    d_in, d_out, r, n = 128, 64, 8, 48
    g = torch.Generator(device="cpu").manual_seed(11)
    Ws = [torch.randn(d_in, d_out, generator=g) / d_in ** 0.5 for _ in range(3)]
    As = [torch.randn(d_in, r, generator=g) / d_in ** 0.5 for _ in range(3)]
    Bs = [torch.randn(r, d_out, generator=g) / r ** 0.5 for _ in range(3)]
    x = torch.randn(n, d_in, generator=g)
    Af = torch.cat(As, dim=1)
    Bf = torch.zeros(3 * r, 3 * d_out)
    for i in range(3):
        Bf[i * r:(i + 1) * r, i * d_out:(i + 1) * d_out] = Bs[i]
    A2, B2, sigma = B.build_ladder(Af.to(DEV), Bf.to(DEV))
    sod, table, rid = B.table_from_host(np.array([0, n], np.int32), np.array([0, 2], np.int32),
                                        np.array([0, 30], np.int32), np.array([30, 18], np.int32),
                                        np.array([1, 0], np.int32), DEV)
    ranks, scales = [6, 3 * r], [1.0, 1.0]
    y = B.chunkwise_lora_linear(x.to(DEV), torch.cat(Ws, dim=1).to(DEV), A2, B2, ranks, scales, 0, sod, table, rid)
    torch.cuda.synchronize()
    x64 = x.numpy().astype(np.float64)
    rA, rB, rs = O.build_ladder(Af.numpy(), Bf.numpy())
    ref = np.concatenate([x64 @ W.numpy().astype(np.float64) for W in Ws], axis=1)
    # rows of the full-rank chunk: each projection's own textbook LoRA layer
    ref[:30] += np.concatenate([x64[:30] @ (a.numpy().astype(np.float64) @ b.numpy().astype(np.float64))
                                for a, b in zip(As, Bs)], axis=1)
    # rows of the rank-6 chunk: the best rank-6 approximation of the fused update
    ref[30:] += x64[30:] @ (rA[:, :6] @ rB[:6, :])
    assert rel_err(host(y), ref) <= 2 * TOL_F32
    assert np.max(np.abs(sigma.cpu().numpy() - rs)) <= TOL_F32 * rs[0]


def test_ladder_with_nan_in_the_factors_poisons_the_result_and_nothing_else():
    A, Bm = factors(64, 48, 8, 2, torch.float32)
    A[5, 3] = float("nan")
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    assert torch.isnan(sigma).any() or torch.isnan(A2).any()
    # the next call on clean factors is unaffected
    A, Bm = factors(64, 48, 8, 2, torch.float32)
    A2, B2, sigma = B.build_ladder(A.to(DEV), Bm.to(DEV))
    torch.cuda.synchronize()
    rA, rB, rs = O.build_ladder(A.numpy(), Bm.numpy())
    assert np.max(np.abs(sigma.cpu().numpy() - rs)) <= TOL_F32 * rs[0]
