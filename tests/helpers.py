"""Shared helpers of the GPU parity tests: error metrics and the oracle side of the pipeline."""
import math

import numpy as np
import torch

import oracle

TOL_F32 = 1e-5     # max relative error, fp32 path
TOL_BF16 = 2e-2    # max relative error, bf16 operands with fp32 accumulation


def rel_err(y, ref):
    """max |y - ref| / max(|ref|, rms(ref)): element-wise relative error with the denominator
    floored at the output RMS (outputs are sums with cancellation, so tiny elements would
    otherwise dominate)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = math.sqrt(float(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(y - ref) / den))


def gate_matrix(n_rows, r_max, ranks, scales, blend_w, seq_offsets, chunk_offsets, chunk_start, chunk_len, rank_idx):
    """The per-token, per-direction weights G[t, i] of the layer (cross-fade included), built directly from the
    definition: used by the tests only."""
    G = np.zeros((n_rows, r_max), dtype=np.float64)
    for b in range(len(seq_offsets) - 1):
        for c in range(chunk_offsets[b], chunk_offsets[b + 1]):
            s0, n = int(chunk_start[c]), int(chunk_len[c])
            r, sc = int(ranks[rank_idx[c]]), float(np.float32(scales[rank_idx[c]]))
            for j in range(n):
                if c == chunk_offsets[b] or blend_w == 0 or j >= blend_w:
                    G[s0 + j, :r] += sc
                else:
                    lam = float(np.float32(np.float32(j + 1) / np.float32(blend_w + 1)))
                    rp, sp = int(ranks[rank_idx[c - 1]]), float(np.float32(scales[rank_idx[c - 1]]))
                    G[s0 + j, :r] += lam * sc
                    G[s0 + j, :rp] += (1.0 - lam) * sp
    return G


def entropy_err(h, ref, vocab):
    """|H - ref| / max(ref, 1e-3 ln max(V, 2), 0.05), maximum over rows.  The 0.05-nat floor is what
    fp32 accumulation can resolve: H = ln S - T/S is formed from S = 1 + eps for a peaked row, and
    eps carries an absolute error of about 2^-24, i.e. ~1e-7 nat on H whatever its size."""
    h = np.asarray(h, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.maximum(ref, 1e-3 * math.log(max(vocab, 2))), 0.05)
    return float(np.max(np.abs(h - ref) / den))


def host(t):
    """Device tensor -> numpy (bf16 widened to fp32, which is exact)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.numpy()


def oracle_table(h_f32, seq_offsets, wl):
    """Oracle's quantise -> partition -> select on given fp32 scores (stage-wise parity)."""
    q, nan_seen = oracle.quantise(h_f32)
    st, tab = oracle.partition(q, seq_offsets, wl.l_min, wl.l_max,
                               oracle.quantise_threshold(wl.theta()),
                               oracle.quantise_threshold(wl.delta()))
    assert st == 0
    tab["rank_idx"] = oracle.select(tab["chunk_sum"], tab["chunk_len"],
                                    [oracle.quantise_threshold(t) for t in wl.taus()])
    tab["q"] = q
    tab["nan_seen"] = nan_seen
    return tab


def gpu_table_to_host(table, rank_idx=None):
    off = table["chunk_offsets"].cpu().numpy()
    n = min(int(off[-1]), table["cap"])
    out = {"chunk_offsets": off, "chunk_start": table["chunk_start"].cpu().numpy()[:n],
           "chunk_len": table["chunk_len"].cpu().numpy()[:n],
           "chunk_sum": table["chunk_sum"].cpu().numpy()[:n] if "chunk_sum" in table else None,
           "status": int(table["status_word"].cpu().item()) if "status_word" in table else 0}
    if rank_idx is not None:
        out["rank_idx"] = rank_idx.cpu().numpy()[:n]
    return out


def assert_tables_equal(gpu, ref):
    assert gpu["chunk_offsets"].tolist() == ref["chunk_offsets"].tolist()
    assert gpu["chunk_start"].tolist() == ref["chunk_start"].tolist()
    assert gpu["chunk_len"].tolist() == ref["chunk_len"].tolist()
    assert gpu["chunk_sum"].tolist() == ref["chunk_sum"].tolist()
    if "rank_idx" in gpu and "rank_idx" in ref:
        assert gpu["rank_idx"].tolist() == ref["rank_idx"].tolist()


def sample_rows(n_rows, chunk_start, chunk_len, blend_w, n_uniform, seed, first_chunks=64):
    """Deterministic row sample: every cross-fade row and the first / last row of the first
    `first_chunks` chunks, plus uniformly drawn rows."""
    rows = set()
    for c in range(min(first_chunks, len(chunk_start))):
        s, n = int(chunk_start[c]), int(chunk_len[c])
        rows.add(s)
        rows.add(s + n - 1)
        for j in range(min(blend_w, n)):
            rows.add(s + j)
    rng = np.random.RandomState(seed)
    rows.update(int(r) for r in rng.randint(0, n_rows, size=n_uniform))
    rows.add(0)
    rows.add(n_rows - 1)
    return np.array(sorted(rows), dtype=np.int64)
