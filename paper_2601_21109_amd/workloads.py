"""Seeded synthetic inputs shaped like the paper's workloads (LLaMA-7B / 70B projections,
32000 / 128000-entry vocabularies, text with interleaved easy and hard spans; Sec. I and
Sec. V-A of arxiv 2601.21109).

This module only draws random numbers and names shapes and policy parameters.  It holds none
of the method's arithmetic and is the one module that both the tests of the HIP path and the
tests of the CPU oracle use.  The paper evaluates on Wikitext-103, SQuAD v2.0 and FLORES-101
with trained weights; none of that is available, so Gaussian stand-ins of the same shapes are
used everywhere.
"""
import math
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np
import torch

BASE_SEED = 260121109


@dataclass
class Workload:
    name: str
    index: int
    dtype: torch.dtype
    n_seqs: int
    seq_len: int
    vocab: int
    projections: List[Tuple[str, int, int]]          # (name, d_in, d_out)
    ladder: List[int]
    l_min: int
    l_max: int
    blend_w: int
    span: Tuple[int, int]                            # span length range (inclusive)
    sigmas: Tuple[float, ...] = (0.5, 2.0, 6.0)
    sigma_probs: Tuple[float, ...] = (1 / 3, 1 / 3, 1 / 3)
    alpha: float = 16.0
    theta_frac: float = 0.90                          # fractions of ln V
    delta_frac: float = 0.30
    tau_fracs: Tuple[float, ...] = field(default_factory=tuple)
    logit_tile_rows: int = 0                          # >0: logits are produced / scored in tiles

    @property
    def n_rows(self):
        return self.n_seqs * self.seq_len

    @property
    def r_max(self):
        return self.ladder[-1]

    @property
    def seed(self):
        return BASE_SEED + self.index

    @property
    def scales(self):
        return [self.alpha / r if r > 0 else 0.0 for r in self.ladder]

    def theta(self):
        return float(np.float32(self.theta_frac * math.log(self.vocab)))

    def delta(self):
        return float(np.float32(self.delta_frac * math.log(self.vocab)))

    def taus(self):
        return [float(np.float32(f * math.log(self.vocab))) for f in self.tau_fracs]


_TAU = {3: (0.45, 0.90), 4: (0.30, 0.60, 0.90), 6: (0.10, 0.30, 0.60, 0.90, 0.95)}


def _mk(**kw):
    kw.setdefault("tau_fracs", _TAU[len(kw["ladder"])])
    return Workload(**kw)


WORKLOADS = {
    "cfg0": _mk(name="cfg0", index=0, dtype=torch.float32, n_seqs=1, seq_len=128, vocab=1024,
                projections=[("proj", 256, 256)], ladder=[4, 8, 16], l_min=8, l_max=64,
                blend_w=2, span=(16, 16)),
    "cfg1": _mk(name="cfg1", index=1, dtype=torch.bfloat16, n_seqs=8, seq_len=2048, vocab=32000,
                projections=[("q_proj", 4096, 4096)], ladder=[8, 16, 32, 64], l_min=32,
                l_max=512, blend_w=4, span=(32, 256)),
    "cfg2": _mk(name="cfg2", index=2, dtype=torch.bfloat16, n_seqs=16, seq_len=4096, vocab=32000,
                projections=[("up_proj", 4096, 11008), ("gate_proj", 4096, 11008),
                             ("down_proj", 11008, 4096)],
                ladder=[8, 16, 32, 64], l_min=32, l_max=512, blend_w=4, span=(32, 256)),
    "cfg3": _mk(name="cfg3", index=3, dtype=torch.bfloat16, n_seqs=32, seq_len=2048, vocab=32000,
                projections=[("q_proj", 4096, 4096), ("k_proj", 4096, 4096),
                             ("v_proj", 4096, 4096), ("o_proj", 4096, 4096),
                             ("gate_proj", 4096, 11008), ("up_proj", 4096, 11008),
                             ("down_proj", 11008, 4096)],
                ladder=[4, 8, 16, 32, 64, 128], l_min=32, l_max=512, blend_w=4, span=(32, 256),
                sigmas=(0.5, 6.0), sigma_probs=(0.7, 0.3)),
    "cfg4": _mk(name="cfg4", index=4, dtype=torch.bfloat16, n_seqs=1, seq_len=32768,
                vocab=128000, projections=[("proj", 8192, 8192)], ladder=[16, 32, 64, 128],
                l_min=64, l_max=2048, blend_w=8, span=(32, 256), logit_tile_rows=4096),
}


def scaled(wl: Workload, *, n_seqs=None, seq_len=None, vocab=None, projections=None, name=None):
    """A smaller / reshaped copy of a workload (same generator, same policy fractions)."""
    import copy
    w = copy.deepcopy(wl)
    if n_seqs is not None:
        w.n_seqs = n_seqs
    if seq_len is not None:
        w.seq_len = seq_len
    if vocab is not None:
        w.vocab = vocab
    if projections is not None:
        w.projections = projections
    if name is not None:
        w.name = name
    return w


def seq_offsets(wl: Workload) -> np.ndarray:
    return (np.arange(wl.n_seqs + 1, dtype=np.int64) * wl.seq_len).astype(np.int32)


def token_sigmas(wl: Workload) -> np.ndarray:
    """Per-token noise level: every sequence is cut into spans, each span draws one sigma."""
    rng = np.random.RandomState(wl.seed % (2 ** 31))
    out = np.empty(wl.n_rows, dtype=np.float32)
    lo, hi = wl.span
    for b in range(wl.n_seqs):
        t = 0
        while t < wl.seq_len:
            n = int(rng.randint(lo, hi + 1))
            s = wl.sigmas[int(rng.choice(len(wl.sigmas), p=np.asarray(wl.sigma_probs)))]
            out[b * wl.seq_len + t: b * wl.seq_len + min(t + n, wl.seq_len)] = s
            t += n
    return out


def _gen(wl: Workload, device, salt):
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed * 1000 + salt)
    return g


def logits_rows(wl: Workload, row0: int, row1: int, device="cpu", sigmas=None) -> torch.Tensor:
    """logits[row0:row1, :] = sigma_span * N(0,1), cast to the workload dtype.

    Rows are drawn in blocks of 512 rows, each block from its own seeded generator, so any
    512-aligned row range gives the same values whichever range it is produced in.
    """
    if sigmas is None:
        sigmas = token_sigmas(wl)
    blk = 512
    assert row0 % blk == 0 or row0 == row1
    out = torch.empty((row1 - row0, wl.vocab), dtype=wl.dtype, device=device)
    for r in range(row0, row1, blk):
        e = min(r + blk, row1)
        g = _gen(wl, device, 7 + r // blk * 16)
        z = torch.randn((e - r, wl.vocab), generator=g, device=device, dtype=torch.float32)
        s = torch.from_numpy(sigmas[r:e]).to(device).unsqueeze(1)
        out[r - row0:e - row0] = (z * s).to(wl.dtype)
    return out


def logits(wl: Workload, device="cpu") -> torch.Tensor:
    return logits_rows(wl, 0, wl.n_rows, device)


def linear_operands(wl: Workload, proj: int = 0, device="cpu", n_rows=None):
    """x ~ N(0,1), W ~ N(0,1/d_in), A ~ N(0,1/d_in), B ~ N(0,1/r_max), in the workload dtype.
    W is [d_in, d_out], A is [d_in, r_max], B is [r_max, d_out]."""
    _, d_in, d_out = wl.projections[proj]
    n = wl.n_rows if n_rows is None else n_rows
    r = wl.r_max

    def draw(shape, std, salt):
        g = _gen(wl, device, 100 + 10 * proj + salt)
        t = torch.empty(shape, dtype=wl.dtype, device=device)
        rows_per = max(1, (1 << 24) // shape[1])
        for i in range(0, shape[0], rows_per):
            j = min(i + rows_per, shape[0])
            t[i:j] = (torch.randn((j - i, shape[1]), generator=g, device=device,
                                  dtype=torch.float32) * std).to(wl.dtype)
        return t

    x = draw((n, d_in), 1.0, 1)
    W = draw((d_in, d_out), 1.0 / math.sqrt(d_in), 2)
    A = draw((d_in, r), 1.0 / math.sqrt(d_in), 3)
    B = draw((r, d_out), 1.0 / math.sqrt(r), 4)
    return x, W, A, B


def random_chunk_table(n_seqs, seq_lens, l_min, l_max, K, seed):
    """A valid random chunk table (not produced by the chunker): used to drive the linear on
    arbitrary joins.  Returns seq_offsets, chunk_offsets, chunk_start, chunk_len, rank_idx."""
    rng = np.random.RandomState(seed)
    so = np.zeros(n_seqs + 1, dtype=np.int32)
    so[1:] = np.cumsum(seq_lens)
    co, cs, cl = [0], [], []
    for b in range(n_seqs):
        t, T = 0, int(seq_lens[b])
        while t < T:
            n = int(rng.randint(l_min, l_max + 1))
            n = min(n, T - t)
            cs.append(int(so[b]) + t)
            cl.append(n)
            t += n
        co.append(len(cs))
    ri = rng.randint(0, K, size=len(cs)).astype(np.int32)
    return (so, np.asarray(co, np.int32), np.asarray(cs, np.int32), np.asarray(cl, np.int32), ri)
