"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments before anything is launched (no GPU is touched here)."""
import ctypes
import math
import os
import re

import pytest

from conftest import ROOT
from paper_2601_21109_amd import binding as B


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2601_21109_amd import build
        build.build()
    return B.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cwl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cwl_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_return_types_of_the_exports(L):
    """Byte counts come back as size_t (a workspace may exceed 2 GiB), statuses as int."""
    for n in B.EXPORTS:
        if n.endswith("_bytes"):
            assert getattr(L, n).restype is ctypes.c_size_t, n
        elif n not in ("cwl_status_string", "cwl_abi_version"):
            assert getattr(L, n).restype is ctypes.c_int, n


def test_static_scratch_entry_argument_errors(L):
    """The entry point without a workspace argument rejects bad arguments, and descriptors that need more
    than its static array, before it touches the device."""
    f = L.cwl_chunkwise_lora_linear_packed_static

    def status(d, x=P(0x10000), packed=P(0x20000), y=P(0x30000)):
        return f(d.ref(), x, packed, P(), 1, P(), P(), P(), P(), 8, y, None)

    assert status(make_desc(n_rows=-1)) == B.ERR_INVALID_ARG
    assert status(make_desc(), x=None) == B.ERR_NULL
    assert status(make_desc(), y=None) == B.ERR_NULL
    assert status(make_desc(), packed=None) == B.ERR_NULL
    assert status(make_desc(), packed=P(0x20010)) == B.ERR_INVALID_ARG
    assert status(make_desc(n_rows=0)) == B.OK
    big = make_desc(n_rows=1 << 20)                          # gate table alone: 16 MiB
    assert L.cwl_linear_packed_workspace_bytes(big.ref()) > B.STATIC_SCRATCH_BYTES
    assert status(big) == B.ERR_CAPACITY
    text = open(os.path.join(ROOT, "include", "cwl.h")).read()
    assert f"#define CWL_STATIC_SCRATCH_BYTES ((size_t){B.STATIC_SCRATCH_BYTES >> 20} << 20)" in text


def test_version_and_status_strings(L):
    assert L.cwl_abi_version() == 1
    seen = {B.status_string(s) for s in range(7)}
    assert len(seen) == 7 and all(seen)


def P(v=0x1000):
    return ctypes.c_void_p(v)


def test_score_tokens_argument_errors(L):
    f = L.cwl_score_tokens
    assert f(P(), B.F32, -1, 8, 8, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), B.F32, 4, 0, 8, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), B.F32, 4, 8, 7, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), 7, 4, 8, 8, P(), None) == B.ERR_INVALID_ARG
    assert f(None, B.F32, 4, 8, 8, P(), None) == B.ERR_NULL
    assert f(P(), B.F32, 4, 8, 8, None, None) == B.ERR_NULL
    assert f(P(0x1002), B.F32, 4, 8, 8, P(), None) == B.ERR_INVALID_ARG     # misaligned fp32
    assert f(None, B.F32, 0, 8, 8, None, None) == B.OK                      # empty: no-op


def test_partition_argument_errors(L):
    f = L.cwl_partition_chunks

    def call(l_min=4, l_max=8, n_rows=64, n_seqs=1, cap=32, ws=P(0x10000), ws_bytes=1 << 20,
             ent=P(), so=P(), status=P()):
        p = B.ChunkParams(l_min, l_max, math.inf, math.inf)
        return f(ent, n_rows, so, n_seqs, ctypes.byref(p), P(), P(), P(), P(), cap, status, ws,
                 ws_bytes, None)

    assert call(l_min=0) == B.ERR_INVALID_ARG
    assert call(l_min=5, l_max=4) == B.ERR_INVALID_ARG
    assert call(l_min=4, l_max=6) == B.ERR_INFEASIBLE
    assert call(n_rows=-1) == B.ERR_INVALID_ARG
    assert call(cap=-1) == B.ERR_INVALID_ARG
    assert call(so=None) == B.ERR_NULL
    assert call(status=None) == B.ERR_NULL
    assert call(ent=None) == B.ERR_NULL
    assert call(ws=None) == B.ERR_NULL
    assert call(ws=P(0x10010)) == B.ERR_INVALID_ARG
    assert call(ws_bytes=16) == B.ERR_CAPACITY
    assert f(P(), 64, P(), 1, None, P(), P(), P(), P(), 8, P(), P(0x10000), 1 << 20, None) == B.ERR_NULL
    p = B.ChunkParams(4, 8, 1.0, 1.0)
    assert L.cwl_partition_workspace_bytes(1000, 3, ctypes.byref(p)) > 1000 * 12
    bad = B.ChunkParams(4, 6, 1.0, 1.0)
    assert L.cwl_partition_workspace_bytes(1000, 3, ctypes.byref(bad)) == 0


def test_select_argument_errors(L):
    f = L.cwl_select_ranks
    th = (ctypes.c_float * 3)(1.0, 2.0, 3.0)
    bad = (ctypes.c_float * 3)(1.0, 3.0, 2.0)
    nan = (ctypes.c_float * 3)(1.0, math.nan, 2.0)
    assert f(P(), P(), P(), 1, 8, th, 0, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), P(), 1, 8, th, B.MAX_LADDER + 1, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), P(), 1, 8, bad, 4, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), P(), 1, 8, nan, 4, P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), P(), 1, 8, None, 4, P(), None) == B.ERR_NULL
    assert f(None, P(), P(), 1, 8, th, 4, P(), None) == B.ERR_NULL
    assert f(P(), P(), P(), 1, 0, th, 4, P(), None) == B.OK


def make_desc(**kw):
    args = dict(n_rows=128, d_in=256, d_out=256, r_max=16, ranks=[4, 8, 16], scales=[4.0, 2.0, 1.0],
                blend_w=2, dt=B.F32, ldx=256, ldw=256, lda=16, ldb=256, ldy=256, group_rows=0)
    args.update(kw)
    return B._Desc(**args)


def test_linear_descriptor_errors(L):
    ws_bytes = L.cwl_linear_workspace_bytes

    def status(d, x=P(0x10000), W=P(0x20000), y=P(0x30000), ws=P(0x40000), nbytes=1 << 30):
        return L.cwl_chunkwise_lora_linear(d.ref(), x, W, P(), P(), P(), 1, P(), P(), P(), P(), 8, y,
                                           ws, nbytes, None)

    assert ws_bytes(make_desc().ref()) > 0
    for kw in (dict(n_rows=-1), dict(d_in=0), dict(r_max=B.MAX_RANK + 1), dict(ranks=[8, 4, 16]),
               dict(ranks=[4, 8, 32]), dict(ranks=[-1, 8, 16]), dict(blend_w=-1), dict(dt=5),
               dict(ldx=255), dict(ldy=100), dict(group_rows=2),
               dict(scales=[1.0, math.nan, 1.0])):
        d = make_desc(**kw)
        assert ws_bytes(d.ref()) == 0, kw
        assert status(d) == B.ERR_INVALID_ARG, kw
    assert status(make_desc(ldw=255)) == B.ERR_INVALID_ARG
    assert status(make_desc(lda=15)) == B.ERR_INVALID_ARG
    # bf16 shape and alignment restrictions
    assert status(make_desc(dt=B.BF16, d_in=200, ldx=200)) == B.ERR_UNSUPPORTED
    assert status(make_desc(dt=B.BF16, d_out=252, ldy=256)) == B.ERR_UNSUPPORTED
    assert status(make_desc(dt=B.BF16), x=P(0x10008)) == B.ERR_UNSUPPORTED
    # pointers and workspace
    assert status(make_desc(), x=None) == B.ERR_NULL
    assert status(make_desc(), y=None) == B.ERR_NULL
    assert status(make_desc(), ws=None) == B.ERR_NULL
    assert status(make_desc(), W=None) == B.ERR_NULL
    assert status(make_desc(), ws=P(0x40010)) == B.ERR_INVALID_ARG
    assert status(make_desc(), nbytes=1024) == B.ERR_CAPACITY
    assert status(make_desc(n_rows=0)) == B.OK
    assert L.cwl_chunkwise_lora_linear(None, P(), P(), P(), P(), P(), 1, P(), P(), P(), P(), 8, P(),
                                       P(), 0, None) == B.ERR_NULL
    # packed entry point and prepack
    d = make_desc()
    assert L.cwl_packed_weights_bytes(d.ref()) >= 4 * (256 * 256 + 64 * 256 * 2)
    assert L.cwl_prepack_weights(d.ref(), P(), P(), P(), P(0x50000), 16, None) == B.ERR_CAPACITY
    assert L.cwl_prepack_weights(d.ref(), None, P(), P(), P(0x50000), 1 << 30, None) == B.ERR_NULL
    assert L.cwl_chunkwise_lora_linear_packed(d.ref(), P(0x10000), None, P(), 1, P(), P(), P(), P(),
                                              8, P(0x30000), P(0x40000), 1 << 30, None) == B.ERR_NULL
    assert L.cwl_linear_packed_workspace_bytes(d.ref()) < L.cwl_linear_workspace_bytes(d.ref())


def test_grouped_calls_argument_errors(L):
    """Projections that share x: the group must have 1..8 projections whose columns add up to d_out."""
    def group(d_outs, ptr=0x1000):
        g = B.Group()
        g.n_proj = len(d_outs)
        for p, n in enumerate(d_outs[:B.MAX_GROUP]):
            g.d_out[p] = n
            g.W[p] = g.A[p] = g.B[p] = ptr
        return g

    d = make_desc(d_out=256, ldy=256)
    ok = group([128, 128])
    assert L.cwl_packed_weights_grouped_bytes(d.ref(), ctypes.byref(ok)) > L.cwl_packed_weights_bytes(d.ref())
    assert L.cwl_linear_grouped_workspace_bytes(d.ref(), ctypes.byref(ok)) > L.cwl_linear_packed_workspace_bytes(d.ref())

    def status(dd, g, x=P(0x10000), packed=P(0x20000), y=P(0x30000), ws=P(0x40000), nbytes=1 << 30):
        return L.cwl_chunkwise_lora_linear_grouped_packed(dd.ref(), ctypes.byref(g) if g is not None else None, x,
                                                          packed, P(), 1, P(), P(), P(), P(), 8, y, ws, nbytes, None)

    assert status(d, None) == B.ERR_NULL
    assert status(d, group([128, 64])) == B.ERR_INVALID_ARG           # columns do not add up
    assert status(d, group([])) == B.ERR_INVALID_ARG
    g9 = group([32] * 8)
    g9.n_proj = 9
    assert status(d, g9) == B.ERR_INVALID_ARG
    assert status(d, group([256, 0])) == B.ERR_INVALID_ARG
    assert status(make_desc(d_out=256, ldy=256, group_rows=1), ok) == B.ERR_UNSUPPORTED
    assert status(make_desc(d_out=256, ldy=256, dt=B.BF16), group([252, 4])) == B.ERR_UNSUPPORTED
    assert status(d, ok, x=None) == B.ERR_NULL
    assert status(d, ok, packed=None) == B.ERR_NULL
    assert status(d, ok, nbytes=64) == B.ERR_CAPACITY
    assert status(make_desc(d_out=256, ldy=256, n_rows=0), ok) == B.OK
    assert L.cwl_packed_weights_grouped_bytes(d.ref(), ctypes.byref(group([128, 64]))) == 0
    # prepack: every projection brings its three pointers
    bad = group([128, 128])
    bad.B[1] = None
    assert L.cwl_prepack_weights_grouped(d.ref(), ctypes.byref(bad), P(0x50000), 1 << 30, None) == B.ERR_NULL
    assert L.cwl_prepack_weights_grouped(d.ref(), ctypes.byref(ok), P(0x50000), 16, None) == B.ERR_CAPACITY
    assert L.cwl_gated_lora_linear_grouped_packed(d.ref(), ctypes.byref(ok), P(0x10000), P(0x20000), None, P(0x30000),
                                                  P(0x40000), 1 << 30, None) == B.ERR_NULL


def test_stream_step_and_gated_linear_argument_errors(L):
    f = L.cwl_stream_step
    p = B.ChunkParams(4, 9, 1.0, 1.0)
    th = (ctypes.c_float * 2)(1.0, 2.0)
    rk = (ctypes.c_int32 * 3)(4, 8, 16)
    sc = (ctypes.c_float * 3)(4.0, 2.0, 1.0)
    ok_args = (P(), 5, ctypes.byref(p), th, 3, rk, sc, 2, P(), P(), P(), P(), P(), None)

    def call(**kw):
        names = ["entropy", "n_seqs", "p", "th", "K", "ranks", "scales", "w", "state", "gate", "cl", "cs",
                 "status", "stream"]
        a = dict(zip(names, ok_args))
        a.update(kw)
        return f(*[a[n] for n in names])

    assert call(p=None) == B.ERR_NULL
    assert call(p=ctypes.byref(B.ChunkParams(4, 6, 1.0, 1.0))) == B.ERR_INFEASIBLE
    assert call(p=ctypes.byref(B.ChunkParams(0, 6, 1.0, 1.0))) == B.ERR_INVALID_ARG
    assert call(K=0) == B.ERR_INVALID_ARG
    assert call(K=B.MAX_LADDER + 1) == B.ERR_INVALID_ARG
    assert call(w=-1) == B.ERR_INVALID_ARG
    assert call(n_seqs=-1) == B.ERR_INVALID_ARG
    assert call(th=(ctypes.c_float * 2)(2.0, 1.0)) == B.ERR_INVALID_ARG
    assert call(ranks=(ctypes.c_int32 * 3)(8, 4, 16)) == B.ERR_INVALID_ARG
    assert call(ranks=(ctypes.c_int32 * 3)(4, 8, B.MAX_RANK + 1)) == B.ERR_INVALID_ARG
    assert call(ranks=None) == B.ERR_NULL
    assert call(state=None) == B.ERR_NULL
    assert call(gate=None) == B.ERR_NULL
    assert call(status=None) == B.ERR_NULL
    assert call(n_seqs=0, entropy=None, state=None, gate=None) == B.OK
    g = L.cwl_gated_lora_linear_packed
    d = make_desc()
    big = 1 << 30
    assert g(None, P(), P(), P(), P(), P(), big, None) == B.ERR_NULL
    assert g(d.ref(), P(0x10000), P(0x20000), None, P(0x30000), P(0x40000), big, None) == B.ERR_NULL
    assert g(d.ref(), P(0x10000), None, P(0x50000), P(0x30000), P(0x40000), big, None) == B.ERR_NULL
    assert g(d.ref(), P(0x10000), P(0x20000), P(0x50004), P(0x30000), P(0x40000), big, None) == B.ERR_INVALID_ARG
    assert g(d.ref(), P(0x10000), P(0x20000), P(0x50000), P(0x30000), P(0x40000), 16, None) == B.ERR_CAPACITY
    assert g(make_desc(group_rows=1).ref(), P(0x10000), P(0x20000), P(0x50000), P(0x30000), P(0x40000), big,
             None) == B.ERR_UNSUPPORTED
    assert g(make_desc(n_rows=0).ref(), P(), P(), P(), P(), P(), 0, None) == B.OK


def test_compose_scores_argument_errors(L):
    f = L.cwl_compose_scores
    mix = lambda **kw: ctypes.byref(B.ScoreMix(**{**dict(n=3, window=64, w_entropy=1.0, w_novelty=0.5, w_prior=0.25,
                                                          prior_len=100.0), **kw}))
    assert f(P(), P(), 10, P(), 1, None, P(), P(), None) == B.ERR_NULL
    assert f(P(), P(), -1, P(), 1, mix(), P(), P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), 10, P(), -1, mix(), P(), P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), 10, P(), 1, mix(n=0), P(), P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), 10, P(), 1, mix(window=-1), P(), P(), None) == B.ERR_INVALID_ARG
    assert f(P(), P(), 10, P(), 1, mix(n=9), P(), P(), None) == B.ERR_UNSUPPORTED
    assert f(P(), P(), 10, P(), 1, mix(window=5000), P(), P(), None) == B.ERR_UNSUPPORTED
    assert f(P(), P(), 10, P(), 1, mix(w_prior=math.nan), P(), P(), None) == B.ERR_INVALID_ARG
    assert f(None, P(), 10, P(), 1, mix(), P(), P(), None) == B.ERR_NULL
    assert f(P(), None, 10, P(), 1, mix(), P(), P(), None) == B.ERR_NULL
    assert f(P(), P(), 10, P(), 1, mix(), None, P(), None) == B.ERR_NULL
    assert f(P(), P(), 10, None, 1, mix(), P(), P(), None) == B.ERR_NULL
    assert f(None, None, 0, None, 0, mix(), None, None, None) == B.OK


def test_missing_library_is_an_error(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libcwl.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def test_budget_bucket_aligned_argument_errors(L):
    th = (ctypes.c_float * 3)(1.0, 2.0, 3.0)
    f = L.cwl_select_ranks_budget
    assert f(P(), P(), P(), 1, 8, th, 4, 0, 1, P(), None, None) == B.ERR_INVALID_ARG      # k_high < 1
    assert f(P(), P(), P(), 1, 8, th, 4, 2, -1, P(), None, None) == B.ERR_INVALID_ARG     # budget < 0
    assert f(P(), P(), P(), 1, 8, th, 0, 2, 1, P(), None, None) == B.ERR_INVALID_ARG
    assert f(P(), P(), P(), 1, 8, None, 4, 2, 1, P(), None, None) == B.ERR_NULL
    assert f(P(), P(), None, 1, 8, th, 4, 2, 1, P(), None, None) == B.ERR_NULL
    assert f(P(), P(), P(), 1, 8, th, 4, 2, 1, None, None, None) == B.ERR_NULL
    assert f(P(), P(), P(), 0, 8, th, 4, 2, 1, P(), None, None) == B.OK

    g = L.cwl_bucket_sequences
    assert g(P(), 64, P(), 2, 0, 0, P(), P(), P(), None, None) == B.ERR_INVALID_ARG        # no buckets
    assert g(P(), -1, P(), 2, 2, 0, P(), P(), P(), None, None) == B.ERR_INVALID_ARG
    assert g(P(), 64, P(), 2, 2, 0, P(), P(), P(), P(), None) == B.ERR_INVALID_ARG         # micro without n_micro
    assert g(P(), 64, P(), 4097, 2, 0, P(), P(), P(), None, None) == B.ERR_UNSUPPORTED
    assert g(P(), 64, None, 2, 2, 0, P(), P(), P(), None, None) == B.ERR_NULL
    assert g(None, 64, P(), 2, 2, 0, P(), P(), P(), None, None) == B.ERR_NULL
    assert g(P(), 64, P(), 2, 2, 0, None, P(), P(), None, None) == B.ERR_NULL
    assert g(P(), 64, P(), 0, 2, 0, None, None, None, None, None) == B.OK

    h = L.cwl_partition_chunks_aligned

    def call(l_min=4, l_max=8, n_rows=64, n_seqs=2, n_buckets=2, cap=32, ws=P(0x10000), ws_bytes=1 << 20,
             sc=P(), so=P(), bk=P(), status=P()):
        p = B.ChunkParams(l_min, l_max, math.inf, math.inf)
        return h(sc, n_rows, so, n_seqs, bk, n_buckets, ctypes.byref(p), P(), P(), P(), P(), cap, status, ws,
                 ws_bytes, None)

    assert call(l_min=0) == B.ERR_INVALID_ARG
    assert call(l_min=4, l_max=6) == B.ERR_INFEASIBLE
    assert call(n_buckets=0) == B.ERR_INVALID_ARG
    assert call(n_seqs=4097) == B.ERR_UNSUPPORTED
    assert call(n_buckets=4097) == B.ERR_UNSUPPORTED
    assert call(bk=None) == B.ERR_NULL
    assert call(so=None) == B.ERR_NULL
    assert call(sc=None) == B.ERR_NULL
    assert call(status=None) == B.ERR_NULL
    assert call(ws=None) == B.ERR_NULL
    assert call(ws=P(0x10010)) == B.ERR_INVALID_ARG
    assert call(ws_bytes=64) == B.ERR_CAPACITY
    p = B.ChunkParams(4, 8, 1.0, 1.0)
    assert L.cwl_aligned_workspace_bytes(1000, 8, 2, ctypes.byref(p)) > L.cwl_partition_workspace_bytes(1000, 2, ctypes.byref(p))
    assert L.cwl_aligned_workspace_bytes(1000, 8, 0, ctypes.byref(p)) == 0


def test_aligned_stream_step_argument_errors(L):
    f = L.cwl_stream_step_aligned
    th = (ctypes.c_float * 2)(1.0, 2.0)
    rk = (ctypes.c_int32 * 3)(4, 8, 16)
    sc = (ctypes.c_float * 3)(1.0, 1.0, 1.0)

    def call(n_seqs=4, l_min=2, l_max=4, bucket=P(), n_buckets=2, bst=P(), k_high=1, budget=0, n_high=P(),
             state=P(), gate=P(), status=P(), ent=P()):
        p = B.ChunkParams(l_min, l_max, math.inf, math.inf)
        return f(ent, n_seqs, ctypes.byref(p), th, 3, rk, sc, 1, bucket, n_buckets, bst, k_high, budget, n_high,
                 state, gate, None, None, status, None)

    assert call(l_min=3, l_max=4) == B.ERR_INFEASIBLE
    assert call(n_buckets=0) == B.ERR_INVALID_ARG
    assert call(bst=None) == B.ERR_NULL
    assert call(n_seqs=4097) == B.ERR_UNSUPPORTED
    assert call(n_buckets=4097) == B.ERR_UNSUPPORTED
    assert call(k_high=0) == B.ERR_INVALID_ARG
    assert call(budget=-1) == B.ERR_INVALID_ARG
    assert call(k_high=0, n_high=None, bucket=None, n_seqs=0) == B.OK     # budget arguments unread without n_high
    assert call(state=None) == B.ERR_NULL
    assert call(gate=None) == B.ERR_NULL
    assert call(status=None) == B.ERR_NULL
    assert call(ent=None) == B.ERR_NULL
    assert call(n_seqs=0) == B.OK


def test_build_ladder_argument_errors(L):
    f = L.cwl_build_ladder

    def call(dt=B.F32, A=P(), lda=8, Bm=P(), ldb=32, d_in=16, d_out=32, r=8, Ao=P(), ldao=8, Bo=P(), ldbo=32,
             sig=P(), ws=P(0x10000), ws_bytes=1 << 24):
        return f(dt, A, lda, Bm, ldb, d_in, d_out, r, Ao, ldao, Bo, ldbo, sig, ws, ws_bytes, None)

    assert call(dt=3) == B.ERR_INVALID_ARG
    assert call(r=0) == B.ERR_INVALID_ARG
    assert call(r=B.MAX_RANK + 1, lda=512, ldao=512) == B.ERR_INVALID_ARG
    assert call(d_in=0) == B.ERR_INVALID_ARG
    assert call(lda=7) == B.ERR_INVALID_ARG
    assert call(ldbo=31) == B.ERR_INVALID_ARG
    for k in ("A", "Bm", "Ao", "Bo", "sig", "ws"):
        assert call(**{k: None}) == B.ERR_NULL, k
    assert call(ws=P(0x10010)) == B.ERR_INVALID_ARG
    assert call(ws_bytes=1024) == B.ERR_CAPACITY
    assert L.cwl_ladder_workspace_bytes(64) >= 8 * 64 * 64 * 8
    assert L.cwl_ladder_workspace_bytes(0) == 0 and L.cwl_ladder_workspace_bytes(B.MAX_RANK + 1) == 0


def test_two_phase_and_schedule_argument_errors(L):
    """cwl_lora_shrink_packed, cwl_chunkwise_lora_linear_packed_shrunk and cwl_schedule_chunks reject bad
    arguments before anything is launched."""
    nbytes = L.cwl_lora_shrink_bytes
    assert nbytes(make_desc().ref()) >= 4 * 128 * 64            # 128 rows x 64 padded directions, fp32
    assert nbytes(make_desc(group_rows=1).ref()) == 0
    assert nbytes(make_desc(n_rows=-1).ref()) == 0

    def shrink(d, x=P(0x10000), packed=P(0x20000), u=P(0x30000), u_bytes=1 << 30):
        return L.cwl_lora_shrink_packed(d.ref(), x, packed, u, u_bytes, None)

    assert shrink(make_desc(n_rows=-1)) == B.ERR_INVALID_ARG
    assert shrink(make_desc(group_rows=1)) == B.ERR_UNSUPPORTED
    assert shrink(make_desc(n_rows=0)) == B.OK
    assert shrink(make_desc(), x=None) == B.ERR_NULL
    assert shrink(make_desc(), packed=None) == B.ERR_NULL
    assert shrink(make_desc(), u=None) == B.ERR_NULL
    assert shrink(make_desc(), u=P(0x30010)) == B.ERR_INVALID_ARG
    assert shrink(make_desc(), u_bytes=16) == B.ERR_CAPACITY

    def second(d, x=P(0x10000), packed=P(0x20000), u=P(0x30000), u_bytes=1 << 30, y=P(0x40000), ws=P(0x50000),
               ws_bytes=1 << 30):
        return L.cwl_chunkwise_lora_linear_packed_shrunk(d.ref(), x, packed, u, u_bytes, P(), 1, P(), P(), P(), P(), 8,
                                                         y, ws, ws_bytes, None)

    assert second(make_desc(n_rows=-1)) == B.ERR_INVALID_ARG
    assert second(make_desc(group_rows=1)) == B.ERR_UNSUPPORTED
    assert second(make_desc(n_rows=0)) == B.OK
    assert second(make_desc(), y=None) == B.ERR_NULL
    assert second(make_desc(), u=None) == B.ERR_NULL
    assert second(make_desc(), u_bytes=16) == B.ERR_CAPACITY
    assert second(make_desc(), ws_bytes=16) == B.ERR_CAPACITY
    assert second(make_desc(), ws=P(0x50010)) == B.ERR_INVALID_ARG

    th = (ctypes.c_float * 2)(1.0, 2.0)

    def schedule(l_min=4, l_max=8, K=3, thresholds=th, rank_idx=P(0x60000), shrink_d=None, x=P(0x10000),
                 packed=P(0x20000), u=P(0x30000), u_bytes=1 << 30, ws=P(0x70000), ws_bytes=1 << 20):
        p = B.ChunkParams(l_min, l_max, math.inf, math.inf)
        return L.cwl_schedule_chunks(P(0x1000), 64, P(0x2000), 1, ctypes.byref(p), thresholds, K, P(0x3000),
                                     P(0x4000), P(0x5000), P(0x6000), rank_idx, 32, P(0x7000), ws, ws_bytes,
                                     shrink_d.ref() if shrink_d is not None else None, x, packed, u, u_bytes, None)

    assert schedule(K=0) == B.ERR_INVALID_ARG
    assert schedule(K=B.MAX_LADDER + 1) == B.ERR_INVALID_ARG
    assert schedule(thresholds=None) == B.ERR_NULL
    assert schedule(thresholds=(ctypes.c_float * 2)(2.0, 1.0)) == B.ERR_INVALID_ARG      # descending
    assert schedule(l_min=5, l_max=8) == B.ERR_INFEASIBLE
    assert schedule(rank_idx=None) == B.ERR_NULL
    assert schedule(ws_bytes=16) == B.ERR_CAPACITY
    assert schedule(shrink_d=make_desc(group_rows=1)) == B.ERR_UNSUPPORTED
    assert schedule(shrink_d=make_desc(), u=None) == B.ERR_NULL
    assert schedule(shrink_d=make_desc(), u_bytes=16) == B.ERR_CAPACITY


def test_kv_cache_argument_errors(L):
    assert L.cwl_kv_workspace_bytes(-1) == 0
    assert L.cwl_kv_workspace_bytes(100) >= 404

    def quantise(n_heads=4, head_dim=64, k_keep=1, kv=P(0x10000), ld=256, n_rows=64, slot=P(0x20000),
                 counts=P(0x30000), codes=P(0x40000), scale=P(0x50000), cap_q=64, pool=P(0x60000), cap_f=64,
                 status=P(0x70000), ws=P(0x80000), ws_bytes=1 << 20):
        p = B.KvParams(n_heads, head_dim, k_keep)
        return L.cwl_kv_quantise_chunks(kv, ld, n_rows, P(0x1000), 1, P(0x2000), P(0x3000), P(0x4000), 32,
                                        ctypes.byref(p), slot, counts, codes, scale, cap_q, pool, cap_f, status, ws,
                                        ws_bytes, None)

    assert quantise(n_heads=0) == B.ERR_INVALID_ARG
    assert quantise(k_keep=-1) == B.ERR_INVALID_ARG
    assert quantise(head_dim=16) == B.ERR_UNSUPPORTED          # fewer than four lanes per head
    assert quantise(head_dim=96, ld=384) == B.ERR_UNSUPPORTED  # lanes per head not a power of two
    assert quantise(n_heads=32, head_dim=512, ld=16384) == B.ERR_UNSUPPORTED   # rows beyond 8192 elements
    assert quantise(ld=128) == B.ERR_INVALID_ARG               # shorter than a row
    assert quantise(ld=260) == B.ERR_UNSUPPORTED
    assert quantise(kv=None) == B.ERR_NULL
    assert quantise(slot=None) == B.ERR_NULL
    assert quantise(counts=None) == B.ERR_NULL
    assert quantise(status=None) == B.ERR_NULL
    assert quantise(codes=None) == B.ERR_NULL
    assert quantise(pool=None) == B.ERR_NULL
    assert quantise(ws=None) == B.ERR_NULL
    assert quantise(ws=P(0x80010)) == B.ERR_INVALID_ARG
    assert quantise(ws_bytes=16) == B.ERR_CAPACITY
    assert quantise(kv=P(0x10008)) == B.ERR_UNSUPPORTED
    assert quantise(n_rows=-1) == B.ERR_INVALID_ARG

    def dequantise(n_heads=4, head_dim=64, slot=P(0x20000), out=P(0x90000), ld=256, n_rows=64):
        p = B.KvParams(n_heads, head_dim, 0)
        return L.cwl_kv_dequantise(slot, n_rows, P(0x40000), P(0x50000), P(0x60000), ctypes.byref(p), out, ld, None)

    assert dequantise(head_dim=16) == B.ERR_UNSUPPORTED
    assert dequantise(ld=128) == B.ERR_INVALID_ARG
    assert dequantise(slot=None) == B.ERR_NULL
    assert dequantise(out=None) == B.ERR_NULL
    assert dequantise(n_rows=0) == B.OK
