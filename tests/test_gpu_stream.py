"""GPU parity of the decode-step form: cwl_stream_step (bit-exact integers, fp32 gate weights) and
cwl_gated_lora_linear_packed against the CPU oracle (Sec. III-A/B/F, III-C/D)."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from helpers import TOL_BF16, TOL_F32, host, rel_err
from paper_2601_21109_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gate_fields(gate):
    g = gate.cpu().numpy()
    return g[:, 0].copy(), g[:, 1].copy(), g[:, 2].copy().view(np.float32), g[:, 3].copy().view(np.float32)


def make_gate(r_cur, r_prev, g_cur, g_prev):
    g = np.empty((len(r_cur), 4), np.int32)
    g[:, 0], g[:, 1] = r_cur, r_prev
    g[:, 2] = np.asarray(g_cur, np.float32).view(np.int32)
    g[:, 3] = np.asarray(g_prev, np.float32).view(np.int32)
    return torch.from_numpy(g).to(DEV)


@pytest.mark.parametrize("n_seqs,steps,l_min,l_max,w,ladder", [
    (37, 300, 4, 9, 2, ([4, 8, 16], [4.0, 2.0, 1.0])),
    (300, 120, 8, 64, 4, ([8, 16, 32, 64], [2.0, 1.0, 0.5, 0.25])),
    (1, 400, 1, 1, 0, ([0, 5], [7.0, 3.2])),
    (5, 200, 3, 40, 3, ([16], [1.0])),
    (33, 150, 4, 16, 3, (list(range(0, 256, 16)), [0.0] + [16.0 / r for r in range(16, 256, 16)])),   # 16 rungs
])
def test_stream_step_matches_oracle(n_seqs, steps, l_min, l_max, w, ladder):
    ranks, scales = ladder
    K = len(ranks)
    vocab_ln = math.log(32000.0)
    theta, delta = 0.9 * vocab_ln, 0.3 * vocab_ln
    taus = [vocab_ln * f for f in np.linspace(0.3, 0.9, K - 1)] if K > 1 else []
    rng = np.random.RandomState(n_seqs)
    # spans of three difficulty levels per sequence, with noise, some exactly on thresholds
    level = rng.choice([0.15, 0.5, 0.95], size=(n_seqs, steps // 10 + 1)).repeat(10, axis=1)[:, :steps]
    h_all = (level * vocab_ln + rng.uniform(-0.4, 0.4, size=(n_seqs, steps))).astype(np.float32)
    h_all[:, 7] = np.float32(theta)
    state = B.stream_state(n_seqs, DEV)
    ost = O.StreamState(n_seqs)
    tq = [O.quantise_threshold(t) for t in taus]
    dev_out = []
    for t in range(steps):
        h = torch.from_numpy(h_all[:, t].copy()).to(DEV)
        out = B.stream_step(h, state, l_min, l_max, theta, delta, taus, ranks, scales, w)
        dev_out.append({k: v.clone() for k, v in out.items()})
    torch.cuda.synchronize()
    for t in range(steps):
        q, nan_seen = O.quantise(h_all[:, t])
        assert not nan_seen
        code, ref = O.stream_step(ost, q, l_min, l_max, O.quantise_threshold(theta), O.quantise_threshold(delta),
                                  tq, ranks, scales, w)
        assert code == 0
        r_cur, r_prev, g_cur, g_prev = gate_fields(dev_out[t]["gate"])
        assert np.array_equal(r_cur, ref["r_cur"]) and np.array_equal(r_prev, ref["r_prev"]), t
        assert np.array_equal(dev_out[t]["closed_len"].cpu().numpy(), ref["closed_len"]), t
        assert np.array_equal(dev_out[t]["closed_sum"].cpu().numpy(), ref["closed_sum"]), t
        np.testing.assert_allclose(g_cur, ref["g_cur"], rtol=1e-6, atol=0)
        np.testing.assert_allclose(g_prev, ref["g_prev"], rtol=1e-6, atol=0)
        assert int(dev_out[t]["status_word"].item()) == 0
    f = B.stream_state_fields(state)
    assert np.array_equal(f["n"], ost.n) and np.array_equal(f["sum"], ost.sum)
    assert np.array_equal(f["k_cur"], ost.k_cur) and np.array_equal(f["n_chunks"], ost.chunks)
    assert np.array_equal(f["pos"], ost.pos)
    closed = ost.chunks > 0
    assert np.array_equal(f["k_prev"][closed], ost.k_prev[closed])
    assert ost.chunks.sum() > 0


def test_stream_step_nan_score_and_no_sequences():
    state = B.stream_state(3, DEV)
    h = torch.tensor([1.0, float("nan"), 2.0], device=DEV)
    out = B.stream_step(h, state, 2, 4, math.inf, math.inf, [1.5], [4, 8], [1.0, 0.5], 0)
    torch.cuda.synchronize()
    assert int(out["status_word"].item()) == B.STATUS_NAN_SCORE
    f = B.stream_state_fields(state)
    assert f["sum"].tolist() == [1024, 0, 2048] and f["n"].tolist() == [1, 1, 1]
    empty = B.stream_step(torch.empty(0, device=DEV), B.stream_state(0, DEV), 2, 4, 1.0, 1.0, [1.5], [4, 8],
                          [1.0, 0.5], 0)
    assert empty["gate"].shape == (0, 4)


@pytest.mark.parametrize("n,d_in,d_out,r_max,dtype,tol", [
    (1, 4096, 4096, 64, torch.bfloat16, TOL_BF16),
    (8, 1024, 1032, 64, torch.bfloat16, TOL_BF16),
    (33, 512, 72, 100, torch.bfloat16, TOL_BF16),
    (200, 704, 520, 16, torch.bfloat16, TOL_BF16),
    (600, 256, 264, 40, torch.bfloat16, TOL_BF16),      # tiled path, gate supplied by the caller
    (70, 100, 72, 12, torch.float32, TOL_F32),
])
def test_gated_linear_matches_oracle(n, d_in, d_out, r_max, dtype, tol):
    g = torch.Generator(device=DEV).manual_seed(n)
    x = torch.randn((n, d_in), generator=g, device=DEV).to(dtype)
    Wm = (torch.randn((d_in, d_out), generator=g, device=DEV) / math.sqrt(d_in)).to(dtype)
    A = (torch.randn((d_in, r_max), generator=g, device=DEV) / math.sqrt(d_in)).to(dtype)
    Bm = (torch.randn((r_max, d_out), generator=g, device=DEV) / math.sqrt(r_max)).to(dtype)
    rng = np.random.RandomState(n)
    r_cur = rng.randint(0, r_max + 1, n)
    r_prev = np.where(rng.rand(n) < 0.5, rng.randint(0, r_max + 1, n), 0)
    g_cur = rng.uniform(0.1, 2.0, n).astype(np.float32)
    g_prev = np.where(r_prev > 0, rng.uniform(0.1, 2.0, n), 0.0).astype(np.float32)
    pw = B.prepack_weights(Wm, A, Bm)
    y = B.gated_lora_linear(x, pw, make_gate(r_cur, r_prev, g_cur, g_prev), [r_max], [1.0])
    torch.cuda.synchronize()
    ref = O.gated_linear(host(x), host(Wm), host(A), host(Bm), r_cur, g_cur.astype(np.float64), r_prev,
                         g_prev.astype(np.float64))
    assert rel_err(host(y), ref) <= tol
    # ranks outside [0, r_max] are clipped
    y2 = B.gated_lora_linear(x, pw, make_gate(np.where(r_cur == r_max, r_max + 50, r_cur), r_prev - (r_prev == 0) * 3,
                                              g_cur, g_prev), [r_max], [1.0])
    assert torch.equal(y, y2)


def test_decode_steps_end_to_end():
    """score_tokens -> stream_step -> gated linear for a few decode steps of 16 sequences, each stage
    against the oracle fed with the device's own output of the stage before."""
    n_seqs, vocab, d_in, d_out, r_max = 16, 2000, 512, 264, 32
    ranks, scales = [8, 16, 32], [2.0, 1.0, 0.5]
    lnv = math.log(vocab)
    theta, delta, taus = 0.9 * lnv, 0.3 * lnv, [0.45 * lnv, 0.9 * lnv]
    g = torch.Generator(device=DEV).manual_seed(3)
    Wm = (torch.randn((d_in, d_out), generator=g, device=DEV) / math.sqrt(d_in)).to(torch.bfloat16)
    A = (torch.randn((d_in, r_max), generator=g, device=DEV) / math.sqrt(d_in)).to(torch.bfloat16)
    Bm = (torch.randn((r_max, d_out), generator=g, device=DEV) / math.sqrt(r_max)).to(torch.bfloat16)
    pw = B.prepack_weights(Wm, A, Bm)
    state = B.stream_state(n_seqs, DEV)
    ost = O.StreamState(n_seqs)
    for step in range(12):
        sigma = torch.tensor([0.5, 2.0, 6.0], device=DEV)[torch.randint(0, 3, (n_seqs, 1), generator=g, device=DEV)]
        logits = (torch.randn((n_seqs, vocab), generator=g, device=DEV) * sigma).to(torch.bfloat16)
        x = torch.randn((n_seqs, d_in), generator=g, device=DEV).to(torch.bfloat16)
        h = B.score_tokens(logits)
        out = B.stream_step(h, state, 2, 4, theta, delta, taus, ranks, scales, 2)
        y = B.gated_lora_linear(x, pw, out["gate"], ranks, scales)
        torch.cuda.synchronize()
        q, _ = O.quantise(host(h))
        _, ref = O.stream_step(ost, q, 2, 4, O.quantise_threshold(theta), O.quantise_threshold(delta),
                               [O.quantise_threshold(t) for t in taus], ranks, scales, 2)
        r_cur, r_prev, g_cur, g_prev = gate_fields(out["gate"])
        assert np.array_equal(r_cur, ref["r_cur"]) and np.array_equal(r_prev, ref["r_prev"])
        yref = O.gated_linear(host(x), host(Wm), host(A), host(Bm), r_cur, g_cur.astype(np.float64), r_prev,
                              g_prev.astype(np.float64))
        assert rel_err(host(y), yref) <= TOL_BF16
    assert ost.chunks.sum() > 0


@pytest.mark.parametrize("n_seqs", [8, 1])        # one sequence: the projections run as matrix-vector products
def test_decode_step_replays_from_a_hip_graph(n_seqs):
    """The calls only enqueue kernels on the caller's stream, so a decode step (scores, scheduler step,
    two projections) can be captured once and replayed.  Every replay, with eager work and
    synchronisations in between, must equal the eager result for the same inputs and state."""
    vocab, d_in, d_out, r_max = 1500, 256, 320, 16
    ranks, scales = [4, 8, 16], [4.0, 2.0, 1.0]
    lnv = math.log(vocab)
    args = (2, 4, 0.9 * lnv, 0.3 * lnv, [0.45 * lnv, 0.9 * lnv], ranks, scales, 2)
    g = torch.Generator(device=DEV).manual_seed(9)
    mk = lambda *s: (torch.randn(s, generator=g, device=DEV) / math.sqrt(s[0])).to(torch.bfloat16)
    pw1 = B.prepack_weights(mk(d_in, d_out), mk(d_in, r_max), mk(r_max, d_out))
    pw2 = B.prepack_weights(mk(d_out, d_in), mk(d_out, r_max), mk(r_max, d_in))
    logits = torch.empty((n_seqs, vocab), dtype=torch.bfloat16, device=DEV)
    x = torch.empty((n_seqs, d_in), dtype=torch.bfloat16, device=DEV)
    h = torch.empty(n_seqs, dtype=torch.float32, device=DEV)
    state = B.stream_state(n_seqs, DEV)
    y1 = torch.empty((n_seqs, d_out), dtype=torch.bfloat16, device=DEV)
    y2 = torch.empty((n_seqs, d_in), dtype=torch.bfloat16, device=DEV)
    ws1 = B.linear_workspace((n_seqs, d_in), torch.bfloat16, d_out, r_max, ranks, scales, 0, DEV)
    ws2 = B.linear_workspace((n_seqs, d_out), torch.bfloat16, d_in, r_max, ranks, scales, 0, DEV)
    out = B.stream_step(h, state, *args)            # allocates the outputs once, outside the graph

    def step():
        B.score_tokens(logits, out=h)
        B.stream_step(h, state, *args, out=out)
        B.gated_lora_linear(x, pw1, out["gate"], ranks, scales, out=y1, workspace=ws1)
        B.gated_lora_linear(y1, pw2, out["gate"], ranks, scales, out=y2, workspace=ws2)

    def new_inputs(i):
        gi = torch.Generator(device=DEV).manual_seed(100 + i)
        sigma = torch.tensor([0.5, 2.0, 6.0], device=DEV)[torch.randint(0, 3, (n_seqs, 1), generator=gi, device=DEV)]
        logits.copy_((torch.randn((n_seqs, vocab), generator=gi, device=DEV) * sigma).to(torch.bfloat16))
        x.copy_(torch.randn((n_seqs, d_in), generator=gi, device=DEV).to(torch.bfloat16))

    # eager reference run over 6 steps
    state.zero_()
    eager = []
    for i in range(6):
        new_inputs(i)
        step()
        torch.cuda.synchronize()
        eager.append((y2.clone(), state.clone(), out["gate"].clone()))
    # captured run
    state.zero_()
    new_inputs(0)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                       # warm-up on the capture stream
        state.zero_()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in range(6):
        new_inputs(i)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y2, eager[i][0]), i
        assert torch.equal(state, eager[i][1]) and torch.equal(out["gate"], eager[i][2]), i
        _ = (x.float() @ x.float().t()).sum().item()    # unrelated eager work between replays
