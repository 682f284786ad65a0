"""The library's calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a serving loop can record them into a HIP graph.  Each case records one call,
replays it several times with eager work and synchronisations in between, and compares every replay
with the eager result bit for bit.  Needs an MI355X."""
import pytest
import torch

from paper_2605_14292_amd import workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def B():
    from paper_2605_14292_amd import binding
    return binding


def _tensors(out):
    return {k: v for k, v in vars(out).items() if isinstance(v, torch.Tensor)}


def _replay_and_compare(call, make_out):
    ref = make_out()
    call(ref)                                   # eager result; also the first-use set-up of the library
    torch.cuda.synchronize()
    out = make_out()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(out)
    for rep in range(3):
        for name, t in _tensors(out).items():   # eager work between the replays: spoil the outputs
            if name in ("K_out", "V_out"):
                t.zero_()                        # (rows past a head's budget are never written and stay zero)
            else:
                t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in _tensors(out).items():
            want = getattr(ref, name)
            assert torch.equal(t.view(torch.int16) if t.dtype == torch.bfloat16 else t,
                               want.view(torch.int16) if want.dtype == torch.bfloat16 else want), (rep, name)


def test_one_decode_event_replays_from_a_graph():
    w = W.WORKLOADS["c2"]
    data = W.generate(w, seed=3, device=DEV)
    b = B()
    lay = b.layout_of(data["K"])
    _replay_and_compare(
        lambda out: b.kvr_retain(data["K"], data["V"], w.b, w.lam, 1e-6, Q=data["Q"], out=out),
        lambda: b.RetainBuffers(lay.heads, lay.n, w.b, lay.d, data["K"].dtype, DEV, True))


def test_long_heads_replay_from_a_graph():
    w = W.WORKLOADS["c5"]
    data = W.generate(w, heads=40, seed=3, device=DEV)
    b = B()
    lay = b.layout_of(data["K"])
    _replay_and_compare(
        lambda out: b.kvr_retain(data["K"], data["V"], w.b, w.lam, 1e-6, Q=data["Q"], out=out),
        lambda: b.RetainBuffers(lay.heads, lay.n, w.b, lay.d, data["K"].dtype, DEV, True))


def test_batched_event_with_given_scores_replays_from_a_graph():
    w = W.WORKLOADS["c3"]
    data = W.generate(w, heads=600, seed=3, device=DEV)
    b = B()
    lay = b.layout_of(data["K"])
    _replay_and_compare(
        lambda out: b.kvr_retain(data["K"], data["V"], w.b, w.lam, 1e-6, s=data["s"], out=out),
        lambda: b.RetainBuffers(lay.heads, lay.n, w.b, lay.d, data["K"].dtype, DEV, False))


def test_flat_mode_and_budgeted_frame_replay_from_a_graph():
    w = W.WORKLOADS["c3"]
    data = W.generate(w, heads=64, seed=4, device=DEV)
    b = B()
    lay = b.layout_of(data["K"])
    s_seq = data["s"][::8].contiguous()
    _replay_and_compare(
        lambda out: b.kvr_retain_flat(data["K"], data["V"], s_seq, 8, w.b, w.lam, 1e-6, out=out),
        lambda: b.FlatBuffers(lay.heads, 8, lay.n, w.b, lay.d, data["K"].dtype, DEV))
    g = torch.Generator().manual_seed(5)
    b_h = torch.randint(0, w.b + 1, (lay.heads,), generator=g, dtype=torch.int32).to(DEV)
    n_h = torch.randint(w.b, lay.n + 1, (lay.heads,), generator=g, dtype=torch.int32).to(DEV)
    keep = torch.zeros((lay.heads, lay.n), dtype=torch.uint8)
    keep[:, :4] = 1
    keep = keep.to(DEV)
    _replay_and_compare(
        lambda out: b.kvr_retain_budgeted(data["K"], data["V"], w.b, w.lam, 1e-6, s=data["s"], n_h=n_h, b_h=b_h,
                                          keep=keep, out=out),
        lambda: b.BudgetBuffers(lay.heads, lay.n, w.b, lay.d, data["K"].dtype, DEV))
