"""The launch-tracing hook and capturability of the entry points (they neither allocate nor synchronise,
so a caller may record them into a HIP graph): every replay must equal the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def _scoring_setup(w):
    d = ab.desc_from_workload(w)
    prm = ab.Params.from_workload(w, DEV)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    bufs = dict(dyn=t(w.dyn), scal=t(w.scal), part=t(w.part), cred=t(w.cred),
                scores=torch.zeros(w.S, w.C, dtype=torch.float32, device=DEV),
                idx=torch.zeros(w.S, dtype=torch.int32, device=DEV),
                best=torch.zeros(w.S, dtype=torch.float32, device=DEV),
                ws=ab.alloc_workspace(d, w.S, w.C, device=DEV))
    run = lambda: ab.ab_score_candidates(d, prm, bufs["dyn"], bufs["scal"], bufs["part"], bufs["cred"],
                                         bufs["scores"], bufs["idx"], bufs["best"], bufs["ws"])
    return bufs, run


def test_trace_hook_brackets_every_launch():
    w = wl.make_config(3, S=8)
    bufs, run = _scoring_setup(w)
    events = []
    ab.ab_set_trace(lambda name, phase, work, is_bytes: events.append((name, phase, work, is_bytes)))
    try:
        run()
    finally:
        ab.ab_set_trace(None)
    torch.cuda.synchronize()
    names = [e[0] for e in events if e[1] == 0]
    # (the feature transform and the layer-1 preparation share the first launch)
    assert names == ["encode_and_prep", "gemm_scenario_term", "gemm_hidden_first", "gemm_hidden_mid",
                     "gemm_hidden_last", "finish_select"]
    # phases alternate 0, 1 with the same name and work
    for a, b in zip(events[0::2], events[1::2]):
        assert a[1] == 0 and b[1] == 1 and a[0] == b[0] and a[2] == b[2]
    flops = {e[0]: e[2] for e in events if not e[3]}
    assert flops["gemm_hidden_mid"] == 2.0 * 8 * 256 * 1024 * 1024
    n = len(events)
    run()                                   # switched off again: nothing more is recorded
    assert len(events) == n
    with ab.KernelTimer() as kt:
        run()
        summary = kt.summary()
    assert summary["finish_select"]["launches"] == 1 and summary["gemm_hidden_mid"]["total_ms"] > 0


def test_scoring_graph_replays_equal_eager():
    w = wl.make_config(3, S=600)              # large enough for the 256 x 256 kernel (dynamic LDS attribute)
    bufs, run = _scoring_setup(w)
    run()
    torch.cuda.synchronize()
    ref = (bufs["scores"].clone(), bufs["idx"].clone(), bufs["best"].clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(3):
        bufs["scores"].zero_(); bufs["idx"].fill_(-5); bufs["best"].zero_()
        bufs["ws"].random_(0, 255)            # the workspace carries nothing over between calls
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs["scores"], ref[0]) and torch.equal(bufs["idx"], ref[1])
        assert torch.equal(bufs["best"], ref[2])


def test_update_graph_replays_equal_eager():
    u = wl.make_update("upd-graph", N=512, batch=128, L=6, hidden=(128, 64), dtype="bf16", seed=33, P=4, Q=4)
    d = ab.desc_from_workload(u)
    x, y = torch.from_numpy(u.x_raw).to(DEV), torch.from_numpy(u.target).to(DEV)
    xb = [x[i * 128:(i + 1) * 128].contiguous() for i in range(4)]
    yb = [y[i * 128:(i + 1) * 128].contiguous() for i in range(4)]

    def fresh():
        prm = ab.Params(u.W, u.b, u.dtype, DEV, trainable=True)
        return prm, ab.alloc_workspace(d, B=128, device=DEV), torch.zeros(1, dtype=torch.float32, device=DEV)

    eager, ws_e, loss_e = fresh()
    eager_losses = []
    for step in range(12):
        ab.ab_online_update(d, eager, xb[step % 4], yb[step % 4], loss_out=loss_e, workspace=ws_e)
        eager_losses.append(loss_e.clone())
    torch.cuda.synchronize()

    graphed, ws_g, loss_g = fresh()
    g = torch.cuda.CUDAGraph()
    losses = torch.zeros(4, dtype=torch.float32, device=DEV)
    with torch.cuda.graph(g):
        for i in range(4):
            ab.ab_online_update(d, graphed, xb[i], yb[i], loss_out=loss_g, workspace=ws_g)
            losses[i:i + 1].copy_(loss_g)
    for rep in range(3):                      # capture does not execute: three replays = 12 steps
        g.replay()
        torch.cuda.synchronize()
        for i in range(4):
            assert losses[i].item() == eager_losses[rep * 4 + i].item()
    for name in ("W", "b", "W_master", "mW", "vW", "mb", "vb"):
        for a, b in zip(getattr(eager, name), getattr(graphed, name)):
            assert torch.equal(a, b), name
    assert int(graphed.step.item()) == 12


def test_calls_on_two_streams_do_not_disturb_each_other():
    """The library keeps no state between or across calls: a scoring pass and update steps issued on two streams
    at the same time (each with its own buffers and workspace) give what they give one after the other."""
    w = wl.make_config(3, S=2048)             # about 2.5 ms of streaming-kernel work to overlap with
    bufs, _ = _scoring_setup(w)
    d = ab.desc_from_workload(w)
    prm = ab.Params.from_workload(w, DEV)
    u = wl.make_update("upd-two-streams", N=1024, batch=256, L=6, hidden=(128, 64), dtype="bf16", seed=35, P=4, Q=4)
    du = ab.desc_from_workload(u)
    x, y = torch.from_numpy(u.x_raw[:256]).to(DEV), torch.from_numpy(u.target[:256]).to(DEV)

    def run(s_score, s_upd):
        pu = ab.Params(u.W, u.b, u.dtype, DEV, trainable=True)
        ws_u = ab.alloc_workspace(du, B=256, device=DEV)
        loss = torch.zeros(8, dtype=torch.float32, device=DEV)
        bufs["scores"].zero_()
        torch.cuda.synchronize()
        ab.ab_score_candidates(d, prm, bufs["dyn"], bufs["scal"], bufs["part"], bufs["cred"], bufs["scores"],
                               bufs["idx"], bufs["best"], bufs["ws"], stream=s_score)
        for i in range(8):
            ab.ab_online_update(du, pu, x, y, loss_out=loss[i:i + 1], workspace=ws_u, stream=s_upd)
        torch.cuda.synchronize()
        return bufs["scores"].clone(), bufs["idx"].clone(), loss.clone(), [t.clone() for t in pu.W_master]

    one = torch.cuda.current_stream()
    serial = run(one, one)
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    both = run(a, b)
    assert torch.equal(serial[0], both[0]) and torch.equal(serial[1], both[1]) and torch.equal(serial[2], both[2])
    for p, q in zip(serial[3], both[3]):
        assert torch.equal(p, q)
    assert float(serial[2][-1]) < float(serial[2][0])
