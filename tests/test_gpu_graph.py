"""The classical step (Sec. III Eq. 1 encoding, class-vector accumulation and majority, Hamming
search) captured once in a HIP graph and replayed: every library call only launches kernels on the
stream it is given (tables and scratch are allocated at create), so a serving loop can record the
step and replay it.  Each replay runs on new inputs, with eager work and synchronisations between
the replays, and is compared with the eager calls on the same inputs; the first one also with the
CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402


def test_classical_step_replayed_from_a_graph():
    from paper_2206_04746_amd import binding
    ntr, nte = 2048, 600
    wl = make_workload(2, seed=77, n_train=ntr, n_test=nte)
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    dev = "cuda"
    x_tr, y_tr = wl.train(ntr)
    x_te, _ = wl.test(nte)
    xt = torch.from_numpy(x_tr).to(dev)
    yt = torch.from_numpy(y_tr.astype(np.int32)).to(dev)
    xs = torch.from_numpy(x_te).to(dev)

    def buffers():
        return dict(hv_t=torch.empty((ntr, ctx.W), dtype=torch.int32, device=dev),
                    hv_s=torch.empty((nte, ctx.W), dtype=torch.int32, device=dev),
                    acc=torch.empty((wl.C, wl.D), dtype=torch.int32, device=dev),
                    cn=torch.empty((wl.C,), dtype=torch.int64, device=dev),
                    cls=torch.empty((wl.C, ctx.W), dtype=torch.int32, device=dev),
                    pred=torch.empty((nte,), dtype=torch.int32, device=dev),
                    dist=torch.empty((nte, wl.C), dtype=torch.int32, device=dev))

    def step(b):
        ctx.hdc_encode(xt, b["hv_t"])
        b["acc"].zero_()
        b["cn"].zero_()
        ctx.hdc_train_classical(b["hv_t"], yt, b["acc"], b["cn"])
        ctx.hdc_binarize_classical(b["acc"], b["cn"], b["cls"])
        ctx.hdc_encode(xs, b["hv_s"])
        ctx.hdc_search(b["hv_s"], b["cls"], b["pred"], b["dist"])

    eager, replay = buffers(), buffers()
    step(replay)                      # (first calls done before the capture)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(replay)
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    for round_ in range(4):
        if round_:                    # new inputs in the captured buffers
            xt.copy_(torch.from_numpy(np.roll(x_tr, round_, axis=0).copy()).to(dev))
            yt.copy_(torch.from_numpy(np.roll(y_tr, round_).astype(np.int32)).to(dev))
            xs.copy_(torch.from_numpy((x_te + rng.normal(0, 0.05, x_te.shape)).astype(x_te.dtype)).to(dev))
        for v in replay.values():
            v.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        step(eager)                   # eager work between the replays
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(eager[k], replay[k]), (round_, k)
        if round_ == 0:
            hv = oracle.encode(x_tr, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
            assert np.array_equal(replay["hv_t"].cpu().numpy().view(np.uint32), hv)
    ctx.close()
