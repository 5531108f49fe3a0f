"""The training step captured into a HIP graph: every launch of the step is a kernel on the caller's
stream and the library allocates nothing once warmed up, so the step can be captured and replayed.
Replays are checked against eager steps from the same start, with eager work between the replays."""
import numpy as np
import pytest

from paper_1702_03192_amd import binding as mt
from test_gpu_fc import make_net

pytestmark = pytest.mark.gpu


def _state(dims, batch, X, labels, W, b, lr, mode):
    import torch
    t = {"X": torch.from_numpy(X).cuda(), "labels": torch.from_numpy(labels).cuda(),
         "W": [torch.from_numpy(w.copy()).cuda() for w in W], "b": [torch.from_numpy(v.copy()).cuda() for v in b]}
    t["gW"] = [torch.empty_like(w) for w in t["W"]]
    t["gb"] = [torch.empty_like(v) for v in t["b"]]
    t["loss"] = torch.zeros(1, device="cuda")
    t["logits"] = torch.empty((batch, dims[-1]), device="cuda")
    t["ws"] = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
    t["desc"], t["keep"] = mt.make_fc_desc(dims, batch, t["X"], t["labels"], t["W"], t["b"], t["gW"], t["gb"],
                                           t["loss"], t["ws"], lr, mode, t["logits"])
    return t


@pytest.mark.parametrize("mode", [1, -1], ids=["nt", "tnn"])
def test_training_step_replayed_from_a_graph_matches_eager_steps(mode):
    import torch
    dims, batch, steps = [96, 512, 256, 10], 128, 4
    X, labels, W, b = make_net(dims, batch, 5400)
    stream = torch.cuda.Stream()
    eager = _state(dims, batch, X, labels, W, b, 0.05, mode)
    losses = []
    with torch.cuda.stream(stream):
        for _ in range(steps):
            mt.mtnn_fc_train_step(eager["desc"])
            losses.append(eager["loss"].clone())
    stream.synchronize()
    want_losses = [float(v.item()) for v in losses]
    assert want_losses[-1] < want_losses[0]                       # the steps do change the weights

    warm = _state(dims, batch, X, labels, W, b, 0.05, mode)       # same shapes: one-time set-up happens here
    with torch.cuda.stream(stream):
        mt.mtnn_fc_train_step(warm["desc"])
    stream.synchronize()

    g = _state(dims, batch, X, labels, W, b, 0.05, mode)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        mt.mtnn_fc_train_step(g["desc"])
    # capture does not run anything: weights are still the initial ones
    assert torch.equal(g["W"][0], torch.from_numpy(W[0]).cuda())
    got_losses = []
    scratch = torch.zeros(1 << 20, device="cuda")
    for i in range(steps):
        graph.replay()
        torch.cuda.synchronize()
        got_losses.append(float(g["loss"].item()))
        scratch.add_(1.0)                                          # unrelated eager work between replays
        assert float(scratch.sum().item()) == (i + 1) * (1 << 20)
    assert got_losses == want_losses
    for l in range(len(dims) - 1):
        assert torch.equal(g["W"][l], eager["W"][l]) and torch.equal(g["b"][l], eager["b"][l])
        assert torch.equal(g["gW"][l], eager["gW"][l])
    assert torch.equal(g["logits"], eager["logits"])
