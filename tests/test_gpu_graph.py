"""Captured-and-replayed training steps (slp_segment_set_graph) against eager launches of the
same kernels: identical bits after every step, with eager work and synchronisations between the
replays, batches that alternate (several graphs cached), a ragged batch, and set-up calls that
must drop what was captured."""

import numpy as np
import pytest
import torch

from paper_2403_11204_amd import api, datagen

pytestmark = pytest.mark.gpu
DEV = "cuda"


def twin(widths, act, loss, dtype, max_batch, wseed, **kw):
    segs = []
    for _ in range(2):
        g = api.Segment(widths, act, loss, max_batch=max_batch, dtype=dtype, lr=0.05, momentum=0.9, **kw)
        for l, (W, b) in enumerate(datagen.uniform_weights(widths, wseed)):
            g.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
        segs.append(g)
    return segs


def same_state(a, b):
    for l in range(a.L):
        Wa, ba = a.get_params(l); Wb, bb = b.get_params(l)
        va, _ = a.get_momentum(l); vb, _ = b.get_momentum(l)
        if not (torch.equal(Wa, Wb) and torch.equal(ba, bb) and torch.equal(va, vb)):
            return False
    return True


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
@pytest.mark.parametrize("loss", [api.MSE_SIL, api.SOFTMAX_XENT])
def test_replayed_steps_equal_eager_steps(dtype, loss):
    B, classes = 90, 10
    widths = [70, 130, 61] if loss == api.MSE_SIL else [70, 130, classes]
    act = api.RELU_ALL if loss == api.MSE_SIL else api.RELU_HIDDEN_IDENTITY_LAST
    eager, graph = twin(widths, act, loss, dtype, B, wseed=5)
    graph.set_graph(True)
    if loss == api.MSE_SIL:
        table = api.make_synthetic_labels(3, classes, widths[-1], api.UNIFORM01, 2.0)
        eager.set_labels(table)
        graph.set_labels(table)
    tdt = torch.bfloat16 if dtype == api.BF16 else torch.float32
    Xs, ys = [], []
    for i, rows in enumerate((B, B, 37)):                 # two full batches and a ragged one
        X, y = datagen.class_mean_inputs(rows, classes, dim=70, seed=9, first=i * B)
        Xs.append(torch.from_numpy(X).to(DEV).to(tdt).contiguous())
        ys.append(torch.from_numpy(y).to(DEV))
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    order = [0, 1, 0, 1, 2, 0, 2, 1, 0, 0]                # first step eager, then captures and replays
    with torch.cuda.stream(stream):
        for it, bi in enumerate(order):
            le = eager.step(Xs[bi], ys[bi]).clone()
            lg = graph.step(Xs[bi], ys[bi]).clone()
            filler = (Xs[bi].float() @ Xs[bi].float().t()).sum()     # the program's own eager work between replays
            if it % 3 == 2:
                torch.cuda.synchronize()
            assert torch.equal(le, lg), (it, float(le), float(lg))
            assert same_state(eager, graph), it
            assert torch.isfinite(filler)
        # a new learning rate must not be served from a graph captured with the old one
        eager.set_lr(0.01, 0.5)
        graph.set_lr(0.01, 0.5)
        for bi in (0, 1, 0):
            le = eager.step(Xs[bi], ys[bi]).clone()
            lg = graph.step(Xs[bi], ys[bi]).clone()
            assert torch.equal(le, lg) and same_state(eager, graph)
        # off again: eager launches, same results
        graph.set_graph(False)
        le, lg = eager.step(Xs[1], ys[1]).clone(), graph.step(Xs[1], ys[1]).clone()
        assert torch.equal(le, lg) and same_state(eager, graph)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()


def test_more_combinations_than_the_cache_holds():
    B, classes = 16, 5
    eager, graph = twin([12, 24, classes], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.F32, B, wseed=2)
    graph.set_graph(True)
    batches = []
    for i in range(20):                                    # the library keeps 16
        X, y = datagen.class_mean_inputs(B, classes, dim=12, seed=4, first=i * B)
        batches.append((torch.from_numpy(X).to(DEV).contiguous(), torch.from_numpy(y).to(DEV)))
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        for rnd in range(3):
            for X, y in batches:
                le, lg = eager.step(X, y).clone(), graph.step(X, y).clone()
                assert torch.equal(le, lg)
            assert same_state(eager, graph), rnd
    torch.cuda.synchronize()


def test_graph_on_the_null_stream_falls_back_to_eager_launches():
    B, classes = 16, 5
    eager, graph = twin([12, 24, classes], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.F32, B, wseed=2)
    graph.set_graph(True)
    X, y = datagen.class_mean_inputs(B, classes, dim=12, seed=4)
    X, y = torch.from_numpy(X).to(DEV).contiguous(), torch.from_numpy(y).to(DEV)
    for _ in range(3):                                     # torch's default stream is the null stream
        le, lg = eager.step(X, y).clone(), graph.step(X, y).clone()
        assert torch.equal(le, lg)
    assert same_state(eager, graph)
    assert np.isfinite(float(le))


def test_staged_epochs_replay_one_graph_and_match_eager_epochs():
    from paper_2403_11204_amd import pipeline
    B, classes, n = 64, 7, 64 * 40 + 23            # 40 full batches (more than the cache holds) and a ragged one
    eager, graph = twin([30, 50, 20], api.RELU_ALL, api.MSE_SIL, api.F32, B, wseed=11)
    table = api.make_synthetic_labels(5, classes, 20, api.UNIFORM_PM1)
    for s in (eager, graph):
        s.set_labels(table)
    graph.set_graph(True)
    X, y = datagen.class_mean_inputs(n, classes, dim=30, seed=6)
    Xd, yd = torch.from_numpy(X).to(DEV).contiguous(), torch.from_numpy(y).to(DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        le = pipeline.train_epochs(eager, Xd, yd, epochs=2, batch=B)
        lg = pipeline.train_epochs(graph, Xd, yd, epochs=2, batch=B, staged=True)
        assert le == lg
        assert same_state(eager, graph)
        # unstaged with graphs on: every batch is a new combination; the handle must fall back to eager launches
        le = pipeline.train_epochs(eager, Xd, yd, epochs=1, batch=B)
        lg = pipeline.train_epochs(graph, Xd, yd, epochs=1, batch=B)
        assert le == lg
        assert same_state(eager, graph)
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_two_replayed_segments_on_a_stream_each_equal_serial_eager_steps(dtype):
    # what `bench.py` does for the graph-replayed configurations: the two partitions are independent (paper Sec. 2), so
    # each replays its own captured step on its own stream, both in flight at once; every step of both must leave the
    # same bits as eager steps taken one after the other on one stream
    B, classes, dim = 200, 12, 96
    wa, wb = [dim, 160, 64], [64, 96, classes]
    ea, ga = twin(wa, api.RELU_ALL, api.MSE_SIL, dtype, B, wseed=21)
    eb, gb = twin(wb, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, dtype, B, wseed=22)
    table = api.make_synthetic_labels(5, classes, wa[-1], api.NORMAL, 1.0)
    ea.set_labels(table)
    ga.set_labels(table)
    ga.set_graph(True)
    gb.set_graph(True)
    tdt = torch.bfloat16 if dtype == api.BF16 else torch.float32
    batches = []
    for i in range(3):
        X, y = datagen.class_mean_inputs(B, classes, dim=dim, seed=31, first=i * B)
        yd = torch.from_numpy(y).to(DEV)
        Xa = torch.from_numpy(X).to(DEV).to(tdt).contiguous()
        Xb = (table.to(torch.float32)[yd.long()] + 0.05 * torch.randn(B, wa[-1], device=DEV)).to(tdt).contiguous()
        batches.append((Xa, Xb, yd))
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for st in (sa, sb):
        st.wait_stream(torch.cuda.current_stream())
    for it in range(9):                                   # every batch is captured once, then replayed twice
        Xa, Xb, yd = batches[it % 3]
        la_e = ea.step(Xa, yd).clone()
        lb_e = eb.step(Xb, yd).clone()
        with torch.cuda.stream(sa):
            la_g = ga.step(Xa, yd).clone()
        with torch.cuda.stream(sb):
            lb_g = gb.step(Xb, yd).clone()
        torch.cuda.synchronize()
        assert torch.equal(la_e, la_g) and torch.equal(lb_e, lb_g), it
        assert same_state(ea, ga) and same_state(eb, gb), it
