"""Steps whose parameter updates are left running beside the caller's next work (slp_segment_set_overlap) against
ordinary steps: identical bits after every step, for two segments stepped alternately on one stream (the use the
switch is for), with reads through the interface, forward passes, an explicit join and a destroy in between."""

import pytest
import torch

from paper_2403_11204_amd import api, datagen

pytestmark = pytest.mark.gpu
DEV = "cuda"


def build(widths, act, loss, dtype, B, wseed, overlap):
    g = api.Segment(widths, act, loss, max_batch=B, dtype=dtype, lr=0.05, momentum=0.9)
    for l, (W, b) in enumerate(datagen.uniform_weights(widths, wseed)):
        g.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
    g.set_overlap(overlap)
    return g


def same_state(a, b):
    for l in range(a.L):
        Wa, ba = a.get_params(l); Wb, bb = b.get_params(l)
        va, _ = a.get_momentum(l); vb, _ = b.get_momentum(l)
        if not (torch.equal(Wa, Wb) and torch.equal(ba, bb) and torch.equal(va, vb)):
            return False
    return True


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_overlapped_steps_equal_ordinary_steps(dtype):
    B, classes = 300, 12
    wl, wr = [96, 2304, 2100, 130], [130, 2200, classes]      # layers large enough for the side-stream update path
    tdt = torch.bfloat16 if dtype == api.BF16 else torch.float32
    table = api.make_synthetic_labels(3, classes, wl[-1], api.NORMAL, 1.0)
    pairs = []
    for overlap in (False, True):
        left = build(wl, api.RELU_ALL, api.MSE_SIL, dtype, B, 5, overlap)
        right = build(wr, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, dtype, B, 6, overlap)
        left.set_labels(table)
        pairs.append((left, right))
    Xs, ys, Rs = [], [], []
    for i in range(3):
        X, y = datagen.class_mean_inputs(B, classes, dim=wl[0], seed=9, first=i * B)
        Xs.append(torch.from_numpy(X).to(DEV).to(tdt).contiguous())
        ys.append(torch.from_numpy(y).to(DEV))
        Rs.append(api.make_segment_inputs(11, table, ys[-1], i * B, 0.05, dtype))
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        for it in range(7):
            bi = it % 3
            losses = []
            for left, right in pairs:                       # left and right alternate on one stream
                ll = left.step(Xs[bi], ys[bi]).clone()
                lr = right.step(Rs[bi], ys[bi]).clone()
                losses.append((ll, lr))
            assert torch.equal(losses[0][0], losses[1][0]) and torch.equal(losses[0][1], losses[1][1]), it
            if it == 2:                                     # a forward pass right behind an overlapped step
                o0 = pairs[0][0].forward(Xs[0]); o1 = pairs[1][0].forward(Xs[0])
                assert torch.equal(o0, o1)
            if it == 4:
                pairs[1][0].join(); pairs[1][1].join()      # explicit joins change nothing
            assert same_state(pairs[0][0], pairs[1][0]) and same_state(pairs[0][1], pairs[1][1]), it
    stream.synchronize()


def test_destroy_right_after_an_overlapped_step():
    B, classes = 128, 10
    widths = [64, 2304, 2100, classes]
    g = build(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.BF16, B, 7, True)
    X, y = datagen.class_mean_inputs(B, classes, dim=widths[0], seed=2)
    Xd = torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous()
    yd = torch.from_numpy(y).to(DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        for _ in range(3):
            g.step(Xd, yd)
        del g                                               # waits for the updates still running on the handle's stream
    torch.cuda.synchronize()
    # the device is healthy and a fresh handle works
    h = build(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.BF16, B, 7, False)
    assert torch.isfinite(h.step(Xd, yd)).all()


def test_recovery_steps_with_overlap_equal_ordinary_ones():
    # Sec. 5's loop (left forward, right input gradient, left step from that gradient) with overlap on for the left
    # partition: step_external leaves its updates running, the next forward on the handle waits for them
    B, classes = 256, 9
    wl, wr = [80, 2304, 2100, 64], [64, 96, classes]
    states = []
    for overlap in (False, True):
        left = build(wl, api.RELU_ALL, api.MSE_SIL, api.F32, B, 3, overlap)
        right = api.Segment(wr, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, max_batch=B, dtype=api.F32, lr=0.05,
                            momentum=0.9, input_grad=True)
        for l, (W, b) in enumerate(datagen.uniform_weights(wr, 4)):
            right.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            for it in range(4):
                X, y = datagen.class_mean_inputs(B, classes, dim=wl[0], seed=5, first=it * B)
                Xd, yd = torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV)
                resp = left.forward(Xd)
                d_resp, _ = right.input_grad(resp, yd)
                left.step_external(Xd, d_resp)
            states.append([left.get_params(l)[0].clone() for l in range(left.L)])
        stream.synchronize()
    for a, b in zip(*states):
        assert torch.equal(a, b)


def test_a_second_stream_between_overlapped_steps():
    # step on stream A with the join deferred, read the parameters on stream B (ordered after A by the caller), step on
    # A again: both streams have to wait for the pending updates, not only the first that touches the handle
    B, classes = 256, 10
    widths = [64, 2304, 2100, classes]
    X, y = datagen.class_mean_inputs(B, classes, dim=widths[0], seed=2)
    Xd = torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous()
    yd = torch.from_numpy(y).to(DEV)
    finals = []
    for overlap in (False, True):
        g = build(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.BF16, B, 7, overlap)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        sa.wait_stream(torch.cuda.current_stream())
        reads = []
        for _ in range(4):
            with torch.cuda.stream(sa):
                g.step(Xd, yd)
            sb.wait_stream(sa)
            with torch.cuda.stream(sb):
                reads.append(g.get_params(1)[0].clone())
            # nothing orders A behind B here: the library's own wait is what keeps the next step behind the updates
        sa.synchronize(); sb.synchronize()
        with torch.cuda.stream(sa):
            g.set_overlap(False)                            # waits on the host; the handle is in plain stream order again
            reads.append(g.get_params(0)[0].clone())
        sa.synchronize()
        finals.append(reads)
        del g
    for a, b in zip(*finals):
        assert torch.equal(a, b)


def test_capturing_stream_with_pending_updates_is_refused():
    B, classes = 128, 10
    widths = [64, 2304, 2100, classes]
    g = build(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.BF16, B, 7, True)
    X, y = datagen.class_mean_inputs(B, classes, dim=widths[0], seed=2)
    Xd = torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous()
    yd = torch.from_numpy(y).to(DEV)
    out = torch.empty(B, classes, dtype=torch.bfloat16, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        g.step(Xd, yd)
        g.step(Xd, yd)                                      # leaves its updates pending
        graph = torch.cuda.CUDAGraph()
        with pytest.raises(api.SlpError) as ei:
            with torch.cuda.graph(graph, stream=stream, capture_error_mode="thread_local"):
                g.forward(Xd, out=out)
        assert ei.value.code == -5      # SLP_ERR_STATE
        g.set_overlap(False)                                # host wait: now the same capture is fine
        ref = g.forward(Xd).clone()
        graph2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph2, stream=stream, capture_error_mode="thread_local"):
            g.forward(Xd, out=out)
        out.zero_()
        graph2.replay()
        stream.synchronize()
        assert torch.equal(out, ref)
