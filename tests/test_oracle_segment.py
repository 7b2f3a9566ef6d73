"""Pins for the oracle's segment training step (paper Sec. 2 and 3).  CPU only.

Each test fixes the oracle to something other than itself: numbers the paper
prints, hand arithmetic, closed forms, finite differences, or an automatic-
differentiation library run in float64."""

import math
import os

import numpy as np
import pytest
import torch

from oracle import rng
from oracle import segment as osg
from paper_2403_11204_amd import datagen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ACTS = {"relu_all": osg.RELU_ALL, "identity_last": osg.RELU_HIDDEN_IDENTITY_LAST}


def _rand_segment(widths, act, loss, seed, **kw):
    seg = osg.Segment(widths, act, loss, **kw)
    for l, (W, b) in enumerate(datagen.uniform_weights(widths, seed)):
        seg.set_params(l, W, b)
    return seg


# ---------------------------------------------------------------------------------
# numbers the paper prints (Sec. 3)
# ---------------------------------------------------------------------------------
def test_paper_parameter_and_mac_counts():
    seen = 0
    for line in open(os.path.join(GOLDEN, "paper_sec3_counts.txt")):
        f = line.split()
        if not f or f[0] not in ("left", "right"):
            continue
        widths = [int(x) for x in f[1].split(",")]
        assert osg.param_count(widths) == int(f[3])
        assert osg.mac_count(widths, ACTS[f[2]]) == int(f[4])
        seen += 1
    assert seen == 2
    # the cut layer carries a ReLU, the network's last layer does not: flipping
    # either convention breaks the printed MAC counts
    assert osg.mac_count([784, 80, 60], osg.RELU_HIDDEN_IDENTITY_LAST) != 67800
    assert osg.mac_count([60, 60, 60, 47], osg.RELU_ALL) != 10307
    assert osg.gemm_flops_per_sample([784, 1024, 1024, 512]) == 12648448


# ---------------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------------
def test_forward_hand_worked():
    # 2 -> 2 -> 1, worked by hand
    seg = osg.Segment([2, 2, 1], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT)
    seg.set_params(0, np.array([[1.0, -2.0], [0.5, 0.25]]), np.array([0.5, -1.0]))
    seg.set_params(1, np.array([[2.0, -3.0]]), np.array([0.25]))
    X = np.array([[1.0, 1.0], [2.0, 4.0]])
    # row 0: z1 = (1-2+.5, .5+.25-1) = (-.5, -.25) -> a1 = (0,0) -> z2 = .25
    # row 1: z1 = (2-8+.5, 1+1-1) = (-5.5, 1) -> a1 = (0,1) -> z2 = -3+.25 = -2.75
    A, Z = seg.forward_all(X)
    assert np.array_equal(Z[1], [[-0.5, -0.25], [-5.5, 1.0]])
    assert np.array_equal(A[1], [[0.0, 0.0], [0.0, 1.0]])
    assert np.array_equal(A[2], [[0.25], [-2.75]])
    # same weights, ReLU on the last layer too
    seg2 = osg.Segment([2, 2, 1], osg.RELU_ALL, osg.MSE_SIL)
    seg2.set_params(0, seg.W[0], seg.b[0])
    seg2.set_params(1, seg.W[1], seg.b[1])
    assert np.array_equal(seg2.forward(X), [[0.25], [0.0]])


def test_forward_special_weights():
    g = np.random.default_rng(0)
    X = g.standard_normal((5, 6))
    seg = osg.Segment([6, 6, 6], osg.RELU_ALL, osg.MSE_SIL)
    bias = g.standard_normal(6)
    seg.set_params(1, np.zeros((6, 6)), bias)             # W = 0 -> act(b)
    assert np.array_equal(seg.forward(X), np.tile(np.maximum(bias, 0), (5, 1)))
    seg.set_params(0, np.eye(6), np.zeros(6))             # identity -> relu(x)
    seg.set_params(1, np.eye(6), np.zeros(6))
    assert np.array_equal(seg.forward(X), np.maximum(X, 0))
    # W is [out, in]: a non-square, non-symmetric case catches a transposed operand
    seg = osg.Segment([3, 2], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT)
    seg.set_params(0, np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 0.5]]), np.zeros(2))
    assert np.array_equal(seg.forward(np.array([[1.0, 10.0, 100.0]])), [[321.0, 40.0]])


# ---------------------------------------------------------------------------------
# losses: closed forms and brute force
# ---------------------------------------------------------------------------------
def test_mse_closed_forms():
    T = rng.make_synthetic_labels(13, 47, 32, rng.BINARY_PM1).astype(np.float64)
    y = datagen.balanced_classes(20, 47)
    seg = osg.Segment([8, 32], osg.RELU_ALL, osg.MSE_SIL)       # W = 0, b = 0
    out = seg.step(np.ones((20, 8)), y, T, update=False)
    assert out["loss"] == 1.0                                    # mean of (+-1)^2
    assert np.all(out["dZ"][1] == 0)                             # ReLU'(0) = 0
    # brute force with python loops on random activations
    g = np.random.default_rng(1)
    AL = g.standard_normal((4, 5))
    Tt = g.standard_normal((3, 5))
    yy = np.array([2, 0, 2, 1])
    loss, G = seg.loss_and_grad(AL, yy, Tt)
    s = 0.0
    for n in range(4):
        for i in range(5):
            d = AL[n, i] - Tt[yy[n], i]
            s += d * d
            assert math.isclose(G[n, i], 2 * d / 20, rel_tol=1e-14)
    assert math.isclose(loss, s / 20, rel_tol=1e-14)


@pytest.mark.parametrize("C", [47, 100, 1000])
def test_cross_entropy_closed_forms(C):
    seg = osg.Segment([4, C], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT)
    B = 6
    y = np.array([0, 1, C - 1, 5, 5, 2])
    loss, G = seg.loss_and_grad(np.zeros((B, C)), y)
    assert math.isclose(loss, math.log(C), rel_tol=1e-14)
    expect = np.full((B, C), 1.0 / C)
    expect[np.arange(B), y] -= 1.0
    assert np.allclose(G, expect / B, rtol=1e-14, atol=0)
    g = np.random.default_rng(2)
    Zl = 5 * g.standard_normal((B, C))
    loss1, G1 = seg.loss_and_grad(Zl, y)
    loss2, G2 = seg.loss_and_grad(Zl + 1000.0, y)              # shift invariance, no overflow
    assert math.isclose(loss1, loss2, rel_tol=1e-9) and np.allclose(G1, G2, atol=1e-12)
    assert np.allclose(G1.sum(axis=1), 0, atol=1e-15)           # rows of dZ sum to zero
    p = G1 * B
    p[np.arange(B), y] += 1
    assert np.allclose(p.sum(axis=1), 1) and np.all(p > 0)
    # brute force
    s = 0.0
    for n in range(B):
        s += math.log(sum(math.exp(v) for v in Zl[n])) - Zl[n, y[n]]
    assert math.isclose(loss1, s / B, rel_tol=1e-12)


# ---------------------------------------------------------------------------------
# gradients
# ---------------------------------------------------------------------------------
def _loss_only(seg, X, y, T):
    A, _ = seg.forward_all(X)
    return seg.loss_and_grad(A[-1], y, T)[0]


@pytest.mark.parametrize("act,loss", [(osg.RELU_ALL, osg.MSE_SIL), (osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT),
                                      (osg.RELU_HIDDEN_IDENTITY_LAST, osg.MSE_SIL), (osg.RELU_ALL, osg.SOFTMAX_XENT)])
def test_gradients_central_differences(act, loss):
    widths = [5, 4, 6, 3]
    seg = _rand_segment(widths, act, loss, seed=4)
    g = np.random.default_rng(3)
    X = g.uniform(0, 1, (3, 5))
    y = np.array([2, 0, 1])
    T = g.uniform(0, 1, (3, 3))
    out = seg.step(X, y, T, update=False)
    h = 1e-6
    for l in range(seg.L):
        for arr, grad in ((seg.W[l], out["dW"][l]), (seg.b[l], out["db"][l])):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                keep = arr[idx]
                arr[idx] = keep + h
                lp = _loss_only(seg, X, y, T)
                arr[idx] = keep - h
                lm = _loss_only(seg, X, y, T)
                arr[idx] = keep
                assert abs((lp - lm) / (2 * h) - grad[idx]) < 1e-7, (l, idx)
    assert out["dZ"][0] is None       # nothing flows out of the segment's first layer


@pytest.mark.parametrize("act,loss,mu", [(osg.RELU_ALL, osg.MSE_SIL, 0.9), (osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, 0.9),
                                         (osg.RELU_ALL, osg.MSE_SIL, 0.0)])
def test_steps_against_autodiff_library(act, loss, mu):
    """Three consecutive steps against torch autograd + torch.optim.SGD in
    float64: pins forward, both losses, every gradient, the momentum convention
    (the paper trains with that framework's SGD, Sec. 3) and the update sign."""
    widths = [7, 9, 8, 5]
    seg = _rand_segment(widths, act, loss, seed=8, lr=0.05, momentum=mu)
    tW = [torch.tensor(w.copy(), dtype=torch.float64, requires_grad=True) for w in seg.W]
    tb = [torch.tensor(b.copy(), dtype=torch.float64, requires_grad=True) for b in seg.b]
    opt = torch.optim.SGD(tW + tb, lr=0.05, momentum=mu)
    g = np.random.default_rng(6)
    T = g.uniform(0, 2, (5, 5))
    for it in range(3):
        X = g.uniform(0, 1, (6, 7))
        y = g.integers(0, 5, 6)
        out = seg.step(X, y, T)
        a = torch.tensor(X)
        for l in range(3):
            a = a @ tW[l].T + tb[l]
            if l < 2 or act == osg.RELU_ALL:
                a = torch.relu(a)
        if loss == osg.MSE_SIL:
            lt = torch.nn.functional.mse_loss(a, torch.tensor(T[y]))
        else:
            lt = torch.nn.functional.cross_entropy(a, torch.tensor(y))
        opt.zero_grad()
        lt.backward()
        assert math.isclose(out["loss"], lt.item(), rel_tol=1e-12)
        for l in range(3):
            assert np.allclose(out["dW"][l], tW[l].grad.numpy(), rtol=1e-10, atol=1e-14)
            assert np.allclose(out["db"][l], tb[l].grad.numpy(), rtol=1e-10, atol=1e-14)
        opt.step()
        for l in range(3):
            assert np.allclose(seg.W[l], tW[l].detach().numpy(), rtol=1e-12, atol=1e-15)
            assert np.allclose(seg.b[l], tb[l].detach().numpy(), rtol=1e-12, atol=1e-15)


def test_single_linear_layer_normal_equations():
    g = np.random.default_rng(10)
    B, K, D = 12, 4, 3
    X = g.standard_normal((B, K))
    T = g.standard_normal((B, D))             # one class per sample: table row n
    y = np.arange(B)
    seg = _rand_segment([K, D], osg.RELU_HIDDEN_IDENTITY_LAST, osg.MSE_SIL, seed=2, lr=0.5)
    out = seg.step(X, y, T, update=False)
    R = X @ seg.W[0].T + seg.b[0] - T
    assert np.allclose(out["dW"][0], 2.0 / (B * D) * R.T @ X, rtol=1e-12)
    assert np.allclose(out["db"][0], 2.0 / (B * D) * R.sum(axis=0), rtol=1e-12)
    for _ in range(6000):
        seg.step(X, y, T)
    Xa = np.hstack([X, np.ones((B, 1))])
    sol = np.linalg.lstsq(Xa, T, rcond=None)[0]      # textbook least squares
    assert np.allclose(seg.W[0], sol[:K].T, atol=1e-6) and np.allclose(seg.b[0], sol[K], atol=1e-6)


def test_sgd_momentum_convention():
    # 1 -> 1 identity layer with input 0: output = b, loss = (b - t)^2, dL/db = 2 (b - t)
    # and dW = dZ * x = 0, so the bias follows the momentum recurrence alone.
    X, T, y = np.array([[0.0]]), np.array([[1.0]]), np.array([0])
    seg = osg.Segment([1, 1], osg.RELU_HIDDEN_IDENTITY_LAST, osg.MSE_SIL, lr=0.1, momentum=0.9)
    # by hand: g1 = -2, v1 = -2, b1 = 0.2 ; g2 = -1.6, v2 = 0.9*(-2) - 1.6 = -3.4, b2 = 0.54
    seg.step(X, y, T)
    assert math.isclose(seg.b[0][0], 0.2, rel_tol=1e-15)
    seg.step(X, y, T)
    assert math.isclose(seg.b[0][0], 0.54, rel_tol=1e-14)
    assert seg.W[0][0, 0] == 0.0
    # momentum 0 is plain gradient descent: b <- b - lr * 2 (b - 1) = 0.8 b + 0.2
    seg = osg.Segment([1, 1], osg.RELU_HIDDEN_IDENTITY_LAST, osg.MSE_SIL, lr=0.1, momentum=0.0)
    for k in range(1, 6):
        seg.step(X, y, T)
        assert math.isclose(seg.b[0][0], 1.0 - 0.8 ** k, rel_tol=1e-13)
    # constant gradient: cross-entropy with one class has p = 1, dZ = 0; instead use
    # a frozen linear loss: two classes, logits (b0, b1) from x = 0, huge margin so
    # the softmax saturates and dL/db = (1, -1)/1 * (p - onehot) ~ (+1, -1) constant
    seg = osg.Segment([1, 2], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, lr=0.01, momentum=0.9)
    seg.set_params(0, np.zeros((2, 1)), np.array([800.0, 0.0]))
    for k in range(1, 8):
        seg.step(X, np.array([1]), None)
        drift = 0.01 * sum((1 - 0.9 ** i) / (1 - 0.9) for i in range(1, k + 1))   # lr g sum_i (1-mu^i)/(1-mu)
        assert math.isclose(seg.b[0][0], 800.0 - drift, rel_tol=1e-13)
        assert math.isclose(seg.b[0][1], drift, rel_tol=1e-12)


def test_loss_decreases_on_separable_toy_set():
    # 3 well separated classes; a 2-segment network trained the paper's way:
    # left on synthetic labels (MSE), right on the left response (cross-entropy)
    g = np.random.default_rng(12)
    centres = np.array([[0.1, 0.1, 0.9, 0.1], [0.9, 0.1, 0.1, 0.5], [0.1, 0.9, 0.5, 0.9]])
    y = datagen.balanced_classes(96, 3)
    X = np.clip(centres[y] + 0.02 * g.standard_normal((96, 4)), 0, 1)
    T = rng.make_synthetic_labels(7, 3, 8, rng.UNIFORM01, kappa=1.0).astype(np.float64)
    # plain SGD with a small rate: the epoch-mean loss must fall monotonically
    plain = _rand_segment([4, 16, 8], osg.RELU_ALL, osg.MSE_SIL, seed=5, lr=0.1, momentum=0.0)
    epoch_loss = []
    for ep in range(40):
        tot = 0.0
        for s in range(0, 96, 32):                          # no shuffling
            tot += plain.step(X[s:s + 32], y[s:s + 32], T)["loss"]
        epoch_loss.append(tot / 3)
    assert all(b < a for a, b in zip(epoch_loss, epoch_loss[1:]))
    assert epoch_loss[-1] < 0.3 * epoch_loss[0]
    # the paper's optimiser setting (momentum 0.9) gets further in the same time
    left = _rand_segment([4, 16, 8], osg.RELU_ALL, osg.MSE_SIL, seed=5, lr=0.05, momentum=0.9)
    mom_loss = []
    for ep in range(40):
        tot = 0.0
        for s in range(0, 96, 32):
            tot += left.step(X[s:s + 32], y[s:s + 32], T)["loss"]
        mom_loss.append(tot / 3)
    assert mom_loss[-1] < 0.1 * mom_loss[0]
    R = left.forward(X)                                     # stored left response
    right = _rand_segment([8, 16, 3], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, seed=6, lr=0.1, momentum=0.9)
    rl = []
    for ep in range(40):
        tot = 0.0
        for s in range(0, 96, 32):
            tot += right.step(R[s:s + 32], y[s:s + 32])["loss"]
        rl.append(tot / 3)
    assert rl[-1] < 0.2 * rl[0]
    pred = right.forward(left.forward(X)).argmax(axis=1)    # joined partitions
    assert (pred == y).mean() > 0.95


def test_simultaneous_variant_on_separable_toy_set():
    # end of Sec. 2: the right partition never sees the left one's response while training -- its inputs are the
    # synthetic label of the sample's class plus noise -- and the two still work when joined afterwards
    g = np.random.default_rng(13)
    centres = np.array([[0.1, 0.1, 0.9, 0.1], [0.9, 0.1, 0.1, 0.5], [0.1, 0.9, 0.5, 0.9]])
    y = datagen.balanced_classes(96, 3)
    X = np.clip(centres[y] + 0.02 * g.standard_normal((96, 4)), 0, 1)
    T32 = rng.make_synthetic_labels(7, 3, 8, rng.UNIFORM01, kappa=1.0)
    T = T32.astype(np.float64)
    left = _rand_segment([4, 16, 8], osg.RELU_ALL, osg.MSE_SIL, seed=5, lr=0.05, momentum=0.9)
    right = _rand_segment([8, 16, 3], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, seed=6, lr=0.1, momentum=0.9)
    ll, rl = [], []
    for ep in range(60):
        a = b = 0.0
        for s in range(0, 96, 32):
            a += left.step(X[s:s + 32], y[s:s + 32], T)["loss"]
            xin = rng.make_segment_inputs(9, T32, y[s:s + 32], s, 0.05).astype(np.float64)
            b += right.step(xin, y[s:s + 32])["loss"]
        ll.append(a / 3)
        rl.append(b / 3)
    assert ll[-1] < 0.1 * ll[0] and rl[-1] < 0.2 * rl[0]
    pred = right.forward(left.forward(X)).argmax(axis=1)    # joined only now
    assert (pred == y).mean() > 0.9


# ---------------------------------------------------------------------------------
# bf16 storage emulation
# ---------------------------------------------------------------------------------
def test_bf16_mode_is_exact_on_representable_values():
    # small integers / powers of two: nothing is rounded, so both modes agree exactly
    widths = [4, 4, 2]
    g = np.random.default_rng(3)
    Ws = [(g.integers(-2, 3, (4, 4)).astype(float), g.integers(-2, 3, 4).astype(float)),
          (g.integers(-2, 3, (2, 4)).astype(float), g.integers(-2, 3, 2).astype(float))]
    X = g.integers(0, 3, (4, 4)).astype(float)
    T = g.integers(0, 3, (2, 2)).astype(float)
    y = np.array([0, 1, 1, 0])
    outs = []
    for mode in ("fp32", "bf16"):
        seg = osg.Segment(widths, osg.RELU_ALL, osg.MSE_SIL, mode=mode)
        for l, (W, b) in enumerate(Ws):
            seg.set_params(l, W, b)
        outs.append(seg.step(X, y, T, update=False))
    for l in range(2):
        assert np.array_equal(outs[0]["dW"][l], outs[1]["dW"][l])
        assert np.array_equal(outs[0]["A"][l + 1], outs[1]["A"][l + 1])
    assert outs[0]["loss"] == outs[1]["loss"]


def test_bf16_mode_rounds_at_storage_points_only():
    widths = [16, 12, 8]
    g = np.random.default_rng(4)
    X = g.uniform(0, 1, (10, 16))
    y = g.integers(0, 5, 10)
    T = g.standard_normal((5, 8))
    a = _rand_segment(widths, osg.RELU_ALL, osg.MSE_SIL, seed=1, mode="fp32")
    b = _rand_segment(widths, osg.RELU_ALL, osg.MSE_SIL, seed=1, mode="bf16")
    oa, ob = a.step(X, y, T, update=False), b.step(X, y, T, update=False)
    for l in (1, 2):
        A = ob["A"][l]
        assert np.array_equal(A, rng.round_to_bf16(A.astype(np.float32)))       # on the bf16 grid
        assert np.max(np.abs(A - oa["A"][l])) <= 2.0 ** -6 * np.max(np.abs(oa["A"][l]))
    dz = ob["dZ"][2]
    assert np.array_equal(dz, rng.round_to_bf16(dz.astype(np.float32)))
    # dW is a float64 product of bf16-grid operands and is not itself rounded
    assert np.allclose(ob["dW"][1], ob["dZ"][2].T @ ob["A"][1], rtol=1e-14)
    assert not np.array_equal(ob["dW"][1], rng.round_to_bf16(ob["dW"][1].astype(np.float32)))
    assert np.max(np.abs(ob["dW"][1] - oa["dW"][1])) <= 0.05 * np.max(np.abs(oa["dW"][1]))


def test_sampled_rows_of_a_larger_batch():
    # A, Z and dZ of a row depend on the other rows only through the batch size in the means
    widths = [9, 11, 7]
    g = np.random.default_rng(21)
    X = g.uniform(0, 1, (12, 9))
    y = g.integers(0, 4, 12)
    T = g.standard_normal((4, 7))
    for act, loss in ((osg.RELU_ALL, osg.MSE_SIL), (osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT)):
        seg = _rand_segment(widths, act, loss, seed=2)
        full = seg.step(X, y, T, update=False)
        rows = np.array([0, 5, 11])
        part = seg.step(X[rows], y[rows], T, update=False, full_batch=12)
        for l in (1, 2):
            assert np.array_equal(part["A"][l], full["A"][l][rows])
            assert np.allclose(part["dZ"][l], full["dZ"][l][rows], rtol=1e-13, atol=0)
        assert part["dW"][0] is None


# ---------------------------------------------------------------------------------
# recovery phase (paper Sec. 5): left partition trained through the frozen right one
# ---------------------------------------------------------------------------------
def _joined_loss(left, right, X, y):
    return right.loss_and_grad(right.forward(left.forward(X)), y)[0]


def test_recovery_gradients_by_finite_differences():
    g = np.random.default_rng(31)
    left = _rand_segment([6, 7, 5], osg.RELU_ALL, osg.MSE_SIL, seed=3)
    right = _rand_segment([5, 6, 4], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, seed=4)
    X = g.uniform(0, 1, (5, 6))
    y = g.integers(0, 4, 5)
    R = left.forward(X)
    back = right.input_gradient(R, y)
    assert math.isclose(back["loss"], _joined_loss(left, right, X, y), rel_tol=1e-14)
    # dX of the right partition = d loss / d (its input), element by element
    h = 1e-6
    for idx in np.ndindex(R.shape):
        Rp, Rm = R.copy(), R.copy()
        Rp[idx] += h
        Rm[idx] -= h
        fd = (right.loss_and_grad(right.forward(Rp), y)[0] - right.loss_and_grad(right.forward(Rm), y)[0]) / (2 * h)
        assert abs(fd - back["dX"][idx]) < 1e-8, idx
    # and the left partition's parameter gradients through the frozen right partition
    out = left.step_external(X, back["dX"], update=False)
    for l in range(left.L):
        for arr, grad in ((left.W[l], out["dW"][l]), (left.b[l], out["db"][l])):
            for idx in np.ndindex(arr.shape):
                keep = arr[idx]
                arr[idx] = keep + h
                lp = _joined_loss(left, right, X, y)
                arr[idx] = keep - h
                lm = _joined_loss(left, right, X, y)
                arr[idx] = keep
                assert abs((lp - lm) / (2 * h) - grad[idx]) < 1e-7, (l, idx)


def test_recovery_steps_against_autodiff_library():
    # joined network in an autograd library, optimiser over the LEFT parameters only
    g = np.random.default_rng(32)
    left = _rand_segment([8, 9, 6], osg.RELU_ALL, osg.MSE_SIL, seed=5, lr=0.05, momentum=0.9)
    right = _rand_segment([6, 7, 5], osg.RELU_HIDDEN_IDENTITY_LAST, osg.SOFTMAX_XENT, seed=6)
    tl = [(torch.tensor(w.copy(), requires_grad=True), torch.tensor(b.copy(), requires_grad=True)) for w, b in zip(left.W, left.b)]
    tr = [(torch.tensor(w.copy()), torch.tensor(b.copy())) for w, b in zip(right.W, right.b)]
    opt = torch.optim.SGD([p for wb in tl for p in wb], lr=0.05, momentum=0.9)
    right_before = [w.copy() for w in right.W]
    for it in range(3):
        X = g.uniform(0, 1, (7, 8))
        y = g.integers(0, 5, 7)
        back = right.input_gradient(left.forward(X), y)
        left.step_external(X, back["dX"])
        a = torch.tensor(X)
        for w, b in tl:
            a = torch.relu(a @ w.T + b)                    # the cut layer keeps its ReLU
        for i, (w, b) in enumerate(tr):
            a = a @ w.T + b
            if i < len(tr) - 1:
                a = torch.relu(a)
        lt = torch.nn.functional.cross_entropy(a, torch.tensor(y))
        opt.zero_grad()
        lt.backward()
        opt.step()
        assert math.isclose(back["loss"], lt.item(), rel_tol=1e-12)
        for l in range(2):
            assert np.allclose(left.W[l], tl[l][0].detach().numpy(), rtol=1e-11, atol=1e-15)
            assert np.allclose(left.b[l], tl[l][1].detach().numpy(), rtol=1e-11, atol=1e-15)
    for l in range(2):
        assert np.array_equal(right.W[l], right_before[l])   # frozen


# ---------------------------------------------------------------------------------
# ReLU decisions at ties
# ---------------------------------------------------------------------------------
def test_tie_decisions_are_taken_only_inside_the_bounds():
    # hand-built 2-2-1 net: unit 0 of layer 1 has pre-activation exactly 0 for sample 0 (a tie), everything else is clear
    seg = osg.Segment([2, 2, 1], osg.RELU_HIDDEN_IDENTITY_LAST, osg.MSE_SIL, lr=0.1, momentum=0.0)
    seg.set_params(0, np.array([[1.0, -1.0], [0.5, 0.5]]), np.array([0.0, 0.0]))
    seg.set_params(1, np.array([[2.0, 3.0]]), np.array([0.0]))
    X = np.array([[1.0, 1.0], [2.0, 1.0]])        # Z1 = [[0, 1], [1, 1.5]]
    y = np.array([0, 0])
    T = np.array([[0.0]])
    own = seg.step(X, y, T, update=False)
    assert np.array_equal(own["Z"][1], np.array([[0.0, 1.0], [1.0, 1.5]]))
    # own decision at the tie: inactive (the derivative of ReLU at 0 is taken as 0)
    # out = [3, 6.5]; G = 2*(out - 0)/2 = out; dZ1 = G * W2 * mask
    assert np.array_equal(own["dZ"][1], np.array([[0.0, 9.0], [13.0, 19.5]]))
    E = seg.forward_error_bound(X)
    # the bound by hand for (sample 0, unit 0): (sqrt(2) + 2) 2^-24 (|1*1| + |1*-1| + 0)
    assert math.isclose(E[1][0, 0], (math.sqrt(2) + 2) * 2.0 ** -24 * 2.0, rel_tol=1e-14)
    assert np.all(E[1] < 2e-6) and np.all(E[1] > 0)
    same = seg.step(X, y, T, update=False, tie_decisions=[None, own["A"][1] > 0, None], tie_bounds=E)
    assert same["ties_taken"] == 0 and same["decisions_refused"] == 0 and not same["tie_rows"].any()
    assert np.array_equal(same["dZ"][1], own["dZ"][1])
    # the other side calls the tie "active": taken over, the gradient flows through that unit
    other = np.array([[True, True], [True, True]])
    took = seg.step(X, y, T, update=False, tie_decisions=[None, other, None], tie_bounds=E)
    assert took["ties_taken"] == 1 and took["decisions_refused"] == 0
    assert np.array_equal(took["tie_rows"], [True, False]) and took["worst_tie_ratio"] == 0.0
    assert np.array_equal(took["dZ"][1], np.array([[6.0, 9.0], [13.0, 19.5]]))
    assert np.array_equal(took["dW"][0], took["dZ"][1].T @ X)
    # a disagreement at a clear pre-activation (1.5, far outside the bound) is refused and counted
    wrong = np.array([[False, True], [True, False]])
    ref = seg.step(X, y, T, update=False, tie_decisions=[None, wrong, None], tie_bounds=E)
    assert ref["ties_taken"] == 0 and ref["decisions_refused"] == 1
    assert np.array_equal(ref["dZ"][1], own["dZ"][1])
    # a pre-activation of 1e-5 is NOT a tie for float32 accumulation of two terms of size 1
    seg.set_params(0, np.array([[1.0, -1.0 + 1e-5], [0.5, 0.5]]), np.array([0.0, 0.0]))
    E = seg.forward_error_bound(X)
    ref = seg.step(X, y, T, update=False, tie_decisions=[None, np.array([[False, True], [True, True]]), None], tie_bounds=E)
    assert ref["ties_taken"] == 0 and ref["decisions_refused"] == 1


def test_stored_deviation_against_brute_force():
    # bf16 storage: two values within E of each other round to the same bfloat16 unless a rounding boundary lies
    # between them; the bound must hold for every sampled neighbour, and be zero only where all neighbours agree
    seg = osg.Segment([2, 2], osg.RELU_ALL, osg.MSE_SIL, mode="bf16")
    g = np.random.default_rng(3)
    pre = np.concatenate([g.standard_normal(4000), g.standard_normal(2000) * 1e-3, [0.0, 1.0, 2.0, 0.5, 1.00390625, 0.998046875]])
    for E in (1e-7, 3e-5, 2e-3):
        bound = seg._stored_deviation(pre, np.full(pre.shape, E))
        worst = np.zeros_like(pre)
        for t in np.linspace(-1.0, 1.0, 41):
            other = torch.tensor((pre + t * E).astype(np.float32)).to(torch.bfloat16).double().numpy()
            mine = torch.tensor(pre.astype(np.float32)).to(torch.bfloat16).double().numpy()
            worst = np.maximum(worst, np.abs(other - mine))
        assert np.all(worst <= bound * (1 + 1e-12) + 1e-300)
        assert np.all(worst[bound == 0.0] == 0.0)
        # not vacuous: for a small E most values are far from a boundary and get a zero bound
        if E == 1e-7:
            assert np.mean(bound == 0.0) > 0.95 and np.any(bound > 0.0)
    # fp32 mode stores the value itself
    seg32 = osg.Segment([2, 2], osg.RELU_ALL, osg.MSE_SIL)
    assert np.array_equal(seg32._stored_deviation(pre, np.full(pre.shape, 1e-5)), np.full(pre.shape, 1e-5))


@pytest.mark.parametrize("mode", ["fp32", "bf16"])
def test_forward_error_bound_covers_a_float32_implementation(mode):
    # another implementation of the forward pass: float32 accumulation (torch CPU, any order), same storage points.
    # Its pre-activations must lie within the oracle's bounds of the oracle's own, layer after layer, and the bounds
    # must stay small against the pre-activations (they decide where a ReLU decision counts as a tie)
    widths = [784, 1024, 512, 256]
    seg = _rand_segment(widths, osg.RELU_ALL, osg.MSE_SIL, 4, mode=mode)
    X, _ = datagen.class_mean_inputs(96, 47, dim=784, seed=2)
    store = (lambda t: t.to(torch.bfloat16).to(torch.float32)) if mode == "bf16" else (lambda t: t)
    a = store(torch.tensor(X))
    Xv = a.double().numpy()
    A, Z = seg.forward_all(Xv)
    E = seg.forward_error_bound(Xv)
    for l in range(1, 4):
        W = store(torch.tensor(seg.W[l - 1], dtype=torch.float32))
        z = a @ W.T + torch.tensor(seg.b[l - 1], dtype=torch.float32)
        dev = np.abs(z.double().numpy() - Z[l])
        assert np.all(dev <= E[l]), (l, float(np.max(dev / E[l])))
        band = np.max(E[l]) / np.max(np.abs(Z[l]))
        assert band <= ((1.5e-5 if l == 1 else 5e-4) if mode == "fp32" else (1.5e-5 if l == 1 else 1.5e-2)), (l, band)
        a = store(torch.relu(z))
    # parameters that differ by a relative 1e-6 of the largest weight: still inside, with param_rel saying so
    g = np.random.default_rng(1)
    E2 = seg.forward_error_bound(Xv, param_rel=1e-6)
    a = store(torch.tensor(X))
    for l in range(1, 4):
        Wm = seg.W[l - 1] + 1e-6 * np.max(np.abs(seg.W[l - 1])) * g.uniform(-1, 1, seg.W[l - 1].shape)
        bm = seg.b[l - 1] + 1e-6 * np.max(np.abs(seg.b[l - 1])) * g.uniform(-1, 1, seg.b[l - 1].shape)
        z = a @ store(torch.tensor(Wm, dtype=torch.float32)).T + torch.tensor(bm, dtype=torch.float32)
        dev = np.abs(z.double().numpy() - Z[l])
        assert np.all(dev <= E2[l]) and np.all(E2[l] >= E[l]), l
        a = store(torch.relu(z))


def test_sampled_weight_gradient_entries_are_entries_of_the_step_gradient():
    seg = _rand_segment([7, 9, 5], osg.RELU_ALL, osg.MSE_SIL, 8)
    g = np.random.default_rng(2)
    X = g.standard_normal((11, 7))
    T = g.standard_normal((3, 5))
    out = seg.step(X, np.arange(11) % 3, T, update=False)
    oi, ki = np.array([0, 8, 3, 3]), np.array([6, 0, 2, 5])
    got, scale = osg.weight_gradient_elements(out["dZ"][1][:, oi], out["A"][0][:, ki])
    assert np.allclose(got, out["dW"][0][oi, ki], rtol=1e-13, atol=1e-16)
    assert np.all(scale >= np.abs(got))
    # second layer, through python loops
    got2, _ = osg.weight_gradient_elements(out["dZ"][2][:, [4]], out["A"][1][:, [7]])
    assert math.isclose(got2[0], sum(out["dZ"][2][n, 4] * out["A"][1][n, 7] for n in range(11)), rel_tol=1e-13)


def test_count_correct_against_loops_and_ties():
    g = np.random.default_rng(5)
    Z = g.standard_normal((50, 7))
    y = g.integers(0, 7, 50)
    hits = 0
    for n in range(50):
        best = 0
        for c in range(1, 7):
            if Z[n, c] > Z[n, best]:
                best = c
        hits += int(best == y[n])
    assert osg.count_correct(Z, y) == hits and 0 < hits < 50
    # equal maxima: the lowest index is the prediction; a class id outside the row never matches
    Z = np.array([[1.0, 3.0, 3.0], [2.0, 2.0, 2.0], [0.0, -1.0, 5.0]])
    assert osg.count_correct(Z, [1, 0, 2]) == 3
    assert osg.count_correct(Z, [2, 1, 7]) == 0
    assert osg.mean_loss([1.0, 2.0, 6.0]) == 3.0
