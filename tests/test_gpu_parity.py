"""HIP path against the CPU oracle, element by element, through the C ABI.

Tolerances (per tensor, max|gpu - ref| / max|ref|):
  float32 path  1e-5   (float32 MFMA accumulation against float64)
  bf16 path     2e-2   (bf16 storage, float32 accumulation)
Labels, generated inputs, initial weights and gather indices are bit-exact."""

import ctypes

import numpy as np
import pytest
import torch

from oracle import rng as orng
from oracle import segment as osg
from paper_2403_11204_amd import api, datagen

pytestmark = pytest.mark.gpu

TOL = {api.F32: 1e-5, api.BF16: 2e-2}
DEV = "cuda"


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy()


def as_input(X, dtype):
    """Host float32 inputs -> (device tensor in the handle's dtype, the exact values it holds as float64)."""
    t = torch.from_numpy(np.ascontiguousarray(X)).to(DEV)
    t = t.to(torch.bfloat16) if dtype == api.BF16 else t
    return t.contiguous(), to_np(t).astype(np.float64)


# ---------------------------------------------------------------------------------
# generators: bit-exact
# ---------------------------------------------------------------------------------
@pytest.mark.parametrize("dist", [api.UNIFORM01, api.UNIFORM_PM1, api.NORMAL, api.BINARY_PM1])
@pytest.mark.parametrize("classes,dim,seed,kappa", [(47, 64, 7, 1.0), (47, 60, 11, 10.0), (47, 2048, 13, 1.0),
                                                    (100, 8192, (21 << 32) | 5, 2.5), (3, 1, 0, 1.0)])
def test_labels_bit_exact(dist, classes, dim, seed, kappa):
    ref = orng.make_synthetic_labels(seed, classes, dim, dist, kappa)
    got = api.make_synthetic_labels(seed, classes, dim, dist, kappa, api.F32)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    got16 = api.make_synthetic_labels(seed, classes, dim, dist, kappa, api.BF16)
    ref16 = orng.round_to_bf16(ref)
    assert np.array_equal(to_np(got16).view(np.uint32), ref16.view(np.uint32))


def test_labels_bit_exact_largest_table():
    # 1000 x 16384 U(-1,1) (comparison config) and N(0,1): every one of the 16.4 M entries
    for dist, seed in ((api.UNIFORM_PM1, 31), (api.NORMAL, 23)):
        got = api.make_synthetic_labels(seed, 1000, 16384, dist).cpu().numpy()
        ref = orng.make_synthetic_labels(seed, 1000, 16384, dist)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_segment_inputs_bit_exact(dtype):
    table = api.make_synthetic_labels(7, 47, 64, api.UNIFORM_PM1)
    y = datagen.balanced_classes(300, 47, first=5)
    first = (1 << 32) - 100          # crosses the 32-bit boundary of the sample counter
    got = api.make_segment_inputs(5, table, torch.from_numpy(y).to(DEV), first, 0.05, dtype)
    ref = orng.make_segment_inputs(5, table.cpu().numpy(), y, first, 0.05)
    if dtype == api.BF16:
        ref = orng.round_to_bf16(ref)
    assert np.array_equal(to_np(got).view(np.uint32), ref.view(np.uint32))


def test_init_weights_bit_exact():
    widths = [37, 70, 129, 47]
    seg = api.Segment(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, max_batch=8)
    seg.init(3)
    for l in range(3):
        W, b = seg.get_params(l)
        rW, rb = orng.init_weights(3, l, widths[l + 1], widths[l])
        assert np.array_equal(W.cpu().numpy().view(np.uint32), rW.view(np.uint32))
        assert np.array_equal(b.cpu().numpy().view(np.uint32), rb.view(np.uint32))


# ---------------------------------------------------------------------------------
# one training step and short runs
# ---------------------------------------------------------------------------------
def make_pair(widths, act, loss, dtype, max_batch, lr, mom, wseed):
    g = api.Segment(widths, act, loss, max_batch=max_batch, dtype=dtype, lr=lr, momentum=mom)
    o = osg.Segment(widths, act, loss, lr=lr, momentum=mom, mode="bf16" if dtype == api.BF16 else "fp32")
    for l, (W, b) in enumerate(datagen.uniform_weights(widths, wseed)):
        g.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
        o.set_params(l, W, b)
    return g, o


U32 = 2.0 ** -24          # unit roundoff of the float32 accumulation on the device
TIE_LOG = []              # (ties taken, worst |Z| / bound, band per layer) of every checked step, printed at the end


def tie_report(out, bounds):
    """One line per checked step: how many ReLU decisions were taken over, how deep inside its bound the worst of them
    sat, and how wide the bounds are against the pre-activations they guard."""
    band = [float(np.max(bounds[l]) / max(np.max(np.abs(out["Z"][l])), 1e-300)) for l in range(1, len(bounds))]
    TIE_LOG.append((out["ties_taken"], out["worst_tie_ratio"], band))
    print("ties taken %d (rows %d), worst |Z|/bound %.3f, bound/max|Z| per layer %s"
          % (out["ties_taken"], int(out["tie_rows"].sum()), out["worst_tie_ratio"], ["%.1e" % x for x in band]), flush=True)


def compare_rows_without_ties(out, free, acts, dzs, tol):
    """out: oracle step with decisions taken over; free: the same step with none taken over; acts / dzs: the device's
    A_l / dZ_l (same rows).  Returns the number of (row, layer) pairs of dZ compared against `free`."""
    L = len(acts) - 1
    tied = np.zeros(acts[1].shape[0], dtype=bool)
    compared = 0
    for l in range(L, 0, -1):
        assert rel_err(acts[l], free["A"][l]) <= tol, ("A, nothing taken over", l)
        tied = tied | out["tie_rows_by_layer"].get(l, False)
        keep = ~tied
        if keep.any():
            scale = max(float(np.max(np.abs(free["dZ"][l]))), 1e-300)
            assert float(np.max(np.abs(dzs[l][keep] - free["dZ"][l][keep]))) <= tol * scale, ("dZ, nothing taken over", l)
            compared += int(keep.sum())
    return compared


def check_step(g, o, X, y, table_np, dtype, steps=1, check_internals=True, tie_cap=1e-4, stored_dW=True):
    tol = TOL[dtype]
    B = X.shape[0]
    Xd, Xv = as_input(X, dtype)
    yd = torch.from_numpy(y).to(DEV)
    if table_np is not None:
        g.set_labels(torch.from_numpy(table_np).to(DEV))
    W_before = [o.W[l].copy() for l in range(o.L)]
    for s in range(steps):
        loss_g = float(g.step(Xd, yd).item())
        # The ReLU mask is an integer decision taken from a floating-point value.  Where the oracle's
        # pre-activation is zero to within the rounding error of the device's arithmetic, "active" and
        # "inactive" are both correct, and one such element changes the whole row of every dZ below it and a
        # row of dW.  The oracle bounds that rounding error element by element from its own values (float32
        # accumulation, the mode's storage points; after s steps the two sides' parameters have drifted apart
        # by the float32 rounding of s updates) and takes over the device's decision only where its own
        # pre-activation lies inside the bound; a disagreement outside is the device's error.
        acts = [None] + [to_np(g.get_activation(l, B)) for l in range(1, o.L + 1)]
        bounds = o.forward_error_bound(Xv, unit=U32, param_rel=8 * s * U32)
        out = o.step(Xv, y, table_np, update=False, tie_decisions=[None] + [a > 0 for a in acts[1:]], tie_bounds=bounds)
        tie_report(out, bounds)
        assert abs(loss_g - out["loss"]) <= tol * abs(out["loss"]), (s, loss_g, out["loss"])
        assert out["decisions_refused"] == 0
        assert out["ties_taken"] <= max(1, int(tie_cap * sum(a.size for a in acts[1:]))), out["ties_taken"]
        if out["ties_taken"] and check_internals and s == steps - 1:
            # the same step with no decision taken over: A_l does not depend on the decisions at all, and dZ_l of a row
            # depends only on those of that row at layers l..L -- every such row must match the oracle on its own
            free = o.step(Xv, y, table_np, update=False)
            dz_got = [None] + [to_np(g.get_activation(l, B, kind=1)).astype(np.float64) for l in range(1, o.L + 1)]
            assert compare_rows_without_ties(out, free, acts, dz_got, tol) > 0
        o.apply_update(out["dW"], out["db"])
    if check_internals:      # state of the last step
        for l in range(o.L, 0, -1):
            assert rel_err(acts[l], out["A"][l]) <= tol, ("A", l)
            dz_ref = out["dZ"][l]
            dz_got = to_np(g.get_activation(l, B, kind=1)).astype(np.float64)
            assert rel_err(dz_got, dz_ref) <= tol, ("dZ", l)
        for l in range(o.L):
            if stored_dW:
                dW, db = g.get_grads(l)
                assert rel_err(to_np(dW), out["dW"][l]) <= tol, ("dW", l)
            else:       # fused update: the weight gradient exists only inside the product (checked through vW and W below)
                db = g.get_bias_grad(l)
            assert rel_err(to_np(db), out["db"][l]) <= tol, ("db", l)
    for l in range(o.L):
        W, b = g.get_params(l)
        assert rel_err(to_np(W), o.W[l]) <= tol, ("W", l)
        assert rel_err(to_np(b), o.b[l]) <= tol, ("b", l)
        # the update itself, not hidden behind the size of the weights
        # (float32 storage of W puts a floor of a few ulp(|W|) under what can be seen of it)
        d_got, d_ref = to_np(W).astype(np.float64) - W_before[l], o.W[l] - W_before[l]
        floor = 4.0 * float(np.spacing(np.float32(np.max(np.abs(o.W[l])))))
        assert np.max(np.abs(d_got - d_ref)) <= tol * np.max(np.abs(d_ref)) + floor, ("dWstep", l)
        if o.mu != 0.0:
            vW, vb = g.get_momentum(l)
            assert rel_err(to_np(vW), o.vW[l]) <= tol, ("vW", l)
            assert rel_err(to_np(vb), o.vb[l]) <= tol, ("vb", l)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_exactly_representable_step_matches_with_no_tie_help(dtype):
    # Small-integer inputs, weights and labels, a batch x width that is a power of two and lr = 1/2: every sum of the
    # step is exact in float32 and every stored bf16 value is the rounding of an exactly known number, so the device
    # and the oracle must agree to the last bit -- masks included, with many pre-activations that are exactly zero
    # (ReLU'(0) = 0 on both sides) and no decision handed from one side to the other.
    rs = np.random.default_rng(11)
    widths, B, classes = [16, 16, 16, 8], 64, 8
    X = rs.integers(0, 4, size=(B, 16)).astype(np.float32)
    y = datagen.balanced_classes(B, classes)
    table = rs.integers(-3, 4, size=(classes, 8)).astype(np.float32)
    g = api.Segment(widths, api.RELU_ALL, api.MSE_SIL, max_batch=B, dtype=dtype, lr=0.5, momentum=0.0)
    o = osg.Segment(widths, osg.RELU_ALL, osg.MSE_SIL, lr=0.5, momentum=0.0, mode="bf16" if dtype == api.BF16 else "fp32")
    for l in range(3):
        W = rs.integers(-2, 3, size=(widths[l + 1], widths[l])).astype(np.float32)
        b = rs.integers(-8, 9, size=widths[l + 1]).astype(np.float32)
        g.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
        o.set_params(l, W, b)
    g.set_labels(torch.from_numpy(table).to(DEV))
    Xd, Xv = as_input(X, dtype)
    assert np.array_equal(Xv, X)
    loss_g = float(g.step(Xd, torch.from_numpy(y).to(DEV)).item())
    out = o.step(Xv, y, table.astype(np.float64))
    assert abs(loss_g - out["loss"]) <= 1e-6 * out["loss"]
    zeros = 0
    for l in range(1, 4):
        zeros += int(np.sum(out["Z"][l] == 0.0))
        assert np.array_equal(to_np(g.get_activation(l, B)).astype(np.float64), out["A"][l]), ("A", l)
        assert np.array_equal(to_np(g.get_activation(l, B, kind=1)).astype(np.float64), out["dZ"][l]), ("dZ", l)
    assert zeros >= 10, zeros            # the exact ties this case is about do occur
    for l in range(3):
        dW, db = g.get_grads(l)
        assert np.array_equal(to_np(dW).astype(np.float64), out["dW"][l]), ("dW", l)
        assert np.array_equal(to_np(db).astype(np.float64), out["db"][l]), ("db", l)
        W, b = g.get_params(l)
        assert np.array_equal(to_np(W).astype(np.float64), o.W[l]), ("W", l)
        assert np.array_equal(to_np(b).astype(np.float64), o.b[l]), ("b", l)


CASES = [
    # name, widths, act, loss, B, dist, classes
    ("tinyA", [784, 128, 64], api.RELU_ALL, api.MSE_SIL, 64, api.UNIFORM_PM1, 47),
    ("tinyB", [64, 64, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, 64, None, 47),
    ("ragged", [37, 70, 129, 47], api.RELU_ALL, api.MSE_SIL, 100, api.NORMAL, 10),
    ("raggedCE", [45, 131, 66, 10], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, 77, None, 10),
    ("one_layer", [20, 12], api.RELU_HIDDEN_IDENTITY_LAST, api.MSE_SIL, 9, api.UNIFORM01, 5),
    ("reluCE", [24, 40, 16], api.RELU_ALL, api.SOFTMAX_XENT, 33, None, 16),
    ("paperA", [784, 1024, 1024, 512], api.RELU_ALL, api.MSE_SIL, 256, api.NORMAL, 47),
    ("paperB", [512, 1024, 1024, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, 256, None, 47),
    ("paper_sec3_left", [784, 80, 60], api.RELU_ALL, api.MSE_SIL, 1410, api.UNIFORM01, 47),
    ("paper_sec3_right", [60, 60, 60, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, 1410, None, 47),
]


def case_data(widths, loss, B, dist, classes, seed):
    X, y = datagen.class_mean_inputs(B, classes, dim=widths[0], seed=seed)
    table = None
    if loss == api.MSE_SIL:
        kappa = 10.0 if dist == api.UNIFORM01 else 1.0
        table = orng.make_synthetic_labels(seed + 10, classes, widths[-1], dist, kappa)
    return X, y, table


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_one_step(case, dtype):
    name, widths, act, loss, B, dist, classes = case
    X, y, table = case_data(widths, loss, B, dist, classes, seed=1)
    g, o = make_pair(widths, act, loss, dtype, max_batch=B, lr=0.01, mom=0.9, wseed=3)
    check_step(g, o, X, y, table, dtype)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_one_step_with_the_update_inside_the_weight_gradient_product(case, dtype):
    # the same cases with the optimiser step applied in the epilogue of the weight-gradient product: parameters,
    # momentum (= the weight gradient after a first step from zero momentum) and everything else against the oracle
    name, widths, act, loss, B, dist, classes = case
    X, y, table = case_data(widths, loss, B, dist, classes, seed=1)
    g, o = make_pair(widths, act, loss, dtype, max_batch=B, lr=0.01, mom=0.9, wseed=3)
    g.set_fused_update(True)
    check_step(g, o, X, y, table, dtype, stored_dW=False)
    with pytest.raises(api.SlpError) as e:
        g.get_grads(0)
    assert e.value.code == -5


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
@pytest.mark.parametrize("mom", [0.0, 0.9])
def test_several_fused_steps_then_back_to_the_separate_update(dtype, mom):
    # five steps with the fused update (ragged shapes: pads of every derived copy must stay zero for the next products),
    # then the switch goes off and two ordinary steps follow on the same handle
    widths = [70, 130, 61, 33]
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, max_batch=90, lr=0.02, mom=mom, wseed=6)
    X, y, table = case_data(widths, api.MSE_SIL, 90, api.UNIFORM01, 20, seed=4)
    g.set_fused_update(True)
    check_step(g, o, X, y, table, dtype, steps=5, check_internals=(dtype == api.F32), stored_dW=False)
    g.set_fused_update(False)
    check_step(g, o, X[:77], y[:77], table, dtype, steps=2, check_internals=False)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_plain_sgd_and_smaller_batches_on_one_handle(dtype):
    # momentum 0 path; then a shorter, ragged batch on the same handle (stale pad columns must not leak)
    widths = [48, 96, 40]
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, max_batch=200, lr=0.05, mom=0.0, wseed=5)
    X, y, table = case_data(widths, api.MSE_SIL, 200, api.UNIFORM_PM1, 12, seed=2)
    check_step(g, o, X, y, table, dtype)
    check_step(g, o, X[:61], y[:61], table, dtype)
    check_step(g, o, X[3:12], y[3:12], table, dtype)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_several_steps_with_momentum(dtype):
    widths = [64, 96, 80, 32]
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, max_batch=128, lr=0.02, mom=0.9, wseed=6)
    X, y, table = case_data(widths, api.MSE_SIL, 128, api.UNIFORM01, 20, seed=4)
    check_step(g, o, X, y, table, dtype, steps=5, check_internals=(dtype == api.F32))


@pytest.mark.parametrize("widths,B", [([1024, 2048, 1024], 2048), ([256, 4096, 4096], 4096)], ids=["tiles128", "tiles256"])
def test_float32_products_on_the_larger_tiles(widths, B):
    # float32 through the 128x128 and the 256x256 tile instantiations (forward, data gradient, weight gradient)
    X, y, table = case_data(widths, api.MSE_SIL, B, api.UNIFORM_PM1, 31, seed=8)
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, api.F32, max_batch=B, lr=0.01, mom=0.9, wseed=9)
    check_step(g, o, X, y, table, api.F32)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_degenerate_shapes(dtype):
    # one sample; one unit per layer; one class (cross-entropy over a single class is 0 with zero gradient)
    X, y, table = case_data([5, 7, 3], api.MSE_SIL, 1, api.NORMAL, 4, seed=3)
    g, o = make_pair([5, 7, 3], api.RELU_ALL, api.MSE_SIL, dtype, max_batch=1, lr=0.1, mom=0.9, wseed=2)
    check_step(g, o, X, y, table, dtype)
    X, y, table = case_data([1, 1, 1], api.MSE_SIL, 17, api.UNIFORM01, 3, seed=3)
    g, o = make_pair([1, 1, 1], api.RELU_ALL, api.MSE_SIL, dtype, max_batch=17, lr=0.1, mom=0.0, wseed=4)
    check_step(g, o, X, y, table, dtype)
    X, y, _ = case_data([6, 4, 1], api.SOFTMAX_XENT, 9, None, 1, seed=3)
    g, o = make_pair([6, 4, 1], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, dtype, max_batch=9, lr=0.1, mom=0.9, wseed=5)
    W_before = [g.get_params(l)[0].clone() for l in range(2)]
    loss = g.step(as_input(X, dtype)[0], torch.from_numpy(y).to(DEV))
    assert float(loss.item()) == 0.0
    for l in range(2):
        assert torch.equal(g.get_params(l)[0], W_before[l])


def test_wide_bf16_config_one_step():
    # the wide 3|3 split at its real shape: 784-4096-4096-2048 (+-1 labels) and 2048-4096-4096-47, batch 1024
    X, y = datagen.class_mean_inputs(1024, 47, dim=784, seed=1)
    table = orng.make_synthetic_labels(13, 47, 2048, api.BINARY_PM1)
    g, o = make_pair([784, 4096, 4096, 2048], api.RELU_ALL, api.MSE_SIL, api.BF16, 1024, 0.01, 0.9, wseed=7)
    check_step(g, o, X, y, table, api.BF16)
    XB = orng.make_segment_inputs(5, table, y, 0, 0.05)
    g, o = make_pair([2048, 4096, 4096, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.BF16, 1024, 0.01, 0.9, wseed=8)
    check_step(g, o, XB, y, None, api.BF16)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_fused_update_by_layer_size(dtype):
    # rule 2: the 2100 x 2100 layer (4.41 M weights) keeps the separate update and its stored gradient, the two
    # small layers are updated inside their products
    widths, B = [64, 2100, 2100, 32], 128
    X, y, table = case_data(widths, api.MSE_SIL, B, api.UNIFORM_PM1, 20, seed=4)
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, max_batch=B, lr=0.02, mom=0.9, wseed=6)
    g.set_fused_update(2)
    check_step(g, o, X, y, table, dtype, steps=2, stored_dW=False)
    dW, _ = g.get_grads(1)                       # the large layer's gradient is there
    assert float(dW.abs().max()) > 0
    for l in (0, 2):
        with pytest.raises(api.SlpError):
            g.get_grads(l)


def test_wide_bf16_config_one_fused_step():
    # the wide configuration's first segment (784-4096-4096-2048, batch 1024, bf16): its weight gradients run on the
    # 128x128 and 256x256 tiles, here with the update in their epilogues
    widths, B = [784, 4096, 4096, 2048], 1024
    X, y, table = case_data(widths, api.MSE_SIL, B, api.BINARY_PM1, 47, seed=1)
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, api.BF16, max_batch=B, lr=0.01, mom=0.9, wseed=3)
    g.set_fused_update(True)
    check_step(g, o, X, y, table, api.BF16, stored_dW=False)


def test_tiny_config_epoch_loss_curve():
    # tiny config: 2048 blob images, batch 64, lr 0.01, one epoch, both segments, float32
    X, y = datagen.blob_images(2048, 47, 28, seed=1)
    table = orng.make_synthetic_labels(7, 47, 64, api.UNIFORM_PM1)
    gA, oA = make_pair([784, 128, 64], api.RELU_ALL, api.MSE_SIL, api.F32, 64, 0.01, 0.0, wseed=3)
    gB, oB = make_pair([64, 64, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.F32, 64, 0.01, 0.0, wseed=4)
    gA.set_labels(torch.from_numpy(table).to(DEV))
    XB = orng.make_segment_inputs(5, table, y, 0, 0.05)
    Xd, Xv = as_input(X, api.F32)
    XBd, XBv = as_input(XB, api.F32)
    yd = torch.from_numpy(y).to(DEV)
    la, lb, ra, rb = [], [], [], []
    for s in range(0, 2048, 64):
        la.append(gA.step(Xd[s:s + 64], yd[s:s + 64]).item())
        lb.append(gB.step(XBd[s:s + 64], yd[s:s + 64]).item())
        ra.append(oA.step(Xv[s:s + 64], y[s:s + 64], table)["loss"])
        rb.append(oB.step(XBv[s:s + 64], y[s:s + 64])["loss"])
    assert np.max(np.abs(np.array(la) - ra) / np.array(ra)) <= 1e-5
    assert np.max(np.abs(np.array(lb) - rb) / np.array(rb)) <= 1e-5
    for l in range(2):
        assert rel_err(to_np(gA.get_params(l)[0]), oA.W[l]) <= 1e-5
        assert rel_err(to_np(gB.get_params(l)[0]), oB.W[l]) <= 1e-5


def test_paper_shaped_config_epoch_loss_curve():
    # paper-shaped config: 112,800 inputs with 47 balanced classes, batch 256 (441 steps per epoch, the last one ragged
    # with 160 rows), lr 0.01, momentum 0.9, float32, both segments, all FIVE epochs the configuration names (2205 steps;
    # the oracle walks them in float64 at ~30 steps a second).  The two sides run free: no state and no ReLU decision
    # crosses over.  What separates them is not rounding as such but the handful of ReLU units per step that the two
    # sides see on different sides of zero: each sends one sample's gradient into a row of dW on one side only, the
    # momentum carries it for ~10 steps, and the kicks diffuse along the walk (measured: per-step loss difference 2e-6
    # after one epoch, 7e-5 / 2e-4 for the two segments after five).  The bars here are therefore wider than the
    # single step's derived 1e-5 and empirical: 5e-4 on every step's loss, 1e-4 on the epoch means.
    N, B, EPOCHS = 112800, 256, 5
    X, y = datagen.class_mean_inputs(N, 47, dim=784, seed=1)
    table = orng.make_synthetic_labels(11, 47, 512, api.NORMAL)
    gA, oA = make_pair([784, 1024, 1024, 512], api.RELU_ALL, api.MSE_SIL, api.F32, B, 0.01, 0.9, wseed=3)
    gB, oB = make_pair([512, 1024, 1024, 47], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, api.F32, B, 0.01, 0.9, wseed=4)
    gA.set_labels(torch.from_numpy(table).to(DEV))
    XB = orng.make_segment_inputs(5, table, y, 0, 0.05)
    Xd, XBd, yd = torch.from_numpy(X).to(DEV), torch.from_numpy(XB).to(DEV), torch.from_numpy(y).to(DEV)
    steps = [s for _ in range(EPOCHS) for s in range(0, N, B)]
    la = torch.zeros(len(steps), device=DEV)
    lb = torch.zeros(len(steps), device=DEV)
    for i, s in enumerate(steps):
        gA.step(Xd[s:s + B], yd[s:s + B], loss_out=la[i:i + 1])
        gB.step(XBd[s:s + B], yd[s:s + B], loss_out=lb[i:i + 1])
    Xv, XBv = X.astype(np.float64), XB.astype(np.float64)
    ra = np.array([oA.step(Xv[s:s + B], y[s:s + B], table)["loss"] for s in steps])
    rb = np.array([oB.step(XBv[s:s + B], y[s:s + B])["loss"] for s in steps])
    ea = float(np.max(np.abs(la.cpu().numpy() - ra) / ra))
    eb = float(np.max(np.abs(lb.cpu().numpy() - rb) / rb))
    per = len(steps) // EPOCHS
    means_g = [(float(la[e * per:(e + 1) * per].mean()), float(lb[e * per:(e + 1) * per].mean())) for e in range(EPOCHS)]
    means_o = [(ra[e * per:(e + 1) * per].mean(), rb[e * per:(e + 1) * per].mean()) for e in range(EPOCHS)]
    print("loss curves over %d steps: worst relative difference A %.2e, B %.2e; epoch means %s" %
          (len(steps), ea, eb, ["%.5f / %.5f" % m for m in means_o]), flush=True)
    assert per == 441 and N - steps[per - 1] == 160
    assert ea <= 5e-4 and eb <= 5e-4
    for (ga, gb), (oa, ob) in zip(means_g, means_o):
        assert abs(ga - oa) <= 1e-4 * oa and abs(gb - ob) <= 1e-4 * ob
    assert all(means_o[e + 1][0] < means_o[e][0] and means_o[e + 1][1] < means_o[e][1] for e in range(EPOCHS - 1))   # both learn
    # Weights at the end of the walk.  With nothing crossing over, a ReLU unit whose pre-activation the two sides see
    # on different sides of zero (a handful per step) sends one sample's gradient into a row of dW on one side only;
    # those kicks diffuse along the walk, so single elements drift far more than rounding alone would move them while
    # the loss curves stay together (measured after five epochs: 2e-4 to 6e-4 in the Frobenius sense, up to 6e-3 on the
    # worst element).  Compared in the Frobenius sense, with a loose bar on the worst element.
    for g_, o_ in ((gA, oA), (gB, oB)):
        for l in range(3):
            got = to_np(g_.get_params(l)[0]).astype(np.float64)
            fro = float(np.linalg.norm(got - o_.W[l]) / np.linalg.norm(o_.W[l]))
            print("layer %d: weights after the walk, relative Frobenius difference %.2e, worst element %.2e" %
                  (l, fro, rel_err(got, o_.W[l])), flush=True)
            assert fro <= 2e-3 and rel_err(got, o_.W[l]) <= 2e-2


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_forward_only_and_determinism(dtype):
    widths = [100, 300, 77]
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, max_batch=500, lr=0.01, mom=0.9, wseed=9)
    X, y, table = case_data(widths, api.MSE_SIL, 500, api.NORMAL, 7, seed=3)
    Xd, Xv = as_input(X, dtype)
    out1 = g.forward(Xd)
    assert rel_err(to_np(out1), o.forward(Xv)) <= TOL[dtype]
    out2 = g.forward(Xd)
    assert torch.equal(out1, out2)
    W0 = [g.get_params(l)[0].clone() for l in range(2)]
    for l in range(2):                                   # forward changes no parameter
        assert torch.equal(W0[l], g.get_params(l)[0])
    # two identical handles stepping on the same data stay bit-identical (fixed summation order)
    g2, _ = make_pair(widths, api.RELU_ALL, api.MSE_SIL, dtype, 500, 0.01, 0.9, wseed=9)
    tb = torch.from_numpy(table).to(DEV)
    g.set_labels(tb)
    g2.set_labels(tb)
    yd = torch.from_numpy(y).to(DEV)
    for _ in range(3):
        l1 = g.step(Xd, yd).clone()
        l2 = g2.step(Xd, yd).clone()
        assert torch.equal(l1, l2)
    for l in range(2):
        assert torch.equal(g.get_params(l)[0], g2.get_params(l)[0])


def test_forward_only_in_place_through_the_big_kernel():
    # a stored-response pass at a size that runs the 256x256 bf16 kernel: the caller's input is read in place (width a
    # multiple of 64) and the result written straight into the caller's buffer by the staged epilogue's 16-byte stores
    widths, B = [4096, 4096, 3968], 3900
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, api.BF16, max_batch=B, lr=0.01, mom=0.9, wseed=21)
    X, _, _ = case_data(widths, api.MSE_SIL, B, api.NORMAL, 7, seed=4)
    Xd, Xv = as_input(X, api.BF16)
    out = torch.full((B + 1, widths[-1]), 7.0, dtype=torch.bfloat16, device=DEV)     # one guard row behind the result
    g.forward(Xd, out=out[:B])
    assert rel_err(to_np(out[:B]), o.forward(Xv)) <= TOL[api.BF16]
    assert bool((out[B] == 7.0).all())


def test_step_argument_errors():
    g, _ = make_pair([16, 8], api.RELU_ALL, api.MSE_SIL, api.F32, 32, 0.01, 0.9, wseed=1)
    X = torch.zeros((64, 16), device=DEV)
    y = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(api.SlpError) as e:
        g.step(X[:8], y[:8])                  # no labels bound
    assert e.value.code == -5
    g.set_labels(torch.zeros((3, 8), device=DEV))
    with pytest.raises(api.SlpError) as e:
        g.step(X, y)                          # batch above max_batch
    assert e.value.code == -2
    fresh = api.Segment([16, 8], api.RELU_ALL, api.MSE_SIL, max_batch=32)
    fresh.set_labels(torch.zeros((3, 8), device=DEV))
    with pytest.raises(api.SlpError) as e:
        fresh.step(X[:8], y[:8])              # no parameters yet
    assert e.value.code == -5


@pytest.mark.parametrize("loss", [api.MSE_SIL, api.SOFTMAX_XENT])
def test_out_of_range_class_ids_are_clamped_and_counted(loss):
    # ids are the caller's data: the kernels clamp them (nothing is read out of bounds) and count the rows
    classes, B = 10, 200
    widths = [12, 20, 16] if loss == api.MSE_SIL else [12, 20, classes]
    act = api.RELU_ALL if loss == api.MSE_SIL else api.RELU_HIDDEN_IDENTITY_LAST
    X, y, table = case_data(widths, loss, B, api.UNIFORM_PM1, classes, seed=5)
    g, o = make_pair(widths, act, loss, api.F32, max_batch=B, lr=0.01, mom=0.0, wseed=5)
    if table is not None:
        g.set_labels(torch.from_numpy(table).to(DEV))
    Xd, Xv = as_input(X, api.F32)
    g.step(Xd, torch.from_numpy(y).to(DEV))
    assert g.target_errors() == 0
    bad = y.copy()
    bad[[3, 77, 199]] = [classes, -1, 1 << 20]
    loss_g = float(g.step(Xd, torch.from_numpy(bad).to(DEV)).item())
    assert g.target_errors() == 3
    o.step(Xv, y, table)                                               # the first, valid step
    ref = o.step(Xv, np.clip(bad, 0, classes - 1), table)["loss"]     # what the clamped ids mean
    assert abs(loss_g - ref) <= 1e-5 * ref


def test_mfma_probe_reports_a_rate_below_the_published_peak():
    for dtype, peak in ((api.BF16, 2516.6), (api.F32, 157.3)):
        tf, ms = api.probe_mfma_rate(dtype, iters=2000)
        assert ms > 0 and 0.05 * peak < tf < 1.02 * peak, (dtype, tf, ms)
    with pytest.raises(api.SlpError) as e:
        tf = ctypes.c_double()
        small = torch.empty(16, device=DEV)
        api._check(api.lib().slp_probe_mfma_rate(api.BF16, 10, api._ptr(small), 64, ctypes.byref(tf), None, None))
    assert e.value.code == -2


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_shapes(seed):
    # layer counts, widths and batch sizes drawn at random (seeded) around the chunk, tile and wavefront
    # boundaries: odd widths, widths of 1, batches that end inside a chunk, every loss / activation / dtype
    r = np.random.default_rng(1000 + seed)
    L = int(r.integers(1, 4))
    pool = [1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 32, 33, 47, 63, 64, 65, 100, 127, 128, 129, 200, 255, 256, 257, 300]
    widths = [int(r.choice(pool)) for _ in range(L + 1)]
    B = int(r.choice([1, 2, 5, 8, 31, 32, 33, 64, 100, 129, 257, 300]))
    dtype = api.BF16 if seed % 2 else api.F32
    if r.integers(0, 2):
        act, loss, classes = api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, widths[-1]
        dist = None
    else:
        act, loss, classes = (api.RELU_ALL if r.integers(0, 2) else api.RELU_HIDDEN_IDENTITY_LAST), api.MSE_SIL, int(r.integers(1, 20))
        dist = int(r.choice([api.UNIFORM01, api.UNIFORM_PM1, api.NORMAL, api.BINARY_PM1]))
    mom = 0.9 if r.integers(0, 2) else 0.0
    X, y, table = case_data(widths, loss, B, dist, classes, seed=seed + 3)
    g, o = make_pair(widths, act, loss, dtype, max_batch=B + int(r.integers(0, 9)), lr=0.05, mom=mom, wseed=seed)
    print("shape", widths, "batch", B, "dtype", dtype, "loss", loss, "act", act, flush=True)
    check_step(g, o, X, y, table, dtype, steps=2)


@pytest.mark.parametrize("widths,B,max_batch", [([4000, 4090, 3999], 3900, 3900), ([4000, 4400, 4100], 3900, 3900),
                                                ([4000, 4090, 3999], 3850, 4000)], ids=["regions", "groups", "regions-batch-below-max"])
def test_bf16_products_on_the_big_tile_with_ragged_edges(widths, B, max_batch):
    # every product of these steps has 224 or more 256x256 tiles, so all run through the big bf16 kernel, with ragged
    # last tiles in rows, columns and contraction: 16 x 16 tile grids (walked by regions) in the first case, 16 x 18
    # and 18 x 17 grids (walked by groups of tile rows) in the second.  The hidden layer's ReLU mask travels from the
    # forward product to the data gradient as bits, 128 batch rows per group of 4 dwords: the last wavefront row of the
    # tile grid lies wholly beyond the batch in all three cases, and in the third the buffers are laid out for a larger
    # batch than the step uses.
    X, y, table = case_data(widths, api.MSE_SIL, B, api.NORMAL, 29, seed=12)
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, api.BF16, max_batch=max_batch, lr=0.05, mom=0.9, wseed=13)
    check_step(g, o, X, y, table, api.BF16)


@pytest.mark.parametrize("seed", range(6))
def test_seeded_random_mid_size_shapes(seed):
    # ragged sizes large enough to reach the 64x64, 128x128 (both forms) and 256x256 tile instantiations
    r = np.random.default_rng(2000 + seed)
    pool = [520, 777, 1000, 1234, 1999, 2500, 3100]
    widths = [int(r.choice(pool)) for _ in range(3)]
    B = int(r.choice([1000, 1500, 2100, 4100]))
    dtype = api.BF16 if seed % 2 else api.F32
    if seed % 3 == 0:
        act, loss, classes, dist = api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, widths[-1], None
    else:
        act, loss, classes, dist = api.RELU_ALL, api.MSE_SIL, 33, api.NORMAL
    X, y, table = case_data(widths, loss, B, dist, classes, seed=seed + 5)
    g, o = make_pair(widths, act, loss, dtype, max_batch=B, lr=0.05, mom=0.9, wseed=seed + 40)
    print("shape", widths, "batch", B, "dtype", dtype, "loss", loss, flush=True)
    check_step(g, o, X, y, table, dtype)
