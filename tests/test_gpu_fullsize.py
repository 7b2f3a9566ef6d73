"""The large configurations at their real shapes and in the launch configuration the
benchmark times (bf16, 256x256 tiles, region walk).

Segments of the deep configuration (width 8192, batch 4096) go through a FULL oracle
step and are compared element by element like the small cases.  A full oracle step of
a 16384-wide segment at batch 8192 is ~27 TFLOP of float64 work, so there:
  * sampled batch rows -- one in every 256-row tile of the matrix products, the rows on
    either side of tile and region boundaries, first and last -- are pushed through the
    oracle's whole forward and backward chain (a row of A_l / dZ_l depends on the other
    rows only through the batch size in the means) and compared element by element
    (ReLU decisions are taken over from the device only inside the oracle's own rounding
    bound, and the rows without such a tie are also compared with no decision taken over);
  * sampled entries of every weight gradient -- one in every 256x256 tile of dW and at
    least 2000 -- are compared with the oracle's definition summed over every row of the
    batch, applied to the device's dZ_l and A_{l-1} columns; the bias gradient likewise
    on the sampled columns;
  * what needs every element at once (loss, the whole of dW and db, the update) is
    checked through properties that hold at any size: the loss against its definition on
    the device's own output, dW against a random projection, the update against
    w - lr * dW.
"""

import numpy as np
import pytest
import torch

from oracle import rng as orng
from oracle import segment as osg
from paper_2403_11204_amd import api, datagen
from test_gpu_parity import U32, check_step, compare_rows_without_ties, make_pair, tie_report

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

TOL = 2e-2
DEV = "cuda"


def f64(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def sample_rows(B):
    """One row in every 256-row tile (at a varying offset), both sides of the 16-tile region boundaries, ends."""
    rows = {0, 1, B - 1}
    for t in range((B + 255) // 256):
        rows.add(min(B - 1, t * 256 + (37 * t + 5) % 256))
    for edge in range(4096, B, 4096):
        rows.update((edge - 1, edge))
    return np.array(sorted(rows))


def run_full_size(widths, act, loss, B, classes, Xd, y, table, params, lr=0.01):
    """One step at full size on the device; sampled rows against the oracle chain; sampled gradient entries against
    the definition; whole-batch properties."""
    L = len(widths) - 1
    seg = api.Segment(widths, act, loss, max_batch=B, dtype=api.BF16, lr=lr, momentum=0.9)
    for l, (W, b) in enumerate(params):
        seg.set_params(l, torch.from_numpy(W), torch.from_numpy(b))
    if table is not None:
        seg.set_labels(torch.from_numpy(table).to(DEV))
    yd = torch.from_numpy(y).to(DEV)
    loss_gpu = float(seg.step(Xd, yd).item())
    print("full-size step done, loss", loss_gpu, flush=True)

    # ---- sampled rows through the oracle chain ---------------------------------------
    rows = sample_rows(B)
    ora = osg.Segment(widths, act, loss, lr=lr, momentum=0.9, mode="bf16")
    for l, (W, b) in enumerate(params):
        ora.set_params(l, W, b)
    ridx = torch.from_numpy(rows).to(DEV)
    Xrows = f64(Xd[ridx])
    acts = [None] + [f64(seg.get_activation(l, B)[ridx]) for l in range(1, L + 1)]
    dzs = [None] + [f64(seg.get_activation(l, B, kind=1)[ridx]) for l in range(1, L + 1)]
    bounds = ora.forward_error_bound(Xrows, unit=U32)
    out = ora.step(Xrows, y[rows], table, update=False, full_batch=B, tie_decisions=[None] + [a > 0 for a in acts[1:]],
                   tie_bounds=bounds)
    print("oracle: %d rows" % len(rows), flush=True)
    tie_report(out, bounds)
    assert out["decisions_refused"] == 0
    assert out["ties_taken"] <= max(1, int(1e-3 * sum(a.size for a in acts[1:])))
    for l in range(L, 0, -1):
        a_ref = out["A"][l]
        assert np.max(np.abs(acts[l] - a_ref)) <= TOL * np.max(np.abs(a_ref)), ("A", l)
        dz_ref = out["dZ"][l]
        assert np.max(np.abs(dzs[l] - dz_ref)) <= TOL * np.max(np.abs(dz_ref)), ("dZ", l)
    if out["ties_taken"]:        # rows without a tie at the layers that matter to them, with no decision taken over
        free = ora.step(Xrows, y[rows], table, update=False, full_batch=B)
        n = compare_rows_without_ties(out, free, acts, dzs, TOL)
        print("(row, layer) pairs of dZ compared with no decision taken over: %d of %d" % (n, len(rows) * L), flush=True)
        assert n > 0
        del free
    del ora, out, bounds

    # ---- properties over the whole batch ---------------------------------------------------
    A = [Xd] + [seg.get_activation(l, B) for l in range(1, L + 1)]
    dZ = [None] + [seg.get_activation(l, B, kind=1) for l in range(1, L + 1)]
    if loss == api.MSE_SIL:
        T = torch.from_numpy(table).to(DEV)[yd.long()]
        diff = A[L].double() - T.double()
        loss_def = float((diff * diff).mean().item())      # definition of the loss on the device's own output
    else:
        Z = A[L].double()
        loss_def = float((torch.logsumexp(Z, dim=1) - Z.gather(1, yd.long()[:, None])[:, 0]).mean().item())
    assert abs(loss_gpu - loss_def) <= 1e-5 * loss_def
    gen = torch.Generator(device="cpu").manual_seed(5)
    rs = np.random.default_rng(17)
    for l in range(L):
        dW, db = seg.get_grads(l)
        N, K = widths[l + 1], widths[l]
        # sampled entries against the definition, summed over the whole batch on the host in float64: one entry at a
        # random place inside every 256x256 tile of dW, then random ones up to 2000
        tn, tk = (N + 255) // 256, (K + 255) // 256
        oi = (np.repeat(np.arange(tn), tk) * 256 + rs.integers(0, 256, tn * tk)).clip(max=N - 1)
        ki = (np.tile(np.arange(tk), tn) * 256 + rs.integers(0, 256, tn * tk)).clip(max=K - 1)
        extra = max(0, 2000 - len(oi))
        oi = np.concatenate([oi, rs.integers(0, N, extra)])
        ki = np.concatenate([ki, rs.integers(0, K, extra)])
        ref, scale = osg.weight_gradient_elements(f64(dZ[l + 1][:, torch.from_numpy(oi).to(DEV)]),
                                                  f64(A[l][:, torch.from_numpy(ki).to(DEV)]))
        got = f64(dW[torch.from_numpy(oi).to(DEV), torch.from_numpy(ki).to(DEV)])
        # float32 accumulation of B exact products, any order: sqrt(B) unit roundoffs of the absolute sum (+ final rounding)
        err = np.abs(got - ref)
        allowed = (np.sqrt(B) + 2.0) * U32 * scale + 1e-30
        assert np.all(err <= allowed), ("dW entries", l, float(np.max(err / allowed)))
        print("layer %d: %d sampled dW entries, worst error / bound %.3f" % (l, len(oi), float(np.max(err / allowed))), flush=True)
        uo = np.unique(oi)
        cols = f64(dZ[l + 1][:, torch.from_numpy(uo).to(DEV)])
        db_ref, db_scale = cols.sum(axis=0), np.abs(cols).sum(axis=0)
        assert np.all(np.abs(f64(db[torch.from_numpy(uo).to(DEV)]) - db_ref) <= (np.sqrt(B) + 2.0) * U32 * db_scale + 1e-30), ("db entries", l)
        del cols
        r = torch.randn(widths[l], generator=gen, dtype=torch.float64).to(DEV)
        # dW r = dZ^T (A r): a wrong tile, a dropped k-slice or a transposed operand breaks this
        lhs = dW.double() @ r
        rhs = dZ[l + 1].double().T @ (A[l].double() @ r)
        assert float((lhs - rhs).abs().max() / rhs.abs().max()) <= 1e-4, ("dW", l)
        col = dZ[l + 1].double().sum(dim=0)
        assert float((db.double() - col).abs().max() / col.abs().max()) <= 1e-4, ("db", l)
        # first step from zero momentum: v = dW, w_new = w_old - lr * dW (float32 arithmetic)
        Wn, bn = seg.get_params(l)
        W0 = torch.from_numpy(params[l][0]).to(DEV)
        expect = W0 - lr * dW
        assert float((Wn - expect).abs().max()) <= 2 * float(np.spacing(np.float32(W0.abs().max().item()))), ("W", l)
        vW, _ = seg.get_momentum(l)
        assert torch.equal(vW, dW)
        del dW, Wn, W0, expect, vW
    del seg
    torch.cuda.empty_cache()


def test_comparison_config_segment_a_full_size():
    widths, B, classes = [784, 16384, 16384, 16384], 8192, 1000
    X, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1)
    table = orng.make_synthetic_labels(31, classes, widths[-1], orng.UNIFORM_PM1)
    Xd = torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous()
    run_full_size(widths, api.RELU_ALL, api.MSE_SIL, B, classes, Xd, y, table, datagen.uniform_weights(widths, seed=17))


def test_comparison_config_segment_b_full_size():
    # the final segment: inputs are the cut's label of the class plus noise, 1000-way cross-entropy (its last
    # layer is the skinny product, 1000 columns)
    widths, B, classes = [16384, 16384, 16384, 1000], 8192, 1000
    _, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1)
    cut = api.make_synthetic_labels(31, classes, widths[0], api.UNIFORM_PM1, 1.0, api.F32)
    Xd = api.make_segment_inputs(6, cut, torch.from_numpy(y).to(DEV), 0, 0.05, api.BF16)
    run_full_size(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, B, classes, Xd, y, None,
                  datagen.uniform_weights(widths, seed=18))


def deep_inputs(B, classes, width, label_seed):
    _, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1)
    cut = orng.make_synthetic_labels(label_seed, classes, width, orng.NORMAL)
    return y, orng.make_segment_inputs(6, cut, y, 0, 0.05)


@pytest.mark.parametrize("which", ["S1", "S2", "S4"])
def test_deep_config_segments_full_oracle_step(which):
    # the 12-layer configuration's segments at their real shape (width 8192, batch 4096, bf16): a full oracle step,
    # every tensor compared element by element.  S1: 784-d data in, N(0,1) labels; S2 (= S3): label + noise in, N(0,1)
    # labels; S4: label + noise in, 100-way cross-entropy.
    B, classes = 4096, 100
    if which == "S1":
        widths, act, loss = [784, 8192, 8192, 8192], api.RELU_ALL, api.MSE_SIL
        X, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1)
        table = orng.make_synthetic_labels(21, classes, 8192, orng.NORMAL)
    elif which == "S2":
        widths, act, loss = [8192, 8192, 8192, 8192], api.RELU_ALL, api.MSE_SIL
        y, X = deep_inputs(B, classes, 8192, 21)
        table = orng.make_synthetic_labels(22, classes, 8192, orng.NORMAL)
    else:
        widths, act, loss = [8192, 8192, 8192, 100], api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT
        y, X = deep_inputs(B, classes, 8192, 23)
        table = None
    g, o = make_pair(widths, act, loss, api.BF16, max_batch=B, lr=0.01, mom=0.9, wseed=19)
    check_step(g, o, X, y, table, api.BF16, tie_cap=1e-3)
    del g, o
    torch.cuda.empty_cache()


def test_comparison_config_end_to_end_network_full_size():
    # the conventional baseline of the comparison: all six layers in one segment, 1000-way cross-entropy
    widths, B, classes = [784, 16384, 16384, 16384, 16384, 16384, 1000], 8192, 1000
    X, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1)
    Xd = torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous()
    run_full_size(widths, api.RELU_HIDDEN_IDENTITY_LAST, api.SOFTMAX_XENT, B, classes, Xd, y, None,
                  datagen.uniform_weights(widths, seed=20))


def test_largest_addressable_layer_float32():
    # one 23168 x 23168 float32 layer: 2,147,024,896 bytes per matrix, 458,752 below the 2 GiB operand limit, so the
    # 32-bit byte offsets of the matrix products run up to the end of their range; ragged batch
    widths, B = [23168, 23168], 200
    X, y = datagen.class_mean_inputs(B, 7, dim=widths[0], seed=2)
    table = orng.make_synthetic_labels(9, 7, widths[1], orng.UNIFORM_PM1)
    g, o = make_pair(widths, api.RELU_ALL, api.MSE_SIL, api.F32, max_batch=B, lr=0.01, mom=0.9, wseed=23)
    check_step(g, o, X, y, table, api.F32)
    del g, o
    torch.cuda.empty_cache()


def test_largest_addressable_batch_bf16():
    # 64768 rows of 16384 bf16 values in rows of 16576 elements (the library skews rows that would be a multiple of
    # 4 KB): 2,147,188,736 bytes per activation matrix, one 64-row step below the 2 GiB operand limit (64832 rows are
    # rejected at create time); one 16384 x 16384 layer
    widths, B, classes = [16384, 16384], 64768, 10
    _, y = datagen.class_mean_inputs(B, classes, dim=8, seed=1)
    cut = api.make_synthetic_labels(41, classes, widths[0], api.UNIFORM_PM1, 1.0, api.F32)
    Xd = api.make_segment_inputs(7, cut, torch.from_numpy(y).to(DEV), 0, 0.05, api.BF16)
    table = orng.make_synthetic_labels(42, classes, widths[-1], orng.NORMAL)
    run_full_size(widths, api.RELU_ALL, api.MSE_SIL, B, classes, Xd, y, table, datagen.uniform_weights(widths, seed=29))
