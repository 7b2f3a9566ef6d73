"""Oracle: one independent training step of one network segment.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What the paper fixes (Sec. 2 and Sec. 3): a fully connected segment with bias,
ReLU after every layer except the network's last one (identity there); a
non-final segment is trained on its inputs against the synthetic intermediate
label of each sample's class, the final segment against the true classes;
stochastic gradient descent with a learning rate and momentum; no shuffling;
gradients never leave the segment.

Readings where the paper is silent (loss functions are never named):
  * non-final segment: mean squared error, mean over batch x width;
  * final segment: softmax cross-entropy, mean over the batch;
  * ReLU' (0) = 0;
  * momentum: v <- mu v + g, theta <- theta - lr v, v0 = 0, no dampening,
    no Nesterov, no weight decay.

The step is the textbook definition in float64:

  A_0 = X;  Z_l = A_{l-1} W_l^T + b_l;  A_l = relu(Z_l)  (or Z_L on an
  identity-last segment)
  MSE :  loss = mean (A_L - T[y])^2 ;  G = 2 (A_L - T[y]) / (B D)
  CE  :  loss = mean_n (lse(Z_L[n]) - Z_L[n, y_n]) ;  G = (softmax - onehot) / B
  dZ_L = G * [A_L > 0]  (ReLU on the last layer)  or  G
  dW_l = dZ_l^T A_{l-1};  db_l = sum_n dZ_l[n];  dZ_{l-1} = (dZ_l W_l) * [A_{l-1} > 0]
  (no data gradient is formed for the segment's first layer)

``mode='bf16'`` emulates a mixed-precision run: float32 master parameters, and a
rounding to bfloat16 (nearest even) at exactly the points where such a run
stores bf16 -- the inputs, the weight copy used by the products, every stored
activation A_l and every dZ_l; products accumulate in float64 in between;
biases, loss, dW, db, momentum and master weights are not rounded to bf16.

parity pins: tests/test_oracle_segment.py (hand-worked network, closed forms,
central finite differences, an automatic-differentiation library in float64,
normal equations, SGD closed form, loss decrease on a separable toy set, the
parameter and multiply-accumulate counts printed in paper Sec. 3; the rounding
bounds that decide ReLU ties against a float32 implementation and brute force).
"""

import numpy as np

RELU_ALL, RELU_HIDDEN_IDENTITY_LAST = 0, 1
MSE_SIL, SOFTMAX_XENT = 0, 1


def _bf16(x):
    """float64 -> float32 -> nearest-even bfloat16, returned as float64."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    b = x32.view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = ((b + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(x32.shape).astype(np.float64)


def param_count(widths):
    """Weights plus biases of a segment (paper Sec. 3 prints 67660 and 10187)."""
    return sum((widths[l] + 1) * widths[l + 1] for l in range(len(widths) - 1))


def mac_count(widths, act):
    """Multiply-accumulates per sample as the paper's counter reports them
    (Sec. 3: 67800 and 10307): one per weight, one per bias, one per ReLU
    output."""
    L = len(widths) - 1
    macs = param_count(widths)
    for l in range(1, L + 1):
        if l < L or act == RELU_ALL:
            macs += widths[l]
    return macs


def gemm_flops_per_sample(widths):
    """2 FLOP per multiply-add over forward, weight-gradient and data-gradient
    products; the first layer has no data gradient."""
    P = sum(widths[l] * widths[l + 1] for l in range(len(widths) - 1))
    return 6 * P - 2 * widths[0] * widths[1]


def count_correct(logits, y):
    """Rows whose largest logit sits at the row's class (paper Sec. 4 reports the joined
    network's accuracy on the test set: this count over the number of rows).  Among equal
    maxima the lowest index is the prediction."""
    logits = np.asarray(logits)
    y = np.asarray(y, dtype=np.int64)
    return int(np.sum(np.argmax(logits, axis=1) == y))


def mean_loss(losses):
    """Epoch figure of a training curve: the mean of its per-step losses."""
    return float(np.mean(np.asarray(losses, dtype=np.float64)))


def weight_gradient_elements(dZ_cols, A_cols):
    """Sampled entries of a weight gradient from their definition: entry s is
    dW[o_s, k_s] = sum_n dZ[n, o_s] A[n, k_s], with dZ_cols[:, s] = dZ[:, o_s] and
    A_cols[:, s] = A[:, k_s] (every row of the batch), summed in float64.  Also returns
    sum_n |dZ[n, o_s] A[n, k_s]|, the scale a float32 accumulation's error is bounded by."""
    dZ_cols = np.asarray(dZ_cols, dtype=np.float64)
    A_cols = np.asarray(A_cols, dtype=np.float64)
    assert dZ_cols.shape == A_cols.shape
    prod = dZ_cols * A_cols
    return prod.sum(axis=0), np.abs(prod).sum(axis=0)


class Segment:
    def __init__(self, widths, act, loss, lr=0.01, momentum=0.0, mode="fp32"):
        assert len(widths) >= 2 and all(w > 0 for w in widths)
        assert act in (RELU_ALL, RELU_HIDDEN_IDENTITY_LAST)
        assert loss in (MSE_SIL, SOFTMAX_XENT)
        assert mode in ("fp32", "bf16")
        self.widths = list(widths)
        self.L = len(widths) - 1
        self.act, self.loss, self.mode = act, loss, mode
        self.lr, self.mu = float(lr), float(momentum)
        self.W = [np.zeros((widths[l + 1], widths[l])) for l in range(self.L)]
        self.b = [np.zeros(widths[l + 1]) for l in range(self.L)]
        self.vW = [np.zeros_like(w) for w in self.W]
        self.vb = [np.zeros_like(b) for b in self.b]

    def set_params(self, layer, W, b):
        assert W.shape == self.W[layer].shape and b.shape == self.b[layer].shape
        self.W[layer] = np.array(W, dtype=np.float64)
        self.b[layer] = np.array(b, dtype=np.float64)

    # -- storage-point rounding ------------------------------------------------
    def _store(self, x):
        return _bf16(x) if self.mode == "bf16" else x

    def _weights_for_products(self):
        return [self._store(w) for w in self.W]

    def _relu_on(self, l):       # l is 1-based
        return l < self.L or self.act == RELU_ALL

    # -- forward -----------------------------------------------------------------
    def forward_all(self, X):
        """Returns (A, Z): A[0..L] stored activations, Z[1..L] pre-activations."""
        Wp = self._weights_for_products()
        A = [self._store(np.asarray(X, dtype=np.float64))]
        Z = [None]
        for l in range(1, self.L + 1):
            z = A[l - 1] @ Wp[l - 1].T + self.b[l - 1]
            a = np.maximum(z, 0.0) if self._relu_on(l) else z
            Z.append(z)
            A.append(self._store(a))
        return A, Z

    def forward(self, X):
        return self.forward_all(X)[0][-1]

    # -- loss and its gradient w.r.t. the stored last activation -----------------
    def loss_and_grad(self, AL, y, table=None, full_batch=None):
        """Loss and its gradient for the given rows.  ``full_batch`` is the size of
        the batch the means run over when the rows are only a sample of it (the
        returned loss is then these rows' share of the batch mean)."""
        rows, D = AL.shape
        B = rows if full_batch is None else int(full_batch)
        y = np.asarray(y, dtype=np.int64)
        if self.loss == MSE_SIL:
            T = np.asarray(table, dtype=np.float64)[y]
            diff = AL - T
            loss = float(np.sum(diff * diff) / (B * D))
            G = 2.0 * diff / (B * D)
        else:
            m = AL.max(axis=1, keepdims=True)
            lse = m[:, 0] + np.log(np.sum(np.exp(AL - m), axis=1))
            loss = float(np.sum(lse - AL[np.arange(rows), y]) / B)
            G = np.exp(AL - lse[:, None])
            G[np.arange(rows), y] -= 1.0
            G /= B
        return loss, G

    # -- how far another implementation's pre-activations may lie from these -----------
    def _stored_deviation(self, pre, E):
        """Bound on |stored(pre') - stored(pre)| for any pre' with |pre' - pre| <= E, where
        ``stored`` is what this mode keeps: the value itself (fp32 mode) or its nearest-even
        bfloat16 (bf16 mode: the two roundings agree unless a rounding boundary -- the
        midpoint between two neighbouring bfloat16 numbers -- lies within E of pre; then they
        differ by at most E plus one spacing of the larger of the two)."""
        if self.mode != "bf16":
            return E
        m = np.abs(np.asarray(pre, dtype=np.float64))
        r = _bf16(m)                                         # nearest bfloat16 of the magnitude
        rb = r.astype(np.float32).view(np.uint32).astype(np.int64)
        up = (rb + 0x10000).astype(np.uint32).view(np.float32).astype(np.float64)
        dn = np.where(rb >= 0x10000, (np.maximum(rb, 0x10000) - 0x10000).astype(np.uint32).view(np.float32).astype(np.float64), -up)
        dist = np.minimum(0.5 * (r + up) - m, m - 0.5 * (r + dn))
        # off by at most E plus half a spacing on either side; the spacing is taken at the far end m + E
        r2 = _bf16(m + E)
        up2 = (r2.astype(np.float32).view(np.uint32).astype(np.int64) + 0x10000).astype(np.uint32).view(np.float32).astype(np.float64)
        return np.where(dist <= E, E + (up2 - r2), 0.0)

    def forward_error_bound(self, X, unit=2.0 ** -24, lam=1.0, lam_prop=4.0, param_rel=0.0, input_dev=None,
                            with_output_dev=False):
        """Per-element bounds E[l] (l = 1..L, shape of Z[l]) on |Z_l' - Z_l|, where Z_l is this
        oracle's pre-activation and Z_l' that of ANOTHER implementation of the same forward
        pass which (a) accumulates every dot product of K terms in an arithmetic of unit
        roundoff ``unit`` in any order, (b) stores what this oracle's mode stores, and (c)
        holds parameters within param_rel * max|W_l| (max|b_l|) of this oracle's, and (d) is
        fed inputs within input_dev (same shape as X; None = the same inputs) of X.  Computed
        from this oracle's own values only:

            E_l = (lam sqrt(K_l) + 2) unit (|A_{l-1}| |W_l|^T + |b_l|)
                  + lam_prop sqrt( dA_{l-1}^2 (W_l^2)^T + A_{l-1}^2 (dW_l^2)^T + db_l^2 )

        First term, rounding inside layer l: the forward error bound of a length-K
        floating-point sum, |fl(s) - s| <= lam sqrt(K) unit sum|a_k w_k|, i.e. the worst-case
        bound K unit sum|a_k w_k| with the square root of its constant taken (rounding errors
        of either sign partly cancel; Higham and Mary, SIAM J. Sci. Comput. 41 (2019), give
        the probabilistic proof of that rule), plus the bias addition and the final rounding.
        Products of two bfloat16 numbers are exact in float32, so in both modes only the
        additions round.
        Second term, what the layer inherits: its inputs deviate by at most dA_{l-1} and its
        parameters by dW_l, db_l, element by element, with signs that are independent of one
        another, so the sum of the K deviations dA_k w_k stays within lam_prop times the root
        of the sum of their squared bounds (Hoeffding's inequality; failure probability
        2 exp(-lam_prop^2 / 2) = 7e-4 at 4), not within the sum of the bounds themselves.
        dA_l, the deviation of the stored activation, follows from E_l: a ReLU does not
        enlarge a difference, and a unit whose pre-activation is below -E_l is zero on both
        sides; bf16 storage either agrees or is off by one spacing (see _stored_deviation).
        Used to decide where a ReLU decision that differs from this oracle's is a tie.
        with_output_dev: also return dA_L, the bound on the deviation of the stored output
        (the input_dev of whatever segment is fed with it)."""
        A, Z = self.forward_all(X)
        E = [None] * (self.L + 1)
        dA = None if input_dev is None else np.asarray(input_dev, dtype=np.float64)
        for l in range(1, self.L + 1):
            W, b = self.W[l - 1], self.b[l - 1]
            Wp = self._store(W)
            K = self.widths[l - 1]
            e = (lam * np.sqrt(K) + 2.0) * unit * (np.abs(A[l - 1]) @ np.abs(Wp).T + np.abs(b))
            inherited = 0.0
            if dA is not None:
                inherited = (dA * dA) @ (Wp * Wp).T
            if param_rel > 0.0:
                dW = self._stored_deviation(W, np.full(W.shape, param_rel * np.max(np.abs(W))))
                inherited = inherited + (A[l - 1] * A[l - 1]) @ (dW * dW).T + (param_rel * np.max(np.abs(b))) ** 2
            E[l] = e + lam_prop * np.sqrt(inherited)
            if self._relu_on(l):
                dA = np.where(Z[l] < -E[l], 0.0, self._stored_deviation(np.maximum(Z[l], 0.0), E[l]))
            else:
                dA = self._stored_deviation(Z[l], E[l])
        return (E, dA) if with_output_dev else E

    # -- backward pass shared by every kind of step ---------------------------------------
    def _backward(self, A, Z, dZ_L, first_layer, want_param_grads, tie_decisions=None, tie_bounds=None):
        """dZ_L is the (already masked and stored) gradient w.r.t. the last pre-activation.
        Walks l = L..1: dW_l = dZ_l^T A_{l-1}, db_l = sum_n dZ_l[n], and for l > first_layer
        dZ_{l-1} = (dZ_l W_l) * [A_{l-1} > 0]; with first_layer = 0 the walk ends with the
        gradient w.r.t. the segment input, dZ[0] = dZ_1 W_1 (no mask: the input is not a
        ReLU output of this segment).  Returns (dZ, dW, db, tie report)."""
        Wp = self._weights_for_products()
        rep = _TieReport(A[0].shape[0])
        dZ = [None] * (self.L + 1)
        dW, db = [None] * self.L, [None] * self.L
        dZ[self.L] = dZ_L
        for l in range(self.L, 0, -1):
            if want_param_grads:
                dW[l - 1] = dZ[l].T @ A[l - 1]
                db[l - 1] = dZ[l].sum(axis=0)
            if l > 1 and l > first_layer:
                dZ[l - 1] = self._store((dZ[l] @ Wp[l - 1]) * _active(A, Z, l - 1, tie_decisions, tie_bounds, rep))
            elif l == 1 and first_layer == 0:
                dZ[0] = self._store(dZ[1] @ Wp[0])
        return dZ, dW, db, rep

    def apply_update(self, dW, db):
        """v <- mu v + g; theta <- theta - lr v (paper Sec. 3: SGD with momentum)."""
        for l in range(self.L):
            self.vW[l] = self.mu * self.vW[l] + dW[l]
            self.vb[l] = self.mu * self.vb[l] + db[l]
            self.W[l] = self.W[l] - self.lr * self.vW[l]
            self.b[l] = self.b[l] - self.lr * self.vb[l]
            if self.mode == "bf16":     # master parameters live in float32
                self.W[l] = self.W[l].astype(np.float32).astype(np.float64)
                self.b[l] = self.b[l].astype(np.float32).astype(np.float64)

    # -- one training step ---------------------------------------------------------
    def step(self, X, y, table=None, update=True, full_batch=None, tie_decisions=None, tie_bounds=None):
        """Forward, loss, backward, SGD.  Returns a dict with everything a
        parity test wants to look at (values *before* the update for A, Z, dZ,
        dW, db; parameters are updated in place).  With ``full_batch`` the rows
        are a sample of a larger batch: A, Z and dZ of those rows are exact (they
        depend on the rest of the batch only through its size); loss is then these
        rows' share, dW and db are not formed and no update may be asked for.

        ``tie_decisions``: whether a ReLU unit passes gradient is an integer decided
        from a floating-point pre-activation; where that value is zero to within the
        rounding error of the arithmetic, "active" and "inactive" are both correct, and
        two correct implementations may differ.  tie_decisions[l] (l = 1..L, boolean,
        shape of A[l]) holds another implementation's decisions; one is taken over ONLY
        where it differs from this oracle's and |Z_l| <= tie_bounds[l] element by element
        (tie_bounds from forward_error_bound: there, and only there, the other
        implementation's pre-activation can have the other sign).  The result reports
        the decisions taken over ("ties_taken"), the batch rows they sit in
        ("tie_rows", and per layer "tie_rows_by_layer": dZ_l of a row is untouched by them
        when the row has none at layers l..L), the largest |Z| / bound among them
        ("worst_tie_ratio") and the
        disagreements outside the bounds ("decisions_refused": those are the other
        side's errors; the oracle keeps its own decision there)."""
        assert full_batch is None or not update
        assert tie_decisions is None or tie_bounds is not None
        A, Z = self.forward_all(X)
        loss, G = self.loss_and_grad(A[self.L], y, table, full_batch)
        rep0 = _TieReport(A[0].shape[0])
        g = G * _active(A, Z, self.L, tie_decisions, tie_bounds, rep0) if self._relu_on(self.L) else G
        dZ, dW, db, rep = self._backward(A, Z, self._store(g), 1, full_batch is None, tie_decisions, tie_bounds)
        rep.merge(rep0)
        if update:
            self.apply_update(dW, db)
        return {"loss": loss, "A": A, "Z": Z, "dZ": dZ, "dW": dW, "db": db, **rep.as_dict()}

    # -- recovery phase (paper Sec. 5) -------------------------------------------------
    # After both partitions are trained, the left one is trained some more *through* the
    # right one, whose weights stay frozen: the loss is the right partition's
    # classification loss on the left partition's response.  That needs two more
    # operations: the gradient of a segment's loss with respect to its INPUT (no parameter
    # gradient, no update), and a training step that starts from a gradient handed in from
    # outside instead of from the segment's own loss.
    def input_gradient(self, X, y, table=None, tie_decisions=None, tie_bounds=None):
        """Forward, loss, and backpropagation through every layer down to the input.
        Parameters are not touched.  Returns {"loss", "dX", "A", "Z", "dZ", tie report}; dX
        is d loss / d X (rounded to bf16 in bf16 mode, like every stored gradient)."""
        assert tie_decisions is None or tie_bounds is not None
        A, Z = self.forward_all(X)
        loss, G = self.loss_and_grad(A[self.L], y, table)
        rep0 = _TieReport(A[0].shape[0])
        g = G * _active(A, Z, self.L, tie_decisions, tie_bounds, rep0) if self._relu_on(self.L) else G
        dZ, _, _, rep = self._backward(A, Z, self._store(g), 0, False, tie_decisions, tie_bounds)
        rep.merge(rep0)
        return {"loss": loss, "dX": dZ[0], "A": A, "Z": Z, "dZ": dZ, **rep.as_dict()}

    def step_external(self, X, dA_out, update=True, tie_decisions=None, tie_bounds=None):
        """A training step driven by dA_out = d loss / d (segment output), supplied by
        whatever sits behind the segment.  dZ_L = dA_out * [A_L > 0] when the last
        layer has a ReLU, else dA_out; then the usual backward pass and SGD update."""
        assert tie_decisions is None or tie_bounds is not None
        A, Z = self.forward_all(X)
        g = self._store(np.asarray(dA_out, dtype=np.float64))
        rep0 = _TieReport(A[0].shape[0])
        if self._relu_on(self.L):
            g = self._store(g * _active(A, Z, self.L, tie_decisions, tie_bounds, rep0))
        dZ, dW, db, rep = self._backward(A, Z, g, 1, True, tie_decisions, tie_bounds)
        rep.merge(rep0)
        if update:
            self.apply_update(dW, db)
        return {"A": A, "Z": Z, "dZ": dZ, "dW": dW, "db": db, **rep.as_dict()}


class _TieReport:
    def __init__(self, rows):
        self.taken, self.refused, self.worst = 0, 0, 0.0
        self.n = rows
        self.rows = {}                      # layer -> batch rows with a decision taken over at that layer

    def merge(self, other):
        self.taken += other.taken
        self.refused += other.refused
        self.worst = max(self.worst, other.worst)
        for l, r in other.rows.items():
            self.rows[l] = self.rows.get(l, np.zeros(self.n, dtype=bool)) | r

    def as_dict(self):
        any_row = np.zeros(self.n, dtype=bool)
        for r in self.rows.values():
            any_row |= r
        return {"ties_taken": self.taken, "decisions_refused": self.refused, "worst_tie_ratio": self.worst,
                "tie_rows": any_row, "tie_rows_by_layer": dict(self.rows)}


def _active(A, Z, l, tie_decisions, tie_bounds, rep):
    """Which units of layer l pass gradient: [A_l > 0] (ReLU'(0) = 0), with another
    implementation's decision taken over at ties (see Segment.step)."""
    own = A[l] > 0.0
    if tie_decisions is None or tie_decisions[l] is None:
        return own
    other = np.asarray(tie_decisions[l], dtype=bool)
    differ = own != other
    near = np.abs(Z[l]) <= tie_bounds[l]
    take = differ & near
    if take.any():
        rep.taken += int(np.sum(take))
        rep.worst = max(rep.worst, float(np.max(np.abs(Z[l][take]) / tie_bounds[l][take])))
        rep.rows[l] = rep.rows.get(l, np.zeros(rep.n, dtype=bool)) | take.any(axis=1)
    rep.refused += int(np.sum(differ & ~near))
    return np.where(take, other, own)
