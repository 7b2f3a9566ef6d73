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
parameter and multiply-accumulate counts printed in paper Sec. 3).
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

    # -- one training step ---------------------------------------------------------
    def step(self, X, y, table=None, update=True, full_batch=None, tie_decisions=None, tie_band=1e-3):
        """Forward, loss, backward, SGD.  Returns a dict with everything a
        parity test wants to look at (values *before* the update for A, Z, dZ,
        dW, db; parameters are updated in place).  With ``full_batch`` the rows
        are a sample of a larger batch: A, Z and dZ of those rows are exact (they
        depend on the rest of the batch only through its size); loss is then these
        rows' share, dW and db are not formed and no update may be asked for.

        ``tie_decisions``: whether a ReLU unit passes gradient is an integer decided
        from a floating-point pre-activation; where that value is zero to within
        rounding, "active" and "inactive" are both correct, and two correct
        implementations may differ.  tie_decisions[l] (l = 1..L, boolean, shape of
        A[l]) holds another implementation's decisions; they are taken over ONLY
        where this oracle's own pre-activation is within tie_band * max|Z_l| of
        zero.  The result reports how many decisions were taken over ("ties_taken")
        and how many disagreements lie outside the band ("decisions_refused": those
        are the other side's errors, and the oracle keeps its own decision there)."""
        assert full_batch is None or not update
        Wp = self._weights_for_products()
        A, Z = self.forward_all(X)
        loss, G = self.loss_and_grad(A[self.L], y, table, full_batch)
        ties_taken, refused = 0, 0

        def active(l):
            nonlocal ties_taken, refused
            own = A[l] > 0.0
            if tie_decisions is None or tie_decisions[l] is None:
                return own
            other = np.asarray(tie_decisions[l], dtype=bool)
            differ = own != other
            near = np.abs(Z[l]) <= tie_band * np.max(np.abs(Z[l]))
            ties_taken += int(np.sum(differ & near))
            refused += int(np.sum(differ & ~near))
            return np.where(near, other, own)

        dZ = [None] * (self.L + 1)
        dW = [None] * self.L
        db = [None] * self.L
        g = G * active(self.L) if self._relu_on(self.L) else G
        dZ[self.L] = self._store(g)
        for l in range(self.L, 0, -1):
            if full_batch is None:       # parameter gradients need every row of the batch
                dW[l - 1] = dZ[l].T @ A[l - 1]
                db[l - 1] = dZ[l].sum(axis=0)
            if l > 1:
                dA = dZ[l] @ Wp[l - 1]
                dZ[l - 1] = self._store(dA * active(l - 1))
        if update:
            for l in range(self.L):
                self.vW[l] = self.mu * self.vW[l] + dW[l]
                self.vb[l] = self.mu * self.vb[l] + db[l]
                self.W[l] = self.W[l] - self.lr * self.vW[l]
                self.b[l] = self.b[l] - self.lr * self.vb[l]
                if self.mode == "bf16":     # master parameters live in float32
                    self.W[l] = self.W[l].astype(np.float32).astype(np.float64)
                    self.b[l] = self.b[l].astype(np.float32).astype(np.float64)
        return {"loss": loss, "A": A, "Z": Z, "dZ": dZ, "dW": dW, "db": db, "ties_taken": ties_taken,
                "decisions_refused": refused}


# -- recovery phase (paper Sec. 5) ---------------------------------------------------
# After both partitions are trained, the left one is trained some more *through* the
# right one, whose weights stay frozen: the loss is the right partition's
# classification loss on the left partition's response.  That needs two more
# operations, added to the class below: the gradient of a segment's loss with
# respect to its INPUT (no parameter gradient, no update), and a training step that
# starts from a gradient handed in from outside instead of from the segment's own loss.
def _input_gradient(self, X, y, table=None):
    """Forward, loss, and backpropagation through every layer down to the input.
    Parameters are not touched.  Returns {"loss", "dX", "A", "Z", "dZ"}; dX is
    d loss / d X (rounded to bf16 in bf16 mode, like every stored gradient)."""
    Wp = self._weights_for_products()
    A, Z = self.forward_all(X)
    loss, G = self.loss_and_grad(A[self.L], y, table)
    dZ = [None] * (self.L + 1)
    dZ[self.L] = self._store(G * (A[self.L] > 0.0) if self._relu_on(self.L) else G)
    for l in range(self.L, 1, -1):
        dZ[l - 1] = self._store((dZ[l] @ Wp[l - 1]) * (A[l - 1] > 0.0))
    dX = self._store(dZ[1] @ Wp[0])          # the input is not a ReLU output of this segment: no mask
    return {"loss": loss, "dX": dX, "A": A, "Z": Z, "dZ": dZ}


def _step_external(self, X, dA_out, update=True):
    """A training step driven by dA_out = d loss / d (segment output), supplied by
    whatever sits behind the segment.  dZ_L = dA_out * [A_L > 0] when the last
    layer has a ReLU, else dA_out; then the usual backward pass and SGD update."""
    Wp = self._weights_for_products()
    A, Z = self.forward_all(X)
    g = self._store(np.asarray(dA_out, dtype=np.float64))
    dZ = [None] * (self.L + 1)
    dZ[self.L] = self._store(g * (A[self.L] > 0.0)) if self._relu_on(self.L) else g
    dW, db = [None] * self.L, [None] * self.L
    for l in range(self.L, 0, -1):
        dW[l - 1] = dZ[l].T @ A[l - 1]
        db[l - 1] = dZ[l].sum(axis=0)
        if l > 1:
            dZ[l - 1] = self._store((dZ[l] @ Wp[l - 1]) * (A[l - 1] > 0.0))
    if update:
        for l in range(self.L):
            self.vW[l] = self.mu * self.vW[l] + dW[l]
            self.vb[l] = self.mu * self.vb[l] + db[l]
            self.W[l] = self.W[l] - self.lr * self.vW[l]
            self.b[l] = self.b[l] - self.lr * self.vb[l]
            if self.mode == "bf16":
                self.W[l] = self.W[l].astype(np.float32).astype(np.float64)
                self.b[l] = self.b[l].astype(np.float32).astype(np.float64)
    return {"A": A, "Z": Z, "dZ": dZ, "dW": dW, "db": db}


Segment.input_gradient = _input_gradient
Segment.step_external = _step_external
