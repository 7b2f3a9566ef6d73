"""The paper's training procedure on top of the segment step (orchestration only).

Every arithmetic step below is a call into the C-ABI library; this module only
walks the dataset in order and moves batches between segments, as the flowcharts
of paper Sec. 2 describe:

  phase 1   the left partition is trained for N_L epochs on (inputs, synthetic
            intermediate label of the sample's class), without shuffling;
  store     one forward pass of the trained left partition over the dataset gives
            the stored response (read here as a separate pass after the last
            update, so that it is deterministic);
  phase 2   the right partition is trained for N_R epochs on (stored response, class);
  recovery  (Sec. 5) the left partition is trained further through the frozen right
            partition;
  join      the partitions are chained for inference;
  simultaneous  every partition trained at once, interior partitions on (synthetic
            label of the previous cut + noise, own target).

With more than two partitions, partition k is trained on the stored response of
partition k-1 against its own label table (Sec. 2, the multi-partition variant).
"""

import torch

from . import api


def _epoch_means(losses):
    """losses[epochs][batches] (float32, device) -> list of per-epoch means, each reduced by the library."""
    means = torch.empty(losses.shape[0], dtype=torch.float32, device=losses.device)
    for ep in range(losses.shape[0]):
        api.mean_loss(losses[ep], out=means[ep:ep + 1])
    return means.tolist()


def _batches(n, batch):
    for s in range(0, n, batch):
        yield s, min(s + batch, n)


def train_epochs(seg, X, y, epochs, batch, staged=False):
    """Consecutive, unshuffled batches for `epochs` passes.  Returns the mean loss of each epoch.

    staged: copy every batch into one fixed pair of buffers and step on those, so that a handle with graph
    replay on (Segment.set_graph) sees a single argument combination per batch size and replays one graph."""
    n = X.shape[0]
    losses = torch.zeros((epochs, (n + batch - 1) // batch), dtype=torch.float32, device=X.device)
    if staged:
        Xs = torch.empty((batch, X.shape[1]), dtype=X.dtype, device=X.device)
        ys = torch.empty(batch, dtype=y.dtype, device=y.device)
    for ep in range(epochs):
        for i, (a, b) in enumerate(_batches(n, batch)):
            if staged:
                Xs[:b - a].copy_(X[a:b])
                ys[:b - a].copy_(y[a:b])
                seg.step(Xs[:b - a], ys[:b - a], loss_out=losses[ep, i:i + 1])
            else:
                seg.step(X[a:b], y[a:b], loss_out=losses[ep, i:i + 1])
    return _epoch_means(losses)


def store_response(seg, X, batch):
    """Forward-only pass over the dataset: the response that feeds the next partition."""
    out = torch.empty((X.shape[0], seg.widths[-1]), dtype=X.dtype, device=X.device)
    for a, b in _batches(X.shape[0], batch):
        seg.forward(X[a:b], out=out[a:b])
    return out


def train_partitioned(segments, X, y, epochs, batch):
    """Sequential variant: segments[k] is trained for epochs[k] on the stored response of segments[k-1].
    Label tables must already be bound.  Returns (per-segment epoch losses, the stored responses)."""
    losses, stored, cur = [], [], X
    for k, seg in enumerate(segments):
        losses.append(train_epochs(seg, cur, y, epochs[k], batch))
        if k + 1 < len(segments):
            cur = store_response(seg, cur, batch)
            stored.append(cur)
    return losses, stored


def recovery_epochs(left, right, X, y, epochs, batch):
    """Sec. 5: forward through left, loss and input gradient from the frozen right partition, update of left.
    `right` must have been created with input_grad=True.  Returns the mean loss of each epoch."""
    n = X.shape[0]
    losses = torch.zeros((epochs, (n + batch - 1) // batch), dtype=torch.float32, device=X.device)
    for ep in range(epochs):
        for i, (a, b) in enumerate(_batches(n, batch)):
            resp = left.forward(X[a:b])
            d_resp, _ = right.input_grad(resp, y[a:b], loss_out=losses[ep, i:i + 1])
            left.step_external(X[a:b], d_resp)
    return _epoch_means(losses)


def train_simultaneous(segments, tables, X, y, epochs, batch, noise_seed=5, sigma=0.05):
    """The variant that trains every partition at once (end of Sec. 2): partition 0 sees the data, partition k > 0
    sees the synthetic label of the sample's class at cut k-1 plus noise (standard deviation sigma, counter = global
    sample index, seed noise_seed + k) instead of the response of partition k-1, so no partition waits for another.
    tables[k] is the float32 label table of cut k (already bound to segments[k] as its target).  Each partition
    steps on a stream of its own.  Returns the mean loss of each epoch, per partition."""
    n = X.shape[0]
    nb = (n + batch - 1) // batch
    losses = [torch.zeros((epochs, nb), dtype=torch.float32, device=X.device) for _ in segments]
    streams = [torch.cuda.Stream() for _ in segments]
    cur = torch.cuda.current_stream()
    for st in streams:
        st.wait_stream(cur)
    for ep in range(epochs):
        for i, (a, b) in enumerate(_batches(n, batch)):
            for k, (seg, st) in enumerate(zip(segments, streams)):
                with torch.cuda.stream(st):
                    xin = X[a:b] if k == 0 else api.make_segment_inputs(noise_seed + k, tables[k - 1], y[a:b], a, sigma, seg.dtype)
                    seg.step(xin, y[a:b], loss_out=losses[k][ep, i:i + 1])
                    xin.record_stream(st)
    for st in streams:
        cur.wait_stream(st)
    return [_epoch_means(l) for l in losses]


def joined_forward(segments, X, batch):
    """The joined network: logits of the last partition."""
    cur = X
    for seg in segments:
        cur = store_response(seg, cur, batch)
    return cur


def accuracy(segments, X, y, batch):
    """Fraction of samples whose arg-max logit of the joined network is their class: the batches go through the chain
    of forward passes one at a time and the library counts the hits of each into one device counter."""
    hits = torch.zeros(1, dtype=torch.int64, device=X.device)
    for a, b in _batches(X.shape[0], batch):
        cur = X[a:b]
        for seg in segments:
            cur = seg.forward(cur)
        api.count_correct(cur, y[a:b], out=hits, accumulate=True)
    return int(hits.item()) / X.shape[0]
