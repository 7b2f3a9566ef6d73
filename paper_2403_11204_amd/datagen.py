"""Seeded synthetic inputs shaped like the paper's workload.

The paper trains on EMNIST-balanced: 112,800 flattened 28x28 grey-scale images
with values in [0,1] and 47 balanced classes (Sec. 3).  That dataset is not
available here; these generators stand in for it with the same shapes, value
range and class balance.  They hold none of the method's arithmetic (no label
generator, no layer, no loss) and serve both the HIP path and the CPU oracle,
so that both see byte-identical inputs.
"""

import numpy as np


def balanced_classes(n, classes, first=0):
    """Class ids in dataset order: sample n has class n mod classes."""
    return ((first + np.arange(n, dtype=np.int64)) % classes).astype(np.int32)


def blob_images(n, classes=47, side=28, seed=1, noise=0.05):
    """Tiny-config data: each class is a Gaussian blob on a side x side canvas
    with its own centre and width; pixel noise is added and the result clipped
    to [0,1].  Returns (X float32 [n, side*side], y int32 [n])."""
    rng = np.random.Generator(np.random.Philox(seed))
    cx = rng.uniform(4.0, side - 4.0, size=classes)
    cy = rng.uniform(4.0, side - 4.0, size=classes)
    sg = rng.uniform(2.0, 5.0, size=classes)
    y = balanced_classes(n, classes)
    r = np.arange(side, dtype=np.float64)[:, None]
    q = np.arange(side, dtype=np.float64)[None, :]
    proto = np.empty((classes, side * side))
    for c in range(classes):
        proto[c] = np.exp(-((r - cy[c]) ** 2 + (q - cx[c]) ** 2) / (2.0 * sg[c] ** 2)).ravel()
    X = proto[y] + noise * rng.standard_normal((n, side * side))
    return np.clip(X, 0.0, 1.0).astype(np.float32), y


def class_mean_inputs(n, classes, dim=784, seed=1, spread=0.25, first=0):
    """Paper-shaped data: x = clip(mean[class] + spread * N(0,1), 0, 1) with a
    class-mean table drawn U[0,1).  ``first`` selects a window of the (virtual)
    dataset so that batches can be generated without materialising all of it;
    the class-mean table depends on the seed only.
    Returns (X float32 [n, dim], y int32 [n])."""
    means = np.random.Generator(np.random.Philox(seed)).uniform(0.0, 1.0, size=(classes, dim))
    y = balanced_classes(n, classes, first)
    rng = np.random.Generator(np.random.Philox(key=seed + 1, counter=[first, 0, 0, 0]))
    X = means[y] + spread * rng.standard_normal((n, dim))
    return np.clip(X, 0.0, 1.0).astype(np.float32), y


def uniform_weights(widths, seed):
    """Host-side initial parameters U(-1/sqrt(fan_in), 1/sqrt(fan_in)) for tests
    that want to hand the same arbitrary starting point to both sides.
    Returns a list of (W float32 [out, in], b float32 [out])."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for l in range(len(widths) - 1):
        bound = 1.0 / np.sqrt(widths[l])
        W = rng.uniform(-bound, bound, size=(widths[l + 1], widths[l])).astype(np.float32)
        b = rng.uniform(-bound, bound, size=widths[l + 1]).astype(np.float32)
        out.append((W, b))
    return out
