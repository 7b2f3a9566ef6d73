"""slp: segment-wise training with synthetic intermediate labels on one MI355X.

Thin Python binding over the C-ABI library ``libslp.so`` (include/slp.h).  The
binding marshals arguments only -- every step of the training path runs in the
library's HIP kernels.  PyTorch provides device memory and streams.

    from paper_2403_11204_amd import api
    table = api.make_synthetic_labels(seed, classes, dim, api.UNIFORM01, kappa=10.0)
    seg = api.Segment([784, 80, 60], api.RELU_ALL, api.MSE_SIL, max_batch=1410)
    seg.init(seed); seg.set_labels(table)
    loss = seg.step(X, y)

The library is loaded on first use; there is no CPU fallback: if it has not been
built (``python -m paper_2403_11204_amd.build``) the first call raises.
"""

__all__ = ["api", "datagen", "build"]
