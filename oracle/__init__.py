"""CPU oracle for segment-wise training with synthetic intermediate labels.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
HIP path is checked against.  It is imported by the test-suite, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else: the product
path never routes through it and shares no code, tables or constants with it.

Contents
--------
rng.py      counter-based generator (Philox4x32-10) and the transforms that turn
            its words into synthetic intermediate labels (paper Eq. 1), input
            noise for interior segments and initial weights.
segment.py  one training step of one network segment (forward, loss, backward
            confined to the segment, SGD with momentum) in float64, with an
            optional emulation of bf16 storage points.

Everything is numpy; matrix products use ``@`` in float64 and nothing is
blocked, fused or reordered beyond the textbook definition.
"""
