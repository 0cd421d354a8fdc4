"""The parity bars of the GPU tests, in one place.

Floating-point outputs are compared with the fp64 oracle by relative Frobenius error:
1e-5 on the fp32 matrix-core path (ranks 8/16/32), 2e-2 on the bf16 path (ranks 64/128/256).
These bars apply to what a kernel outputs: states, decompressed gradients, statistics, weights.

A weight update is also judged on dW = W - W0, which no kernel outputs: the kernel stores W in
fp32, and that last rounding (at most 2^-24 |W| per entry, whatever the arithmetic before it)
is part of the difference.  Relative to dW it can be as large as 2^-24 ||W|| / ||dW||, which for
a learning rate of 1e-3 exceeds 1e-5 by itself.  The bar on dW is therefore the path's bar plus
exactly that term, computed from the oracle's own values; W itself is held to 1e-6 (fp32 path).
"""
import numpy as np

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def tol_for(r):
    return TOL_F32 if r <= 32 else TOL_BF16


def update_bar(r, W_ref, W0):
    """Bar on ||dW_gpu - dW_ref|| / ||dW_ref|| for fp32 weights: the path's bar plus the rounding
    of the stored weights relative to the size of the update."""
    dW = np.linalg.norm(np.asarray(W_ref) - np.asarray(W0))
    return tol_for(r) + 2.0 ** -24 * float(np.linalg.norm(W_ref)) / float(dW if dW > 0 else 1.0)
