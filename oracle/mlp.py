"""CPU oracle of the decoder m(y; Phi) that follows the encoding (Fig. 3: the interpolated features are
"fed into an MLP"; Table 1: 64 hidden neurons).  TEST INFRASTRUCTURE ONLY.  Plain numpy, fp64.

What the paper fixes: a multi-layer perceptron with 64 neurons per hidden layer.  What it does not say and
this build ASSUMES (the hash-grid encoding it extends uses the same): two hidden layers, ReLU after each
hidden layer, a linear output layer, no biases.

    h1 = relu(W1 y)    h2 = relu(W2 h1)    out = W3 h2          W1 [64, n_in], W2 [64, 64], W3 [n_out, 64]

The backward pass is the chain rule through these three products; relu'(0) = 0.
"""
import numpy as np


def mlp_fwd(y, W1, W2, W3, want_mag=False):
    """out [N, n_out]; with want_mag also the magnitude sums the comparison tolerance refers to:
    mag = |W3| (|W2| (|W1| |y|)), the value the output would have if no term cancelled."""
    y, W1, W2, W3 = (np.asarray(a, dtype=np.float64) for a in (y, W1, W2, W3))
    a1 = y @ W1.T
    h1 = np.maximum(a1, 0.0)
    a2 = h1 @ W2.T
    h2 = np.maximum(a2, 0.0)
    out = h2 @ W3.T
    if not want_mag:
        return out
    mag = ((np.abs(y) @ np.abs(W1).T) @ np.abs(W2).T) @ np.abs(W3).T
    return out, mag, (a1, a2)


def mlp_bwd(y, W1, W2, W3, dout, masks=None):
    """Gradients of sum(out * dout) with respect to y and the three matrices, each with the sum of the
    magnitudes of the terms that form it (tolerances are relative to those).

    masks = (M1, M2), boolean [N, 64] each: use these as relu' of the two hidden layers instead of (a1 > 0),
    (a2 > 0).  relu' is a decision on the sign of a floating-point sum; where that sum is within rounding error
    of zero an implementation in lower precision may decide either way, and a test bounds what that can change by
    evaluating the magnitude sums with such units switched on and switched off (tests/test_gpu_mlp.py)."""
    y, W1, W2, W3, dout = (np.asarray(a, dtype=np.float64) for a in (y, W1, W2, W3, dout))
    a1 = y @ W1.T
    h1 = np.maximum(a1, 0.0)
    a2 = h1 @ W2.T
    h2 = np.maximum(a2, 0.0)
    M1, M2 = (a1 > 0, a2 > 0) if masks is None else masks
    dh2 = (dout @ W3) * M2
    dh1 = (dh2 @ W2) * M1
    dy = dh1 @ W1
    dW3 = dout.T @ h2
    dW2 = dh2.T @ h1
    dW1 = dh1.T @ y
    # magnitudes: the same chains with absolute values in every factor (masks kept), i.e. what each result
    # would be if no term cancelled anywhere along the way -- hidden activations included, because their
    # own rounding error is relative to that sum, not to their value
    mh1 = (np.abs(y) @ np.abs(W1).T) * M1
    mh2 = (mh1 @ np.abs(W2).T) * M2
    m2 = (np.abs(dout) @ np.abs(W3)) * M2
    m1 = (m2 @ np.abs(W2)) * M1
    mag = {"dy": m1 @ np.abs(W1), "dW3": np.abs(dout).T @ mh2, "dW2": m2.T @ mh1, "dW1": m1.T @ np.abs(y)}
    return {"dy": dy, "dW1": dW1, "dW2": dW2, "dW3": dW3}, mag, (a1, a2)
