"""A synthetic smoothing vector for the tests (input preparation; the method's path takes it as an input)."""
import numpy as np


def smoothing_vector(X: np.ndarray, W: np.ndarray, alpha: float = 0.5, beta: float = 0.5) -> np.ndarray:
    """A per-channel smoothing vector for a layer's inputs, of the shape the paper's App. A.1 describes
    (channel maximum of the activations to the power alpha over channel maximum of the weights to the
    power beta), computed on the synthetic tensors themselves.  It is an INPUT of the path (the paper
    calibrates it offline); channels that are all zero get 1."""
    ax = np.abs(X).max(axis=0).astype(np.float64)
    aw = np.abs(W).max(axis=0).astype(np.float64)
    g = np.where((ax > 0) & (aw > 0), ax ** alpha / np.maximum(aw, 1e-30) ** beta, 1.0)
    return g.astype(np.float32)
