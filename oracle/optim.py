"""Adam step and replica weight synchronisation (oracle; test infrastructure).

The paper trains its language models with Adam at an initial learning rate of
6e-3 (Section 7, experiment setup) and says that node n keeps, besides a replica
of node n+1's layers, their optimizer state, and that FRC/BRC use the same
parameters as node n+1 (Section 5.1); it gives no update formula and no
mechanism for keeping the replica equal.  This file writes out the textbook
update of the Adam paper (Kingma & Ba, Algorithm 1) in float64, and the
simplest synchronisation that satisfies Section 5.1: after every update the
replica's parameters are overwritten with the successor's.

Readings (the paper is silent): beta1 = 0.9, beta2 = 0.999, eps = 1e-8, no weight
decay, no gradient clipping, gradients used as accumulated over the
micro-batches of the iteration (any averaging is part of the upstream gradients).
"""
import numpy as np


def adam_step(w, g, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One update of a parameter array.  step counts from 1.  Returns (w, m, v).

    m <- beta1 m + (1 - beta1) g          first-moment estimate
    v <- beta2 v + (1 - beta2) g^2        second-moment estimate
    w <- w - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
    """
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    w = w - lr * m_hat / (np.sqrt(v_hat) + eps)
    return w, m, v


class AdamState:
    """Per-layer, per-tensor moments for a stack of layers (dicts of arrays)."""

    def __init__(self, layers):
        self.m = [{n: np.zeros_like(p[n], dtype=np.float64) for n in p} for p in layers]
        self.v = [{n: np.zeros_like(p[n], dtype=np.float64) for n in p} for p in layers]
        self.step = 0

    def apply(self, layers, grads, lr, beta1=0.9, beta2=0.999, eps=1e-8):
        """Updates `layers` (list of dicts) in place from `grads` (same structure)."""
        self.step += 1
        for p, g, m, v in zip(layers, grads, self.m, self.v):
            for n in p:
                p[n], m[n], v[n] = adam_step(p[n], g[n], m[n], v[n], self.step, lr, beta1, beta2, eps)


def sync_replica(shadow_layers, successor_layers):
    """Replica weight synchronisation: the replica takes the successor's values."""
    for dst, src in zip(shadow_layers, successor_layers):
        for n in src:
            dst[n] = src[n].copy()
