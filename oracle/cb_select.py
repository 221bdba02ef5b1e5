"""Threshold selection (Sec. III-F) on the CPU oracle.  TEST INFRASTRUCTURE ONLY.

A network is a chain of change-based convolution layers (oracle/cb_oracle.c), each optionally
followed by the change-based 2x2 max-pooling of Sec. III-E.  The quality metric is the one the
paper names for sequences without annotated frames: the change-based model's output for the last
frame of every sequence compared with the original model's output (a threshold of zero reproduces
the original model, Sec. III-F first paragraph), here as the mean squared difference in float64.

The procedure follows the paper's description step by step: all thresholds start at zero; the
layers are visited from first to last; for the layer being visited the threshold starts at an
initial value and is multiplied by a fixed factor until the quality loss this layer introduces --
relative to the same network with this layer's threshold at zero -- exceeds the acceptable limit;
the value before that is kept.  Thresholds are float32 (what the layers take); the sequence
tau0, tau0*f, tau0*f*f, ... is formed by float32 multiplications.

Nothing in the product package imports this module.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import cb_oracle as orc


class OracleNetwork:
    """Chain of OracleLayer objects with optional pooling after each; every layer detects its own
    changes against its own input state (closed loop, Sec. III-C)."""

    def __init__(self, specs, H: int, W: int, bf16: bool = False):
        self.layers, self.pool_after, self.pools = [], [], []
        h, w = H, W
        for sp in specs:
            L = orc.OracleLayer(sp.weight, sp.bias, sp.stride, sp.pad, h, w, sp.relu, bf16=bf16)
            self.layers.append(L)
            h, w = L.Ho, L.Wo
            self.pool_after.append(bool(sp.pool))
            if sp.pool:
                h, w = -(-h // 2), -(-w // 2)
                self.pools.append(np.zeros((L.O, h, w), np.float32))
            else:
                self.pools.append(None)

    def reset(self):
        for L in self.layers:
            L.reset()

    def forward(self, x: np.ndarray, taus: Sequence[float]) -> np.ndarray:
        for l, L in enumerate(self.layers):
            L.process(x, float(taus[l]))
            x = L.out
            if self.pool_after[l]:
                orc.pool_update(x, L.idx, L.mt, self.pools[l])
                x = self.pools[l].copy()
        return x


def reference_outputs(net: OracleNetwork, sequences) -> List[np.ndarray]:
    """Output of the original model for the last frame of every sequence (all thresholds zero)."""
    zeros = [0.0] * len(net.layers)
    refs = []
    for seq in sequences:
        net.reset()
        out = None
        for f in seq:
            out = net.forward(f, zeros)
        refs.append(out.copy())
    return refs


def quality(net: OracleNetwork, sequences, refs, taus) -> float:
    """Mean squared difference between the change-based model's last-frame outputs and refs."""
    total, count = 0.0, 0
    for seq, ref in zip(sequences, refs):
        net.reset()
        out = None
        for f in seq:
            out = net.forward(f, taus)
        d = out.astype(np.float64) - ref.astype(np.float64)
        total += float(np.sum(d * d))
        count += d.size
    return total / count


def select_thresholds(net: OracleNetwork, sequences, tau0: float, factor: float, max_loss: Sequence[float],
                      max_steps: int = 200):
    """Returns (thresholds, per-layer log).  log[l] = list of (tau, loss) tried for layer l, where
    loss = quality(with tau at layer l) - quality(with 0 at layer l)."""
    n = len(net.layers)
    refs = reference_outputs(net, sequences)
    taus = [np.float32(0.0)] * n
    log = []
    for l in range(n):
        base = quality(net, sequences, refs, taus)
        tau, kept, tried = np.float32(tau0), np.float32(0.0), []
        for _ in range(max_steps):
            trial = list(taus)
            trial[l] = tau
            loss = quality(net, sequences, refs, trial) - base
            tried.append((float(tau), loss))
            if loss > max_loss[l]:
                break
            kept = tau
            tau = np.float32(tau * np.float32(factor))
        taus[l] = kept
        log.append(tried)
    return [float(t) for t in taus], log
