"""CPU oracle for the layers between sparse convolutions (Sec. III, Fig. "hpc" caption: batch
normalisation, activation and pooling layers sit between the SparseConv blocks; Sec. IV-A: a
40-category classifier trained with a cross-entropy objective).

TEST INFRASTRUCTURE ONLY, like the rest of `oracle/`: plain numpy in float64, each function is the
textbook definition written out.  Pinned against torch's library routines (and autograd for the
backward passes) in tests/test_oracle_pins.py.

The paper gives no formulas for these layers; the definitions are the standard ones:
  - batch normalisation in training mode over all N rows of the sparse tensor, per channel, biased
    variance, followed (optionally) by ReLU;
  - global average pooling per cloud (rows grouped by the batch index, column 0 of C);
  - a linear layer and the mean softmax cross-entropy over the clouds of the batch.
"""
from __future__ import annotations

import numpy as np


def bn_relu_fwd(x, gamma, beta, eps: float, relu: bool):
    """y = gamma * (x - mean) / sqrt(var + eps) + beta per channel (mean/var over rows, biased), then max(y, 0).

    Returns (y, mean, rstd) with rstd = 1/sqrt(var + eps).
    """
    x = np.asarray(x, np.float64)
    mean = x.mean(axis=0)
    var = ((x - mean) ** 2).mean(axis=0)
    rstd = 1.0 / np.sqrt(var + eps)
    y = (x - mean) * rstd * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    return y, mean, rstd


def bn_relu_bwd(x, y, dy, gamma, mean, rstd, relu: bool):
    """Gradients of bn_relu_fwd.  With relu, dy is first masked where the forward output y was not positive.

    xhat = (x - mean) * rstd;  dbeta = sum dy;  dgamma = sum dy * xhat;
    dx = gamma * rstd / N * (N * dy - dbeta - xhat * dgamma).
    Returns (dx, dgamma, dbeta).
    """
    x = np.asarray(x, np.float64)
    dy = np.asarray(dy, np.float64)
    gamma = np.asarray(gamma, np.float64)
    n = x.shape[0]
    xhat = (x - mean) * rstd
    if relu:
        dy = dy * (np.asarray(y, np.float64) > 0)
    dbeta = dy.sum(axis=0)
    dgamma = (dy * xhat).sum(axis=0)
    dx = gamma * rstd / n * (n * dy - dbeta - xhat * dgamma)
    return dx, dgamma, dbeta


def pool_avg_fwd(batch_index, x, n_clouds: int):
    """out[b] = mean of the rows whose batch index is b (zero for an empty cloud).  Returns (out, counts)."""
    x = np.asarray(x, np.float64)
    b = np.asarray(batch_index, np.int64)
    out = np.zeros((n_clouds, x.shape[1]))
    np.add.at(out, b, x)
    counts = np.bincount(b, minlength=n_clouds).astype(np.float64)
    out /= np.maximum(counts, 1.0)[:, None]
    return out, counts


def pool_avg_bwd(batch_index, dout, counts):
    """dx[r] = dout[b(r)] / count[b(r)]."""
    b = np.asarray(batch_index, np.int64)
    return np.asarray(dout, np.float64)[b] / np.maximum(np.asarray(counts, np.float64), 1.0)[b][:, None]


def linear_fwd(x, w, bias):
    """out = x @ w^T + bias;  w is [m][c]."""
    return np.asarray(x, np.float64) @ np.asarray(w, np.float64).T + np.asarray(bias, np.float64)


def linear_bwd(x, w, dout):
    """Returns (dx, dw, dbias)."""
    x, w, dout = (np.asarray(a, np.float64) for a in (x, w, dout))
    return dout @ w, dout.T @ x, dout.sum(axis=0)


def softmax_ce(logits, labels):
    """Mean over the clouds of -log softmax(logits)[label].  Returns (loss, dlogits)."""
    z = np.asarray(logits, np.float64)
    lab = np.asarray(labels, np.int64)
    z = z - z.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    n = z.shape[0]
    loss = -logp[np.arange(n), lab].mean()
    d = np.exp(logp)
    d[np.arange(n), lab] -= 1.0
    return loss, d / n
