"""BN folding on the oracle side.  Test infrastructure only.

A batch-norm y = gamma * (z - mean) / sqrt(var + eps) + beta that follows a
bias-free convolution z = conv(x, W) equals a convolution with
W'[k] = W[k] * gamma[k] / sqrt(var[k] + eps) and bias
b'[k] = beta[k] - mean[k] * gamma[k] / sqrt(var[k] + eps).
Folding is done in float32, one operation at a time, before the cast to the
storage type.
"""
import numpy as np


def fold_bn(w, bn):
    f32 = np.float32
    scale = (bn["gamma"].astype(f32) / np.sqrt(bn["var"].astype(f32) + f32(bn["eps"]))).astype(f32)
    wf = (w.astype(f32) * scale.reshape((-1,) + (1,) * (w.ndim - 1))).astype(f32)
    bf = (bn["beta"].astype(f32) - (bn["mean"].astype(f32) * scale).astype(f32)).astype(f32)
    return wf, bf


def batchnorm(z, bn):
    """Inference batch-norm over the last (channel) axis, in float64."""
    z = z.astype(np.float64)
    return (bn["gamma"].astype(np.float64) * (z - bn["mean"].astype(np.float64))
            / np.sqrt(bn["var"].astype(np.float64) + bn["eps"]) + bn["beta"].astype(np.float64))
