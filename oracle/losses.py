"""Per-sample softmax cross-entropy, the loss value the sampler ranks samples by.

The paper ranks samples by "loss value" (Section 4.2) and stores one float per sample
(Section 4.3, limitations); its experiments are classification, so the loss is the
softmax cross-entropy with natural logarithm.
"""
import numpy as np


def softmax_cross_entropy(logits, y):
    """logits float64 [B, C], y int [B] -> (loss [B], dloss_dlogits [B, C]).

    loss_b = log(sum_c exp(z_bc)) - z_b,y_b, evaluated with the maximum subtracted so that
    large logits stay finite.  The second result is the derivative of loss_b (not of the
    batch mean) with respect to z_b: softmax(z_b) - onehot(y_b).
    """
    z = np.asarray(logits, dtype=np.float64)
    y = np.asarray(y).astype(np.int64)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=1, keepdims=True)
    rows = np.arange(z.shape[0])
    loss = (m[:, 0] + np.log(s[:, 0])) - z[rows, y]
    p = e / s
    p[rows, y] -= 1.0
    return loss, p
