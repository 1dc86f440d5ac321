"""Mini-batch SGD update used for the local steps (Section 2, local SGD update rule).

The paper trains with PyTorch's SGD optimiser (Appendix A.1); momentum, L2 weight decay
(coupled: added to the gradient), no dampening and no Nesterov follow that optimiser's
documented update rule:  g <- g + wd*x;  buf <- mu*buf + g;  x <- x - lr*buf.
A zero buffer before the first step makes the first buffer equal the gradient.
"""
import numpy as np


def sgd_update(x, buf, grad, lr, momentum=0.0, weight_decay=0.0):
    """Returns (x_new, buf_new); all float64 arrays of one shape."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64) + weight_decay * x
    buf_new = momentum * np.asarray(buf, dtype=np.float64) + g
    return x - lr * buf_new, buf_new
