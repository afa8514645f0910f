"""TEST INFRASTRUCTURE -- oracle for the loss at the last layer (fp64, numpy).

The paper leaves the loss open ("prediction errors", Sec. 1.1); the benchmark
fixes softmax cross-entropy.  The pixel-of-interest mask of Sec. 4.3 keeps the
errors of chosen pixels and zeroes the others; the mini-batch of the chosen
patches is averaged (Sec. 1.1: gradients of the K patches are averaged).

    p      = softmax over classes of scores[n, :, i, j]
    loss   = -(1/|M|) * sum_{(n,i,j) in M} log p[label[n,i,j]]
    delta  = mask * (p - onehot(label)) / |M|          (d loss / d scores)

|M| = number of non-zero mask entries over the whole batch; |M| = 0 gives
loss 0 and delta 0.
"""
import numpy as np


def masked_softmax_xent(scores, labels, mask):
    """scores [N, Cls, H, W]; labels int [N, H, W]; mask [N, H, W] (non-zero = chosen).
    Returns (loss: float, delta: float64 [N, Cls, H, W], count: int)."""
    s = np.asarray(scores, np.float64)
    N, Cls, H, W = s.shape
    lab = np.asarray(labels).astype(np.int64)
    m = np.asarray(mask) != 0
    count = int(m.sum())
    delta = np.zeros_like(s)
    if count == 0:
        return 0.0, delta, 0
    z = s - s.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    onehot = np.zeros_like(s)
    np.put_along_axis(onehot, lab[:, None, :, :], 1.0, axis=1)
    logp_label = np.take_along_axis(z, lab[:, None, :, :], axis=1)[:, 0] - np.log(e.sum(axis=1))
    loss = -float(logp_label[m].sum()) / count
    delta = (p - onehot) * m[:, None, :, :] / count
    return loss, delta, count
