from workloads.harness import DeviceLayer, HostLayer, edge_tokens, err_metric, err_unfloored, to_device  # noqa: F401

import numpy as np


def tae_margin(w):
    """TAE (Eq. 1) and top-two margin of gate weights, numpy fp64 - used only to place thresholds."""
    p = w / w.sum(1, keepdims=True)
    K = p.shape[1]
    tae = -(np.where(p > 0, p * np.log(np.where(p > 0, p, 1.0)), 0.0)).sum(1) / np.log(K)
    top = -np.sort(-p, axis=1)
    return tae, top[:, 0] - top[:, 1]


def safe_threshold(values, q):
    """A threshold near the q-quantile of `values` in the middle of the widest nearby gap, so that the
    fp32 device value and the fp64 oracle value of every token fall on the same side of it."""
    v = np.unique(values)
    if len(v) < 2:
        return float(v[0]) + 0.25
    i = int(q * (len(v) - 1))
    lo, hi = max(0, i - 8), min(len(v) - 1, i + 8)
    j = lo + int(np.argmax(np.diff(v[lo:hi + 1])))
    assert v[j + 1] - v[j] > 2e-5, "no safe gap"
    return float(0.5 * (v[j] + v[j + 1]))


def beta_pair(delta):
    """(largest fp32 value <= delta, smallest fp32 value > delta): the distribution gate is closed at the
    first and open at the second, one fp32 step apart."""
    b = np.float32(delta)
    if float(b) > delta:
        b = np.nextafter(b, np.float32(-1))
    return float(b), float(np.nextafter(b, np.float32(2)))
