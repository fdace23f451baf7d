"""Definitional nested loops in pure Python -- TEST INFRASTRUCTURE, tiny inputs only.

Every sum is spelled out index by index with Python floats (IEEE double), so
the strided C routines and the library-op forward can be checked against
something that has no strides, no slicing helpers and no vector code.
"""
import numpy as np


def conv2d(x, w, stride, pad):
    """x [N][H][W][C], w [K][R][S][C] (already the active slice) -> [N][Ho][Wo][K]."""
    n_, h_, w_, c_ = x.shape
    k_, r_, s_, _ = w.shape
    ho = (h_ + 2 * pad - r_) // stride + 1
    wo = (w_ + 2 * pad - s_) // stride + 1
    y = np.zeros((n_, ho, wo, k_))
    for n in range(n_):
        for p in range(ho):
            for q in range(wo):
                for k in range(k_):
                    acc = 0.0
                    for r in range(r_):
                        for s in range(s_):
                            ih, iw = p * stride + r - pad, q * stride + s - pad
                            if 0 <= ih < h_ and 0 <= iw < w_:
                                for c in range(c_):
                                    acc += float(x[n, ih, iw, c]) * float(w[k, r, s, c])
                    y[n, p, q, k] = acc
    return y


def depthwise(x, w, stride, pad):
    """x [N][H][W][C], w [R][S][C] -> [N][Ho][Wo][C]."""
    n_, h_, w_, c_ = x.shape
    r_, s_, _ = w.shape
    ho = (h_ + 2 * pad - r_) // stride + 1
    wo = (w_ + 2 * pad - s_) // stride + 1
    y = np.zeros((n_, ho, wo, c_))
    for n in range(n_):
        for p in range(ho):
            for q in range(wo):
                for c in range(c_):
                    acc = 0.0
                    for r in range(r_):
                        for s in range(s_):
                            ih, iw = p * stride + r - pad, q * stride + s - pad
                            if 0 <= ih < h_ and 0 <= iw < w_:
                                acc += float(x[n, ih, iw, c]) * float(w[r, s, c])
                    y[n, p, q, c] = acc
    return y


def linear(x, w, b=None):
    m_, c_ = x.shape
    k_ = w.shape[0]
    y = np.zeros((m_, k_))
    for m in range(m_):
        for k in range(k_):
            acc = 0.0
            for c in range(c_):
                acc += float(x[m, c]) * float(w[k, c])
            y[m, k] = acc + (float(b[k]) if b is not None else 0.0)
    return y


def maxpool_3x3_s2(x):
    n_, h_, w_, c_ = x.shape
    ho, wo = (h_ + 2 - 3) // 2 + 1, (w_ + 2 - 3) // 2 + 1
    y = np.zeros((n_, ho, wo, c_))
    for n in range(n_):
        for p in range(ho):
            for q in range(wo):
                for c in range(c_):
                    best = None
                    for r in range(3):
                        for s in range(3):
                            ih, iw = 2 * p + r - 1, 2 * q + s - 1
                            if 0 <= ih < h_ and 0 <= iw < w_:
                                v = float(x[n, ih, iw, c])
                                best = v if best is None or v > best else best
                    y[n, p, q, c] = best
    return y
