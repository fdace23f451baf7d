"""CPU oracle building blocks -- TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; it shares no code with the HIP library.

Activations are float64 numpy arrays in NHWC (or [tokens][features]).  The
strided conv / depthwise / linear sums are the C routines of sna_oracle.c; the
rest are the plain definitions written with numpy in float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsna_oracle.so")
_SRC = os.path.join(_HERE, "sna_oracle.c")


def build(force: bool = False) -> str:
    """Compile sna_oracle.c with gcc (OpenMP) into libsna_oracle.so."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared",
                               "-o", _SO, _SRC])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        dp, fp = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)
        i, l = ctypes.c_int, ctypes.c_long
        _lib.ora_conv2d.argtypes = [dp, i, i, i, i, fp, l, l, l, i, i, i, i, i, i, i, dp, i, i]
        _lib.ora_depthwise.argtypes = [dp, i, i, i, i, fp, l, l, i, i, i, i, i, i, dp, i, i]
        _lib.ora_linear.argtypes = [dp, i, l, i, fp, l, i, dp]
        for f in (_lib.ora_conv2d, _lib.ora_depthwise, _lib.ora_linear):
            f.restype = None
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check_w(w):
    assert w.dtype == np.float32 and w.flags.c_contiguous, "weights: contiguous fp32 max-size tensor"


def out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


# ---------------------------------------------------------------- WeightSlice layers
def conv2d_sliced(x, w_max, c_out: int, k: int, stride: int):
    """WeightSlice convolution (WeightSlice paragraph): leading c_out output and
    x.shape[-1] input channels, centre k x k window of the stored kernel, zero
    padding k//2; w_max is the stored [K_max][R_max][S_max][C_max] tensor."""
    _check_w(w_max)
    x = _f64(x)
    n, h, wd, c = x.shape
    kmax, rmax, smax, cmax = w_max.shape
    assert c_out <= kmax and c <= cmax and k <= rmax and (rmax - k) % 2 == 0
    pad = k // 2
    ho, wo = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    y = np.empty((n, ho, wo, c_out), dtype=np.float64)
    lib().ora_conv2d(_dp(x), n, h, wd, c, _fp(w_max), rmax * smax * cmax, smax * cmax, cmax,
                     c_out, k, k, (rmax - k) // 2, (smax - k) // 2, stride, pad, _dp(y), ho, wo)
    return y


def depthwise_sliced(x, w_max, k: int, stride: int):
    """Depthwise convolution on the leading x.shape[-1] channels with the centre
    k x k window of the stored [R_max][S_max][C_max] kernel, zero padding k//2."""
    _check_w(w_max)
    x = _f64(x)
    n, h, wd, c = x.shape
    rmax, smax, cmax = w_max.shape
    assert c <= cmax and k <= rmax and (rmax - k) % 2 == 0
    pad = k // 2
    ho, wo = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    y = np.empty((n, ho, wo, c), dtype=np.float64)
    lib().ora_depthwise(_dp(x), n, h, wd, c, _fp(w_max), smax * cmax, cmax,
                        k, k, (rmax - k) // 2, (smax - k) // 2, stride, pad, _dp(y), ho, wo)
    return y


def linear_sliced(x, w_max, n_out: int, bias=None):
    """WeightSlice fully-connected layer: y = x . w_max[:n_out, :x.shape[-1]]^T (+ bias[:n_out])."""
    _check_w(w_max)
    x = _f64(x)
    lead, c = x.shape[:-1], x.shape[-1]
    x2 = x.reshape(-1, c)
    kmax, cmax = w_max.shape
    assert n_out <= kmax and c <= cmax
    y = np.empty((x2.shape[0], n_out), dtype=np.float64)
    lib().ora_linear(_dp(x2), x2.shape[0], c, c, _fp(w_max), cmax, n_out, _dp(y))
    if bias is not None:
        y = y + bias[:n_out].astype(np.float64)
    return y.reshape(*lead, n_out)


# ---------------------------------------------------------------- SubnetNorm
EPS = 1e-5


class CalibrationTable:
    """A layer's statistics table [n_subnets][4][C_max] that is being calibrated: subnet_norm fills
    the mean and variance of row i from the very batch it is about to normalise."""

    def __init__(self, table):
        self.table = table


def subnet_norm(x, stats_layer, subnet_id: int):
    """SubnetNorm (SubnetNorm paragraph): look up the statistics stored for
    (subnet i, layer j) and normalise with them.  stats_layer is the layer's
    table [n_subnets][4][C_max] = (mean, var, gamma, beta); the leading
    x.shape[-1] entries of row i are used:  gamma*(x-mean)/sqrt(var+eps)+beta.

    Calibration (the paper computes each subnet's statistics by forward passes
    over data before serving): when the table comes wrapped in CalibrationTable,
    the per-channel mean and (population) variance of x over batch and pixels
    are stored into row i first, in the table's own precision, and the
    normalisation then reads them back like any later forward would."""
    c = x.shape[-1]
    if isinstance(stats_layer, CalibrationTable):
        stats_layer = stats_layer.table
        flat = _f64(x).reshape(-1, c)
        stats_layer[subnet_id, 0, :c] = flat.mean(axis=0)
        stats_layer[subnet_id, 1, :c] = flat.var(axis=0)
    mean, var, gamma, beta = (stats_layer[subnet_id, f, :c].astype(np.float64) for f in range(4))
    return gamma * (x - mean) / np.sqrt(var + EPS) + beta


# ---------------------------------------------------------------- activations & pooling
def relu(x):
    return np.maximum(x, 0.0)


def hardsigmoid(x):
    return np.clip(x + 3.0, 0.0, 6.0) / 6.0


def hardswish(x):
    return x * np.clip(x + 3.0, 0.0, 6.0) / 6.0


def gelu(x):
    from scipy.special import erf
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


ACT = {"relu": relu, "hswish": hardswish, "none": lambda x: x}


def maxpool_3x3_s2(x):
    """3x3 max pooling, stride 2, padding 1 (padding never wins the max)."""
    n, h, w, c = x.shape
    ho, wo = out_size(h, 3, 2, 1), out_size(w, 3, 2, 1)
    xp = np.full((n, h + 2, w + 2, c), -np.inf)
    xp[:, 1:h + 1, 1:w + 1] = x
    y = np.full((n, ho, wo, c), -np.inf)
    for r in range(3):
        for s in range(3):
            y = np.maximum(y, xp[:, r:r + 2 * ho:2, s:s + 2 * wo:2])
    return y


def global_avg_pool(x):
    return x.mean(axis=(1, 2))


def layer_norm(x, gamma, beta, eps=1e-5):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma.astype(np.float64) + beta.astype(np.float64)


def softmax(x):
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


# ---------------------------------------------------------------- storage rounding
def round_f64(a):
    return np.asarray(a, dtype=np.float64)


def round_fp32(a):
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_bf16(a):
    """Round float64 values to the nearest bfloat16 (ties to even) in one step.

    bfloat16 keeps 7 explicit mantissa bits; float64 has 52, so the low 45 bits
    are rounded away.  Values must lie in bfloat16's normal range or be zero."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = a.view(np.uint64)
    lsb = (b >> np.uint64(45)) & np.uint64(1)
    r = (b + np.uint64((1 << 44) - 1) + lsb) & ~np.uint64((1 << 45) - 1)
    out = r.view(np.float64)
    mag = np.abs(out)
    ok = (mag == 0) | ((mag >= 2.0 ** -126) & (mag < 2.0 ** 128))
    tiny = np.abs(a) < 2.0 ** -126          # flush what bf16 cannot hold as a normal
    out = np.where(tiny, 0.0, out)
    assert np.all(ok | tiny), "value outside bfloat16 normal range"
    return out


ROUND = {"f64": round_f64, "fp32": round_fp32, "bf16": round_bf16}
