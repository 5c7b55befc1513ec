"""ctypes front end of ops.c.  Test infrastructure only.

All tensors are float32 numpy arrays in NHWC order holding values that are
representable in the storage type named by `dtype` ("f32", "f16", "bf16").
"""
import ctypes as C
import numpy as np
from . import build as _build

_DT = {"f32": 0, "f16": 1, "bf16": 2}
_ACT = {"none": 0, "relu": 1, "relu6": 2}
_lib = None
_fp = C.POINTER(C.c_float)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.orc_round_store.restype = C.c_double
        _lib.orc_round_store.argtypes = [C.c_double, C.c_int]
        _lib.orc_conv_point.restype = C.c_double
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_fp)


def out_dim(n, pad, k, stride):
    return (n + 2 * pad - k) // stride + 1


def round_store(v, dtype):
    return lib().orc_round_store(float(v), _DT[dtype])


def round_array(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32).copy()
    lib().orc_round_array(_p(a), C.c_size_t(a.size), _DT[dtype])
    return a


def num_threads():
    return lib().orc_num_threads()


def _out(y, n, p, q, k, c_off, c_tot):
    c_tot = c_tot or k
    if y is None:
        y = np.zeros((n, p, q, c_tot), dtype=np.float32)
    assert y.shape == (n, p, q, c_tot) and c_off + k <= c_tot
    return y, c_tot


def conv(x, w, bias=None, stride=(1, 1), pad=(0, 0), act="none", res=None, dtype="f32",
         y=None, c_off=0, c_tot=0, groups=1):
    n, h, wd, c = x.shape
    k, r, s, c2 = w.shape
    if groups > 1:
        # Grouped convolution, by its definition: group g maps input channels [g*C/G, (g+1)*C/G) to output
        # channels [g*K/G, (g+1)*K/G) with its own filters; the groups do not interact.
        assert c % groups == 0 and k % groups == 0 and c2 == c // groups
        cg, kg = c // groups, k // groups
        p, q = out_dim(h, pad[0], r, stride[0]), out_dim(wd, pad[1], s, stride[1])
        y, c_tot = _out(y, n, p, q, k, c_off, c_tot)
        for g in range(groups):
            xg = np.ascontiguousarray(x[..., g * cg:(g + 1) * cg])
            wg = np.ascontiguousarray(w[g * kg:(g + 1) * kg])
            bg = None if bias is None else np.ascontiguousarray(bias[g * kg:(g + 1) * kg])
            rg = None if res is None else np.ascontiguousarray(res[..., g * kg:(g + 1) * kg])
            conv(xg, wg, bg, stride, pad, act, rg, dtype, y, c_off + g * kg, c_tot)
        return y
    assert c == c2
    p, q = out_dim(h, pad[0], r, stride[0]), out_dim(wd, pad[1], s, stride[1])
    y, c_tot = _out(y, n, p, q, k, c_off, c_tot)
    res_ct = 0
    if res is not None:
        assert res.shape[:3] == (n, p, q) and res.shape[3] >= k
        res_ct = res.shape[3]
    lib().orc_conv(_p(x), n, h, wd, c, _p(w), k, r, s, stride[0], stride[1], pad[0], pad[1],
                   _p(bias), _p(res), res_ct, _ACT[act], _DT[dtype], _p(y), c_off, c_tot)
    return y


def dwconv(x, w, bias=None, stride=(1, 1), pad=(0, 0), act="none", dtype="f32", y=None, c_off=0, c_tot=0):
    n, h, wd, c = x.shape
    c2, r, s = w.shape
    assert c == c2
    p, q = out_dim(h, pad[0], r, stride[0]), out_dim(wd, pad[1], s, stride[1])
    y, c_tot = _out(y, n, p, q, c, c_off, c_tot)
    lib().orc_dwconv(_p(x), n, h, wd, c, _p(w), r, s, stride[0], stride[1], pad[0], pad[1],
                     _p(bias), _ACT[act], _DT[dtype], _p(y), c_off, c_tot)
    return y


def _pool(fn, x, k, stride, pad, dtype, y, c_off, c_tot):
    n, h, wd, c = x.shape
    p, q = out_dim(h, pad[0], k[0], stride[0]), out_dim(wd, pad[1], k[1], stride[1])
    y, c_tot = _out(y, n, p, q, c, c_off, c_tot)
    fn(_p(x), n, h, wd, c, k[0], k[1], stride[0], stride[1], pad[0], pad[1], _DT[dtype], _p(y), c_off, c_tot)
    return y


def maxpool(x, k, stride, pad=(0, 0), dtype="f32", y=None, c_off=0, c_tot=0):
    return _pool(lib().orc_maxpool, x, k, stride, pad, dtype, y, c_off, c_tot)


def avgpool(x, k, stride, pad=(0, 0), dtype="f32", y=None, c_off=0, c_tot=0):
    return _pool(lib().orc_avgpool, x, k, stride, pad, dtype, y, c_off, c_tot)


def global_avgpool(x, dtype="f32", y=None, c_off=0, c_tot=0):
    n, h, wd, c = x.shape
    y, c_tot = _out(y, n, 1, 1, c, c_off, c_tot)
    lib().orc_global_avgpool(_p(x), n, h, wd, c, _DT[dtype], _p(y), c_off, c_tot)
    return y


def fc(x, w, bias=None, act="none", dtype="f32"):
    n = x.shape[0]
    j = int(np.prod(x.shape[1:]))
    k, j2 = w.shape
    assert j == j2
    y = np.zeros((n, 1, 1, k), dtype=np.float32)
    lib().orc_fc(_p(np.ascontiguousarray(x.reshape(n, j))), n, j, _p(w), k, _p(bias), _ACT[act], _DT[dtype], _p(y))
    return y


def lrn(x, size, alpha, beta, k, dtype="f32"):
    """Local response normalisation across channels, as the AlexNet paper defines it (its Sec. 3.3):
    b[c] = a[c] / (k + alpha * sum_{j = max(0, c - size/2)}^{min(C-1, c + size/2)} a[j]^2) ** beta,
    alpha NOT divided by the window size.  Double precision, one rounding to the storage type."""
    n, h, wd, c = x.shape
    a = x.astype(np.float64)
    sq = a * a
    half = size // 2
    den = np.zeros_like(a)
    for ch in range(c):
        lo, hi = max(0, ch - half), min(c - 1, ch + half)
        den[..., ch] = sq[..., lo:hi + 1].sum(axis=-1)
    out = a / np.power(float(k) + float(alpha) * den, float(beta))
    return round_array_f64(out, dtype)


def add(x, other, act="none", dtype="f32"):
    """Element-wise sum of two tensors of the same shape, then the activation, one rounding."""
    assert x.shape == other.shape
    v = x.astype(np.float64) + other.astype(np.float64)
    if act == "relu":
        v = np.maximum(v, 0.0)
    elif act == "relu6":
        v = np.minimum(np.maximum(v, 0.0), 6.0)
    else:
        assert act == "none"
    return round_array_f64(v, dtype)


def round_array_f64(a, dtype):
    """Rounds a float64 array to the storage type."""
    flat = np.ascontiguousarray(a, dtype=np.float64).ravel()
    out = np.empty(flat.shape, dtype=np.float32)
    lib().orc_round_array_f64(flat.ctypes.data_as(C.POINTER(C.c_double)), _p(out), C.c_size_t(flat.size), _DT[dtype])
    return out.reshape(a.shape)


def conv_point(x, w, stride, pad, n, p, q, k):
    """Unrounded, bias-free value of one convolution output element."""
    _, h, wd, c = x.shape
    _, r, s, _ = w.shape
    return lib().orc_conv_point(_p(x), h, wd, c, _p(w), r, s, stride[0], stride[1], pad[0], pad[1], n, p, q, k)
