"""Oracle of the uniform integer quantizer that the paper compares against (Section IV-A, Eq. (4)) and of a linear
layer computed on its codes.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, written from the equation:

    X_int = s * (clamp(round(X / s) + z; 0, 2^b - 1) - z),   s = (max(X) - min(X)) / (2^b - 1),   z = -round(min(X) / s)

Readings (the paper gives the real-number formula only):
  - round-to-nearest breaks ties towards the even integer (as for the floating-point quantizer);
  - fp32 evaluation order, needed for bit-exact codes: range = fl32(max - min), s = fl32(range / (2^b - 1)) (s = 1 for a
    constant tensor), r = fl32(1 / s), and every x / s is formed as y = fl32(x * r), one multiply, then rounded;
    z = -round(fl32(min * r)) is an integer that is NOT clamped to the code range (a tensor whose values all have one
    sign gets a zero point outside 0 .. 2^b - 1, as the equation says);
  - the code is the clamped integer q in 0 .. 2^b - 1; its value is s * (q - z);
  - weights take one (s, z) per output channel (the workload's granularity; per tensor is the case of equal entries);
  - the layer: Y[m, n] = sx * sw[n] * sum_k (qx[m, k] - zx) (qw[n, k] - zw[n]) (+ bias[n]), the sum in exact integers.
"""
import numpy as np


def params(x, bits):
    """(s, z) of Eq. (4) for the tensor x: fp32 scale and integer zero point."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    lo, hi = (np.float32(0), np.float32(0)) if x.size == 0 else (x.min(), x.max())
    rng = np.float32(hi - lo)
    s = np.float32(1.0) if rng == 0 else np.float32(rng / np.float32(2 ** bits - 1))
    r = np.float32(np.float32(1.0) / s)
    z = -int(np.rint(np.float32(lo * r)))
    return float(s), z


def quantize(x, bits, s, z):
    """Codes q = clamp(round(x / s) + z; 0, 2^b - 1) as uint8, same shape as x."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    r = np.float32(np.float32(1.0) / np.float32(s))
    y = (x * r).astype(np.float32)                      # one fp32 multiply per element
    q = np.rint(y.astype(np.float64)) + float(z)        # ties to even; integers far below 2^53
    return np.clip(q, 0, 2 ** bits - 1).astype(np.uint8)


def dequantize(q, s, z):
    """s * (q - z) in double (s, z scalars or arrays broadcast over the leading axis)."""
    q = np.asarray(q, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    z = np.asarray(z, dtype=np.float64)
    if s.ndim == 1:
        s = s.reshape((-1,) + (1,) * (q.ndim - 1))
        z = z.reshape((-1,) + (1,) * (q.ndim - 1))
    return s * (q - z)


def pack_weights(w, bits):
    """Per-output-channel Eq. (4) on w[N, K]: (codes uint8 [N, K], s float32 [N], z int32 [N])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    N = w.shape[0]
    codes = np.empty(w.shape, dtype=np.uint8)
    s = np.empty(N, dtype=np.float32)
    z = np.empty(N, dtype=np.int32)
    for n in range(N):
        sn, zn = params(w[n], bits)
        s[n], z[n] = sn, zn
        codes[n] = quantize(w[n], bits, sn, zn)
    return codes, s, z


def gemm(xq, sx, zx, wq, sw, zw, bias=None, rows=None):
    """Linear layer on integer codes: (Y, T) float64 [M or len(rows), N], T = sx * sw[n] * sum_k |(qx - zx)(qw - zw)|."""
    xq = np.asarray(xq)
    if rows is not None:
        xq = xq[np.asarray(rows)]
    a = xq.astype(np.int64) - int(zx)                                   # [M, K]
    b = np.asarray(wq).astype(np.int64) - np.asarray(zw).astype(np.int64)[:, None]   # [N, K]
    acc = a @ b.T                                                       # exact: |entries| < 2^63
    tacc = np.abs(a) @ np.abs(b).T
    scale = float(np.float32(sx)) * np.asarray(sw, dtype=np.float64)[None, :]
    Y = scale * acc.astype(np.float64)
    T = scale * tacc.astype(np.float64)
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[None, :]
    return Y, T
