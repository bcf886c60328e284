"""CPU oracle of gradient-based rounding learning (Section V-B, Eq. (10)-(14)), in double precision with numpy.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

A linear layer without bias, as in the paper's exposition: weights W [N, K], one scale sw[n] per output channel,
format (e, m, b, c), one learnable parameter alpha per weight, calibration activations A [M, K] in full precision.

    y      = fl32(W * fl32(1 / sw))                the weight on the format's axis (same fp32 contract as Eq. (12))
    y'     = clamp(y, -c, c)                       Eq. (6)
    s      = 2^(max(floor(log2 |y'|) + b, 1) - b - m)            Eq. (9), from the clipped, unrounded weight
    q(a)   = clamp(s * (floor(y' / s) + sigmoid(a)), -c, c)      Eq. (12) with the sigmoid in place of the 0 / 1 decision
    Wq(a)  = q(a) * sw                             the soft-quantized weight
    mse    = mean over [M, N] of (A Wq^T - A W^T)^2              Eq. (11)
    reg    = mean over [N, K] of 1 - (2 |sigmoid(a) - 0.5|)^20   Eq. (14)
    loss   = mse + reg_weight * reg                Eq. (13)

One step of learning is plain gradient descent on alpha.  The hard decision used at inference is
h = [sigmoid(alpha) >= 0.5], which is the mask fpq_pack_weights / oracle.pack_weights take.
"""
import numpy as np


def sigmoid(a):
    a = np.asarray(a, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-a))


def on_format_axis(W, sw, fmt):
    """(y', s, floor(y' / s)) of every weight; y' uses the library's fp32 contract, the rest is exact in double."""
    e, m, b, c = fmt
    W = np.asarray(W, dtype=np.float32)
    r = (np.float32(1.0) / np.asarray(sw, dtype=np.float32)).astype(np.float32)
    y = (W * r[:, None]).astype(np.float32).astype(np.float64)
    yc = np.clip(y, -c, c)
    _, ex = np.frexp(np.abs(yc))                   # |y'| = mant * 2^ex, mant in [0.5, 1): floor(log2 |y'|) = ex - 1
    P = np.maximum(np.where(yc == 0, 1, ex - 1 + b), 1)
    s = np.ldexp(1.0, (P - b - m).astype(np.int64))
    return yc, s, np.floor(yc / s)


def soft_weights(W, sw, alpha, fmt):
    """Wq(alpha) [N, K] and its derivative with respect to alpha (zero where the outer clamp is active)."""
    c = fmt[3]
    yc, s, fl = on_format_axis(W, sw, fmt)
    sg = sigmoid(alpha)
    pre = s * (fl + sg)
    inside = (pre > -c) & (pre < c)
    swd = np.asarray(sw, dtype=np.float64)[:, None]
    return np.clip(pre, -c, c) * swd, np.where(inside, s * sg * (1.0 - sg), 0.0) * swd


def regulariser(alpha):
    """Mean of Eq. (14) over all weights, and its derivative with respect to each alpha."""
    sg = sigmoid(alpha)
    d = sg - 0.5
    u = 2.0 * np.abs(d)
    lam = 1.0 - u ** 20
    dlam = -20.0 * u ** 19 * 2.0 * np.sign(d) * sg * (1.0 - sg)
    return float(lam.mean()), dlam / lam.size


def loss(W, sw, alpha, A, fmt, reg_weight=1.0):
    """(mse, reg): loss = mse + reg_weight * reg."""
    Wq, _ = soft_weights(W, sw, alpha, fmt)
    A = np.asarray(A, dtype=np.float64)
    Yq = A @ Wq.T
    Y = A @ np.asarray(W, dtype=np.float64).T
    return float(np.mean((Yq - Y) ** 2)), regulariser(alpha)[0]


def gradient(W, sw, alpha, A, fmt, reg_weight=1.0):
    """d loss / d alpha [N, K], by the chain rule through Eq. (11)-(14)."""
    Wq, dWq = soft_weights(W, sw, alpha, fmt)
    A = np.asarray(A, dtype=np.float64)
    R = A @ Wq.T - A @ np.asarray(W, dtype=np.float64).T            # [M, N]
    G = (2.0 / R.size) * (R.T @ A)                                   # d mse / d Wq
    return G * dWq + reg_weight * regulariser(alpha)[1]


def step(W, sw, alpha, A, fmt, lr, reg_weight=1.0):
    """One gradient-descent step; returns (alpha_new, mse, reg) with the losses of the alpha that came in."""
    mse, reg = loss(W, sw, alpha, A, fmt, reg_weight)
    return np.asarray(alpha, dtype=np.float64) - lr * gradient(W, sw, alpha, A, fmt, reg_weight), mse, reg


def init_alpha(W, sw, fmt, eps=1e-3):
    """alpha with sigmoid(alpha) = the fractional position of each weight between its two grid neighbours (clipped to
    [eps, 1 - eps]), so that learning starts from the unquantized weights."""
    yc, s, fl = on_format_axis(W, sw, fmt)
    frac = np.clip(yc / s - fl, eps, 1.0 - eps)
    return np.log(frac / (1.0 - frac))


def mask(alpha):
    """The decision used at inference: 1 (round up) where sigmoid(alpha) >= 0.5."""
    return (sigmoid(alpha) >= 0.5).astype(np.uint8)


def im2col(x, kh, kw, stride, pad):
    """Patch matrix of a convolution input x [B, C, H, W]: row (b, ho, wo), column (ci, r, c) = x[b, ci, ho stride - pad + r,
    wo stride - pad + c], zero outside the image: a convolution with weight [Cout, C, kh, kw] is the linear layer with the
    weight flattened to [Cout, C kh kw] on this matrix."""
    x = np.asarray(x, dtype=np.float64)
    B, C, H, W = x.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    xp = np.zeros((B, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    a = np.zeros((B, Ho, Wo, C, kh, kw))
    for r in range(kh):
        for c in range(kw):
            a[:, :, :, :, r, c] = xp[:, :, r:r + stride * Ho:stride, c:c + stride * Wo:stride].transpose(0, 2, 3, 1)
    return a.reshape(B * Ho * Wo, C * kh * kw)
