"""Float64 CPU oracle of the sparse operators around the dropout.

TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this.  It never touches the HIP library and shares
no code with it.

arxiv 2411.01238, Section 4.3 (closing remark) proposes sparse operators for the
layer directly before the dropout as well.  The block this file defines is

    Z = H W0^T + b0            the producing layer (W0 holds one row per output feature)
    X = m . act(Z)             its activation, then the block mask m' of Section 3.2
    Y = s X W                  eq. (1) (X is already masked), s = 1/(1-p)

and everything below is that definition, or its derivative, written out with
dense numpy products: the element mask is expanded from the block flags and
multiplied in, nothing is skipped or reordered.
"""
import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_GELU_ERF = 0, 1, 2, 3


def expand(keep, BM, BK):
    """Element mask m[M,K] of the block flags keep[MB,KB] (Section 3.2: one flag per BM x BK block)."""
    return np.kron(np.asarray(keep, dtype=np.float64), np.ones((BM, BK)))


def scale_of(p, scale_one=False):
    """s of eq. (1)-(3); 0 when everything is dropped; 1 for a product that is no dropout output."""
    if scale_one:
        return 1.0
    return 1.0 / (1.0 - p) if p < 1.0 else 0.0


def act(v, kind):
    """ReLU, GELU in its tanh form 0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3))), or GELU itself,
    0.5 v (1 + erf(v / sqrt 2)) = v Phi(v)."""
    v = np.asarray(v, dtype=np.float64)
    if kind == ACT_NONE:
        return v
    if kind == ACT_RELU:
        return np.where(v > 0.0, v, 0.0)
    if kind == ACT_GELU_TANH:
        return 0.5 * v * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (v + 0.044715 * v ** 3)))
    if kind == ACT_GELU_ERF:
        from scipy.special import erf          # the error function itself is a library primitive
        return 0.5 * v * (1.0 + erf(v / np.sqrt(2.0)))
    raise ValueError("unknown activation")


GATE_RELU, GATE_GELU_TANH, GATE_GELU_ERF = 0, 1, 2


def act_grad(z, kind):
    """Derivative of act(., kind) at z.

    ReLU: [z > 0].  tanh-GELU g = 0.5 z (1 + t), t = tanh(u), u = c (z + a z^3):
    g' = 0.5 (1 + t) + 0.5 z (1 - t^2) c (1 + 3 a z^2).  GELU g = z Phi(z): g' = Phi(z) + z phi(z)."""
    z = np.asarray(z, dtype=np.float64)
    if kind == ACT_NONE:
        return np.ones_like(z)
    if kind == ACT_RELU:
        return (z > 0.0).astype(np.float64)
    if kind == ACT_GELU_TANH:
        c, a = np.sqrt(2.0 / np.pi), 0.044715
        t = np.tanh(c * (z + a * z ** 3))
        return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * c * (1.0 + 3.0 * a * z * z)
    if kind == ACT_GELU_ERF:
        from scipy.special import erf
        return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    raise ValueError("unknown activation")


def gate(v, g, gate_mode):
    """v gated by g: zero where g <= 0 (ReLU), or times the GELU's derivative at g."""
    g = np.asarray(g, dtype=np.float64)
    if gate_mode == GATE_RELU:
        return np.where(g > 0.0, v, 0.0)
    return v * act_grad(g, ACT_GELU_TANH if gate_mode == GATE_GELU_TANH else ACT_GELU_ERF)


def tail(v, bias=None, kind=ACT_NONE, relu_mask=None, gate_mode=GATE_RELU):
    """gate(act(v + bias[column]), relu_mask)."""
    v = np.asarray(v, dtype=np.float64)
    if bias is not None:
        v = v + np.asarray(bias, dtype=np.float64)[None, :]
    v = act(v, kind)
    if relu_mask is not None:
        v = gate(v, relu_mask, gate_mode)
    return v


def fwd_tail(X, W, keep, BM, BK, p, scale_one=False, bias=None, kind=ACT_NONE, relu_mask=None, gate_mode=GATE_RELU):
    """eq. (1) followed by the tail: [relu_mask > 0] act(s (X . m) W + bias)."""
    X = np.asarray(X, dtype=np.float64)
    m = expand(keep, BM, BK)
    # dropped blocks of X may hold anything (NaN included): they are excluded, not multiplied by 0
    Xm = np.where(m > 0.0, X, 0.0)
    return tail(scale_of(p, scale_one) * (Xm @ np.asarray(W, dtype=np.float64)), bias, kind, relu_mask, gate_mode)


def bwd_dx_tail(dY, W, keep, BM, BK, p, scale_one=False, bias=None, kind=ACT_NONE, relu_mask=None, gate_mode=GATE_RELU):
    """eq. (2) with the tail on the kept blocks: m . [relu_mask > 0] act(s dY W^T + bias)."""
    m = expand(keep, BM, BK)
    full = scale_of(p, scale_one) * (np.asarray(dY, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T)
    rm = None if relu_mask is None else np.where(m > 0.0, np.asarray(relu_mask, dtype=np.float64), 0.0)
    return np.where(m > 0.0, tail(full, bias, kind, rm, gate_mode), 0.0)


def bwd_dw_scaled(X, dY, keep, BM, BK, p, scale_one=False):
    """eq. (3) with the chosen scale: s (X . m)^T dY."""
    m = expand(keep, BM, BK)
    Xm = np.where(m > 0.0, np.asarray(X, dtype=np.float64), 0.0)
    return scale_of(p, scale_one) * (Xm.T @ np.asarray(dY, dtype=np.float64))


def bias_grad(dZ, keep, BM, BK):
    """db0 of the block: column sums of dZ over the kept blocks, db0[k] = sum_r (dZ . m)[r, k]
    (b0 enters Z = H W0^T + b0 once per row, and only the kept blocks of Z reach the output)."""
    m = expand(keep, BM, BK)
    # dropped blocks of dZ may hold anything: excluded, not multiplied by 0
    return np.where(m > 0.0, np.asarray(dZ, dtype=np.float64), 0.0).sum(axis=0)


def producer(H, W0, b0, keep, BM, BK, kind=ACT_NONE):
    """X = m . act(H W0^T + b0), W0 is [K, N0]."""
    Z = np.asarray(H, dtype=np.float64) @ np.asarray(W0, dtype=np.float64).T
    return expand(keep, BM, BK) * tail(Z, b0, kind)


def producer_preact(H, W0, b0, keep, BM, BK):
    """m . (H W0^T + b0): the producing layer's value before the activation, on the kept blocks."""
    return producer(H, W0, b0, keep, BM, BK, ACT_NONE)


def block_forward(H, W0, b0, W, keep, BM, BK, p, kind=ACT_RELU):
    """Returns (X, Y) of the block defined at the top."""
    X = producer(H, W0, b0, keep, BM, BK, kind)
    Y = scale_of(p) * (X @ np.asarray(W, dtype=np.float64))
    return X, Y


def block_backward(H, W0, b0, W, keep, BM, BK, p, dY, kind=ACT_RELU):
    """Gradients of sum(Y . dY) for the block, by the chain rule:

        dX  = s (dY W^T) . m            eq. (2)
        dZ  = dX . act'(Z)              [Z > 0] for ReLU
        dW  = s X^T dY                  eq. (3)
        dH  = dZ W0,   dW0 = dZ^T H,   db0 = column sums of dZ

    Returns a dict with dH, dW0, db0, dW, dZ and Z.
    """
    H = np.asarray(H, dtype=np.float64)
    W0 = np.asarray(W0, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    m = expand(keep, BM, BK)
    s = scale_of(p)
    Z = H @ W0.T + (0.0 if b0 is None else np.asarray(b0, dtype=np.float64)[None, :])
    X = m * act(Z, kind)
    dX = s * (dY @ W.T) * m
    dZ = dX * act_grad(Z, kind)
    return {"dH": dZ @ W0, "dW0": dZ.T @ H, "db0": bias_grad(dZ, keep, BM, BK), "dW": s * (X.T @ dY), "dZ": dZ, "Z": Z}
