"""Agile Swin Transformer Layer (ASTL) -- plain CPU oracle, fp64 numpy.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg of the benchmark
call this; the HIP library never does and shares no code with it.

The layer (AgileIR, Sec. "Agile Swin Transformer Block", Eq. 4-5), token by token over the
feature map x [B, H, W, C]:

    x1 = GSWA(LN_1(x)) + x                                             Eq. 4
    y  = MLP(LN_2(x1)) + x1                                            Eq. 5
    LN(u)  = (u - mean(u)) / sqrt(var(u) + eps) * gamma + beta         over the C channels of a token,
                                                                       var = mean of squared deviations
    MLP(u) = GELU(u W1^T + b1) W2^T + b2                               two fully connected layers
    GELU(t) = t * Phi(t),  Phi(t) = (1 + erf(t / sqrt 2)) / 2          the Gaussian-CDF form

GSWA is the attention layer of ``gswa_oracle`` (Eq. 6-8), called as it stands.  The paper
states the two equations, "two fully-connected layers and GELU" and the placement of the
LayerNorms; the hidden width, eps and the exact (erf) form of GELU are this oracle's readings:
they are parameters (hidden = rows of W1, eps) or the textbook definition (GELU).

Every step is its definition written out with numpy matrix products; the backward pass is the
hand-derived adjoint of the same steps, in reverse order.  No autograd library is involved.

Parity pins (tests, CPU only): LayerNorm, GELU and the MLP half against torch's CPU routines
and its autograd in fp64 (a library written independently of this file); printed values of the
Gaussian CDF; closed forms (zero W2 leaves x1, zero gamma_1 feeds GSWA zeros, LN output
statistics, invariance of LN under shift and scale of its input); central finite differences
of the whole layer for every gradient, attention half included; for a sequence of layers,
central differences through two layers and the alternation of the shift.
"""
import numpy as np
from scipy.special import erf

from . import gswa_oracle

PARAM_NAMES = ("ln1_w", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "table",
               "ln2_w", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
_ATTN = ("w_qkv", "b_qkv", "w_proj", "b_proj", "table")


def layer_norm(u, gamma, beta, eps):
    """LN over the last axis; returns (out, normalised input, 1/sqrt(var+eps))."""
    mean = u.mean(axis=-1, keepdims=True)
    var = ((u - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (u - mean) * rstd
    return xhat * gamma + beta, xhat, rstd


def layer_norm_backward(dout, xhat, rstd, gamma):
    """Adjoint of layer_norm: (du, dgamma, dbeta) for out = xhat * gamma + beta."""
    dxhat = dout * gamma
    du = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    C = dout.shape[-1]
    return du, (dout * xhat).reshape(-1, C).sum(axis=0), dout.reshape(-1, C).sum(axis=0)


def gelu(t):
    return t * 0.5 * (1.0 + erf(t / np.sqrt(2.0)))


def gelu_grad(t):
    """d GELU / dt = Phi(t) + t * phi(t), phi the standard normal density."""
    return 0.5 * (1.0 + erf(t / np.sqrt(2.0))) + t * np.exp(-0.5 * t * t) / np.sqrt(2.0 * np.pi)


def mlp(u, w1, b1, w2, b2):
    """[.., C] -> [.., C]; returns (out, pre-activation, hidden)."""
    pre = u @ w1.T + b1
    h = gelu(pre)
    return h @ w2.T + b2, pre, h


def mlp_backward(dout, u, pre, h, w1, w2):
    """Adjoint of mlp: (du, dw1, db1, dw2, db2)."""
    C, Hd = u.shape[-1], pre.shape[-1]
    d2, h2, u2 = dout.reshape(-1, C), h.reshape(-1, Hd), u.reshape(-1, C)
    dw2 = d2.T @ h2
    db2 = d2.sum(axis=0)
    dpre = (d2 @ w2) * gelu_grad(pre.reshape(-1, Hd))
    dw1 = dpre.T @ u2
    db1 = dpre.sum(axis=0)
    return (dpre @ w1).reshape(u.shape), dw1, db1, dw2, db2


def _f64(p):
    return {k: np.asarray(p[k], dtype=np.float64) for k in PARAM_NAMES}


def forward(x, p, *, heads, groups, window, shift, eps=1e-5, cascade=True, dqk=0, want_mid=False):
    """y = ASTL(x); p maps PARAM_NAMES to arrays (hidden width = rows of w_fc1)."""
    x = np.asarray(x, dtype=np.float64)
    p = _f64(p)
    kw = dict(heads=heads, groups=groups, window=window, shift=shift, cascade=cascade, dqk=dqk)
    xn, _, _ = layer_norm(x, p["ln1_w"], p["ln1_b"], eps)
    x1 = gswa_oracle.forward(xn, *[p[k] for k in _ATTN], **kw) + x
    x1n, _, _ = layer_norm(x1, p["ln2_w"], p["ln2_b"], eps)
    m, _, _ = mlp(x1n, p["w_fc1"], p["b_fc1"], p["w_fc2"], p["b_fc2"])
    y = m + x1
    return (y, x1) if want_mid else y


def backward(x, dy, p, *, heads, groups, window, shift, eps=1e-5, cascade=True, dqk=0):
    """Gradients of sum(dy * y): (dx, dict of parameter gradients keyed like p)."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    p = _f64(p)
    kw = dict(heads=heads, groups=groups, window=window, shift=shift, cascade=cascade, dqk=dqk)
    attn = [p[k] for k in _ATTN]
    # forward, keeping what the adjoint needs
    xn, xhat1, rstd1 = layer_norm(x, p["ln1_w"], p["ln1_b"], eps)
    x1 = gswa_oracle.forward(xn, *attn, **kw) + x
    x1n, xhat2, rstd2 = layer_norm(x1, p["ln2_w"], p["ln2_b"], eps)
    _, pre, h = mlp(x1n, p["w_fc1"], p["b_fc1"], p["w_fc2"], p["b_fc2"])
    # Eq. 5 backwards: y = MLP(LN_2(x1)) + x1
    g = {}
    dx1n, g["w_fc1"], g["b_fc1"], g["w_fc2"], g["b_fc2"] = mlp_backward(
        dy, x1n, pre, h, p["w_fc1"], p["w_fc2"])
    dx1, g["ln2_w"], g["ln2_b"] = layer_norm_backward(dx1n, xhat2, rstd2, p["ln2_w"])
    dx1 = dx1 + dy
    # Eq. 4 backwards: x1 = GSWA(LN_1(x)) + x
    dxn, *dattn = gswa_oracle.backward(xn, dx1, *attn, **kw)
    g.update(zip(_ATTN, dattn))
    dx, g["ln1_w"], g["ln1_b"] = layer_norm_backward(dxn, xhat1, rstd1, p["ln1_w"])
    return dx + dx1, g


def stack_forward(x, params, *, heads, groups, window, shift, eps=1e-5, dqk=0, want_inputs=False, store=None):
    """A sequence of layers (Sec. "Agile Swin Transformer Block"): layer l has shift 0 for even l and
    ``shift`` for odd l, its own parameters ``params[l]``, and takes the output of layer l - 1.

    ``store`` (optional callable, array -> array) is applied to every activation that crosses a layer
    boundary: with the rounding of the storage type it states that the tensor handed from one layer
    to the next IS a tensor of that type ("bf16 activations with fp32 accumulation"); None keeps
    fp64 throughout.  The arithmetic inside a layer is fp64 either way."""
    acts = [np.asarray(x, dtype=np.float64)]
    for l, p in enumerate(params):
        y = forward(acts[-1], p, heads=heads, groups=groups, window=window,
                    shift=shift if l % 2 else 0, eps=eps, dqk=dqk)
        if store is not None and l + 1 < len(params):
            y = np.asarray(store(y), dtype=np.float64)
        acts.append(y)
    return (acts[-1], acts[:-1]) if want_inputs else acts[-1]


def stack_backward(x, dy, params, *, heads, groups, window, shift, eps=1e-5, dqk=0, store=None):
    """Gradients of sum(dy * y) through the sequence: (dx, list of per-layer gradient dicts).
    ``store`` as in stack_forward; it is also applied to the gradient handed from layer l to layer
    l - 1 (the same boundary, crossed in the other direction)."""
    _, inputs = stack_forward(x, params, heads=heads, groups=groups, window=window, shift=shift, eps=eps,
                              dqk=dqk, want_inputs=True, store=store)
    g = np.asarray(dy, dtype=np.float64)
    grads = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        g, grads[l] = backward(inputs[l], g, params[l], heads=heads, groups=groups, window=window,
                               shift=shift if l % 2 else 0, eps=eps, dqk=dqk)
        if store is not None and l > 0:
            g = np.asarray(store(g), dtype=np.float64)
    return g, grads
