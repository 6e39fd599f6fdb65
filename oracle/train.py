"""Oracle for the operations that close a training step behind the residual blocks: global average pooling, the
fully connected layer, the softmax cross-entropy loss, and the optimizer updates.

TEST INFRASTRUCTURE ONLY (see the package docstring): plain numpy float64, one definition per function, no blocking
or fusion.  Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this module.

What the paper fixes and what it leaves open:
  * the network is the ResNet recipe (section "Experiments and Discussion"): its head is a global average pool, a
    fully connected layer and a cross-entropy loss; the recipe's optimizer is SGD with momentum and weight decay;
  * the fully connected layer is the `@` operator of section "Automatic Differentiation": y = x @ w multiplies by the
    TRANSPOSED weight, w is stored [outputs][inputs]; its two gradients follow the matrix-multiply gradient rule of
    the same section and are accumulated into existing buffers;
  * the last node of a step must be a loss (same section); the recurrent experiment names cross entropy, AdamW with
    learning rate 0.001, weight decay 0.0001 and a gradient clip of 5 (section "Experiments and Discussion");
  * gradient buffers of parameters are overwritten with zeros once the optimizer has used them (section "Caching and
    Pooling").
The paper gives no formulas for any of these, so the textbook definitions are used: mean over the spatial positions;
loss = mean over the batch of (log-sum-exp of the logits - logit of the label); SGD as v <- mu*v + (g + wd*w),
w <- w - lr*v; AdamW as in Loshchilov & Hutter (decoupled decay, bias-corrected moments); the clip scales all
gradients by min(1, c / (global L2 norm + 1e-6)).
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


# ----------------------------------------------------------------------------- global average pool

def global_avgpool_fwd(x) -> np.ndarray:
    """y[n][c] = mean over (h, w) of x[n][c][h][w]  (head of the ResNet recipe, section "Experiments and Discussion")."""
    x = _f64(x)
    return x.sum(axis=(2, 3)) / float(x.shape[2] * x.shape[3])


def global_avgpool_bwd(dy, xshape, into: Optional[np.ndarray] = None) -> np.ndarray:
    """dx[n][c][h][w] (+)= dy[n][c] / (H*W): every position contributed with weight 1/(H*W)."""
    dy = _f64(dy)
    N, C, H, W = xshape
    dx = np.broadcast_to(dy[:, :, None, None] / float(H * W), (N, C, H, W))
    return dx.copy() if into is None else _f64(into) + dx


# ----------------------------------------------------------------------------- fully connected layer (the `@` operator)

def linear_fwd(x, w, bias=None) -> np.ndarray:
    """y[n][k] = sum_c x[n][c] * w[k][c] (+ bias[k]): `x @ w` with w transposed (section "Automatic Differentiation")."""
    y = _f64(x) @ _f64(w).T
    return y if bias is None else y + _f64(bias)[None, :]


def linear_dgrad(dy, w, into: Optional[np.ndarray] = None) -> np.ndarray:
    """dx[n][c] (+)= sum_k dy[n][k] * w[k][c]."""
    dx = _f64(dy) @ _f64(w)
    return dx if into is None else _f64(into) + dx


def linear_wgrad(x, dy, into_dw: Optional[np.ndarray] = None, into_db: Optional[np.ndarray] = None):
    """dw[k][c] (+)= sum_n dy[n][k] * x[n][c];  db[k] (+)= sum_n dy[n][k]."""
    dw = _f64(dy).T @ _f64(x)
    db = _f64(dy).sum(axis=0)
    if into_dw is not None:
        dw = _f64(into_dw) + dw
    if into_db is not None:
        db = _f64(into_db) + db
    return dw, db


# ----------------------------------------------------------------------------- loss

def softmax_xent_fwd(logits, labels) -> Tuple[float, np.ndarray]:
    """loss = mean_n ( log sum_k exp(z[n][k]) - z[n][label_n] ).  Returns (loss, per-sample losses)."""
    z = _f64(logits)
    labels = np.asarray(labels, dtype=np.int64)
    zmax = z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(z - zmax).sum(axis=1)) + zmax[:, 0]
    per = lse - z[np.arange(z.shape[0]), labels]
    return float(per.mean()), per


def softmax_xent_bwd(logits, labels, dloss: float = 1.0) -> np.ndarray:
    """dz[n][k] = dloss/N * (softmax(z[n])[k] - [k == label_n])."""
    z = _f64(logits)
    labels = np.asarray(labels, dtype=np.int64)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    p[np.arange(z.shape[0]), labels] -= 1.0
    return p * (dloss / z.shape[0])


# ----------------------------------------------------------------------------- optimizer

def clip_scale(grads, max_norm: float) -> float:
    """min(1, max_norm / (sqrt(sum of squares of all gradients) + 1e-6))."""
    total = 0.0
    for g in grads:
        g = _f64(g)
        total += float((g * g).sum())
    return min(1.0, max_norm / (np.sqrt(total) + 1e-6))


def sgd_momentum_step(w, g, v, lr: float, momentum: float, weight_decay: float, grad_scale: float = 1.0):
    """g' = grad_scale*g + wd*w;  v <- mu*v + g';  w <- w - lr*v;  the gradient buffer becomes zero.
    Returns (w, v, g)."""
    w, g, v = _f64(w), _f64(g), _f64(v)
    g2 = grad_scale * g + weight_decay * w
    v = momentum * v + g2
    w = w - lr * v
    return w, v, np.zeros_like(g)


def adamw_step(w, g, m, v, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.0, grad_scale: float = 1.0):
    """AdamW, step counted from 1:  w <- w*(1 - lr*wd);  m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g^2;
    w <- w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps);  the gradient buffer becomes zero.
    Returns (w, m, v, g)."""
    w, g, m, v = _f64(w), _f64(g) * grad_scale, _f64(m), _f64(v)
    w = w * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    w = w - lr * mhat / (np.sqrt(vhat) + eps)
    return w, m, v, np.zeros_like(g)
