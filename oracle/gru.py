"""Oracle for the recurrent workload: embedding lookup, one GRU layer, and their gradients through time.

TEST INFRASTRUCTURE ONLY (see the package docstring): plain numpy float64, one definition per function, time steps
in a Python loop, no fusion.  Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this module.

What the paper fixes (section "Experiments and Discussion"): an embedding layer over the vocabulary, one GRU layer
with hidden size 256 and an output layer; batch 50, sequence length 200, vocabulary 32768, cross entropy over 2
classes, AdamW.  It prints no equations; the GRU is the one of its reference [gru] in the gate convention of the
framework it compares against (reset gate applied to the recurrent candidate term, separate input and recurrent
biases):
    r = sigmoid(W_ir x + b_ir + W_hr h + b_hr)
    z = sigmoid(W_iz x + b_iz + W_hz h + b_hz)
    n = tanh(W_in x + b_in + r * (W_hn h + b_hn))
    h' = (1 - z) * n + z * h
Weights are stored [3H][inputs] with the gates in the order (r, z, n), and a product with a weight is the `@` operator
of section "Automatic Differentiation" (multiplication by the transposed weight).  Gradients are derived by hand from
these four lines and accumulated over the time steps (the accumulation rule of the same section).
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


# ----------------------------------------------------------------------------- embedding

def embedding_fwd(tokens, table) -> np.ndarray:
    """out[i] = table[tokens[i]]."""
    return _f64(table)[np.asarray(tokens, dtype=np.int64)]


def embedding_bwd(tokens, dout, vocab: int, into: Optional[np.ndarray] = None) -> np.ndarray:
    """dtable[v] (+)= sum over the positions i with tokens[i] == v of dout[i]."""
    tokens = np.asarray(tokens, dtype=np.int64).reshape(-1)
    dout = _f64(dout).reshape(tokens.size, -1)
    dtable = np.zeros((vocab, dout.shape[1])) if into is None else _f64(into).copy()
    for i, v in enumerate(tokens):
        dtable[v] += dout[i]
    return dtable


# ----------------------------------------------------------------------------- one GRU step

def gru_gates_fwd(gi, gh, b_ih, b_hh, h_prev):
    """The elementwise part of a step from the two products gi = x @ W_ih and gh = h @ W_hh ([N, 3H], gates r, z, n).
    Returns (h_new, r, z, n, q) with q = gh_n + b_hn (the recurrent candidate term the backward pass needs)."""
    gi, gh, h_prev = _f64(gi), _f64(gh), _f64(h_prev)
    b_ih, b_hh = _f64(b_ih), _f64(b_hh)
    H = h_prev.shape[1]
    r = _sigmoid(gi[:, :H] + b_ih[:H] + gh[:, :H] + b_hh[:H])
    z = _sigmoid(gi[:, H:2 * H] + b_ih[H:2 * H] + gh[:, H:2 * H] + b_hh[H:2 * H])
    q = gh[:, 2 * H:] + b_hh[2 * H:]
    n = np.tanh(gi[:, 2 * H:] + b_ih[2 * H:] + r * q)
    return (1.0 - z) * n + z * h_prev, r, z, n, q


def gru_gates_bwd(r, z, n, q, h_prev, dh):
    """Gradients of the step with respect to gi, gh ([N, 3H] each) and the direct part of dh_prev (dh * z); the part of
    dh_prev that flows through gh @ W_hh is the caller's matrix product."""
    r, z, n, q, h_prev, dh = (_f64(a) for a in (r, z, n, q, h_prev, dh))
    dn = dh * (1.0 - z)
    dz = dh * (h_prev - n)
    da_n = dn * (1.0 - n * n)                 # through tanh
    da_z = dz * z * (1.0 - z)                 # through sigmoid
    dr = da_n * q
    da_r = dr * r * (1.0 - r)
    dgi = np.concatenate([da_r, da_z, da_n], axis=1)
    dgh = np.concatenate([da_r, da_z, da_n * r], axis=1)
    return dgi, dgh, dh * z


# ----------------------------------------------------------------------------- the layer over time

def gru_forward(x, h0, w_ih, w_hh, b_ih, b_hh) -> dict:
    """x: [T, N, E], h0: [N, H].  Returns dict(h=[T+1, N, H] with h[0] = h0, r, z, n, q=[T, N, H])."""
    x, w_ih, w_hh = _f64(x), _f64(w_ih), _f64(w_hh)
    T = x.shape[0]
    h = [_f64(h0)]
    saved = {k: [] for k in "rznq"}
    for t in range(T):
        gi = x[t] @ w_ih.T
        gh = h[-1] @ w_hh.T
        hn, r, z, n, q = gru_gates_fwd(gi, gh, b_ih, b_hh, h[-1])
        h.append(hn)
        for k, v in zip("rznq", (r, z, n, q)):
            saved[k].append(v)
    out = {k: np.stack(v) for k, v in saved.items()}
    out["h"] = np.stack(h)
    return out


def gru_backward(x, fwd: dict, w_ih, w_hh, dh_all) -> dict:
    """dh_all: [T, N, H], the gradient reaching every h[t+1] from outside the recurrence (zeros where there is none).
    Returns dx [T, N, E], dh0, dw_ih, dw_hh, db_ih, db_hh; parameter gradients are summed over the time steps."""
    x, w_ih, w_hh, dh_all = _f64(x), _f64(w_ih), _f64(w_hh), _f64(dh_all)
    T, N, E = x.shape
    H = w_hh.shape[1]
    dx = np.zeros_like(x)
    dw_ih, dw_hh = np.zeros_like(w_ih), np.zeros_like(w_hh)
    db_ih, db_hh = np.zeros(3 * H), np.zeros(3 * H)
    dh = np.zeros((N, H))
    for t in reversed(range(T)):
        dh = dh + dh_all[t]
        dgi, dgh, dh_direct = gru_gates_bwd(fwd["r"][t], fwd["z"][t], fwd["n"][t], fwd["q"][t], fwd["h"][t], dh)
        dx[t] = dgi @ w_ih
        dw_ih += dgi.T @ x[t]
        dw_hh += dgh.T @ fwd["h"][t]
        db_ih += dgi.sum(axis=0)
        db_hh += dgh.sum(axis=0)
        dh = dh_direct + dgh @ w_hh
    return dict(dx=dx, dh0=dh, dw_ih=dw_ih, dw_hh=dw_hh, db_ih=db_ih, db_hh=db_hh)
