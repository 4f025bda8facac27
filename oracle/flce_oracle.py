"""ctypes binding of the fp64 CPU oracle (flce_oracle.cpp).

TEST INFRASTRUCTURE ONLY: the slow plain definition of the loss and gradients
of a linear projection followed by softmax cross entropy (paper section 3.2,
CE and FLCE paragraphs), used to check the HIP path.  It imports nothing from
the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flce_oracle.cpp")
_LIB = os.path.join(_HERE, "libflce_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (portable x86-64-v3 code, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c++17",
               "-Wall", "-Wextra", _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        p, i64 = ctypes.c_void_p, ctypes.c_int64
        sig = [p, p, p, i64, i64, i64, i64, p, i64, p, i64, p, p, p, p, p]
        for name in ("flce_oracle_f64", "flce_oracle_f32in"):
            fn = getattr(lib, name)
            fn.argtypes, fn.restype = sig, ctypes.c_int
        lib.ce_oracle_f64.argtypes = [p, p, i64, i64, i64, p, p]
        lib.ce_oracle_f64.restype = ctypes.c_int
        lib.flce_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().flce_oracle_threads())


@dataclass
class OracleResult:
    loss: float
    lse: np.ndarray            # [BT] log-sum-exp of each row's logits
    dX: np.ndarray | None      # [BT or len(rows), H] fp64
    dW: np.ndarray | None      # [V or len(vocab), H] fp64
    G: np.ndarray | None       # [BT, V] dlogits, only when asked for


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def flce(X, W, targets, ignore_index=-100, rows=None, vocab=None, want_dX=True, want_dW=True,
         want_G=False) -> OracleResult:
    """Loss (mean over non-ignored rows), dX and dW of cross_entropy(X @ W.T, targets).

    X [BT, H] and W [V, H] are float64, or float32 (widened exactly inside).
    `rows` / `vocab` (int arrays) restrict dX / dW to those rows / vocabulary ids.
    """
    lib = _load()
    if X.dtype == np.float64 and W.dtype == np.float64:
        fn = lib.flce_oracle_f64
    elif X.dtype == np.float32 and W.dtype == np.float32:
        fn = lib.flce_oracle_f32in
    else:
        raise TypeError("X and W must both be float64 or both float32")
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    t = np.ascontiguousarray(targets, dtype=np.int64)
    BT, H = X.shape
    V, H2 = W.shape
    assert H == H2 and t.shape == (BT,)
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    vocab_a = None if vocab is None else np.ascontiguousarray(vocab, dtype=np.int64)
    if rows_a is not None:
        assert rows_a.ndim == 1 and ((rows_a >= 0) & (rows_a < BT)).all()
    if vocab_a is not None:
        assert vocab_a.ndim == 1 and ((vocab_a >= 0) & (vocab_a < V)).all()
    loss = np.zeros(1)
    lse = np.zeros(BT)
    dX = np.empty((BT if rows_a is None else len(rows_a), H)) if want_dX else None
    dW = np.empty((V if vocab_a is None else len(vocab_a), H)) if want_dW else None
    G = np.empty((BT, V)) if want_G else None
    rc = fn(_ptr(X), _ptr(W), _ptr(t), BT, H, V, ignore_index,
            _ptr(rows_a), 0 if rows_a is None else len(rows_a),
            _ptr(vocab_a), 0 if vocab_a is None else len(vocab_a),
            _ptr(loss), _ptr(lse), _ptr(dX), _ptr(dW), _ptr(G))
    if rc != 0:
        raise ValueError(f"oracle rejected its arguments (code {rc})")
    return OracleResult(float(loss[0]), lse, dX, dW, G)


@dataclass
class MultiHeadResult:
    loss: float                # sum_j weights[j] * head_losses[j]
    head_losses: list          # unweighted mean loss of each head
    dX: np.ndarray | None      # [BT, H] fp64, gradient of `loss`
    dWs: list | None           # per head [V, H] fp64, gradient of `loss`


def flce_multihead(X, Ws, targets, weights=None, ignore_index=-100, want_dX=True,
                   want_dW=True) -> MultiHeadResult:
    """Several heads on the same hidden states (paper section 4.2, Medusa
    paragraph): every head has a mean cross-entropy loss of its own over its own
    valid rows, and the training loss is their weighted sum.  Differentiation is
    linear, so the gradient of the sum is the weighted sum of each head's
    gradients: dX adds up over the heads, dW_j comes from head j alone."""
    n = len(Ws)
    assert len(targets) == n
    weights = [1.0] * n if weights is None else [float(w) for w in weights]
    assert len(weights) == n
    total, head_losses = 0.0, []
    dX = np.zeros(X.shape, dtype=np.float64) if want_dX else None
    dWs = [] if want_dW else None
    for W, t, w in zip(Ws, targets, weights):
        r = flce(X, W, t, ignore_index, want_dX=want_dX, want_dW=want_dW)
        head_losses.append(r.loss)
        total += w * r.loss
        if want_dX:
            dX += w * r.dX
        if want_dW:
            dWs.append(w * r.dW)
    return MultiHeadResult(total, head_losses, dX, dWs)


@dataclass
class RmsNormResult:
    loss: float
    y: np.ndarray              # [BT, H] normalised, scaled hidden states
    dh: np.ndarray | None      # [BT, H]
    dgamma: np.ndarray | None  # [H]
    dW: np.ndarray | None      # [V, H]


def rmsnorm_flce(h, gamma, eps, W, targets, ignore_index=-100, want_dh=True,
                 want_dW=True, vocab=None) -> RmsNormResult:
    """RMSNorm (paper section 3.2, RMSNorm paragraph) followed by the projection
    and cross entropy.  Forward, row by row: RMS = sqrt(sum_j h_j^2 / n + eps),
    xhat = h / RMS, y = xhat * gamma.  Backward with g = dL/dy:
    dh = (g*gamma - [xhat . (g*gamma) / n] xhat) / RMS, dgamma = sum over rows of
    g * xhat.  g is the dX of the linear cross-entropy oracle evaluated at X = y.
    `vocab` restricts dW to those vocabulary ids."""
    h = np.asarray(h, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    n = h.shape[1]
    rms = np.sqrt((h * h).sum(axis=1) / n + eps)
    xhat = h / rms[:, None]
    y = xhat * gamma[None, :]
    r = flce(y, np.asarray(W, dtype=np.float64), targets, ignore_index, vocab=vocab,
             want_dX=want_dh, want_dW=want_dW)
    dh = dgamma = None
    if want_dh:
        gg = r.dX * gamma[None, :]
        inner = (xhat * gg).sum(axis=1) / n
        dh = (gg - inner[:, None] * xhat) / rms[:, None]
        dgamma = (r.dX * xhat).sum(axis=0)
    return RmsNormResult(r.loss, y, dh, dgamma, r.dW)


def cross_entropy(Z, targets, ignore_index=-100):
    """Stand-alone CE on given logits Z [BT, V] (fp64): (loss, dlogits, lse)."""
    lib = _load()
    G = np.array(Z, dtype=np.float64, order="C", copy=True)
    t = np.ascontiguousarray(targets, dtype=np.int64)
    BT, V = G.shape
    loss = np.zeros(1)
    lse = np.zeros(BT)
    rc = lib.ce_oracle_f64(_ptr(G), _ptr(t), BT, V, ignore_index, _ptr(loss), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle rejected its arguments (code {rc})")
    return float(loss[0]), G, lse
