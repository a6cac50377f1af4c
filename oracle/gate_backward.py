"""CPU oracle of the gate gradients of one MeteoRA module (Sec. 3.2, Eq. 4; App. "Top-k strategy").

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy in float64, token by token.

Training keeps W, A_i and B_i fixed and updates only the gate (Sec. 3.2).  For one module with
input x[T,d_in] the joint loss of Eq. 4 reaches the gate parameters along two roads:

  * the language-model loss, through the module's output o (Eq. 2).  Its gradient with respect to o,
    dy[T,d_out], is handed in by the caller.  o depends on the gate through the weights w of the k
    selected adapters only (Eq. 3); the selection I(x) itself is piecewise constant and carries no
    gradient.  With v_j = scale * (x A_{a_j}) B_{a_j} the LoRA term is sum_j w_j v_j, so
        dL/dw_j = <dy, v_j>,
    and the softmax over the k selected logits gives
        dL/dg_{a_j} = w_j * (dL/dw_j - sum_i w_i dL/dw_i).
    For k = 1 the weight is the constant 1 and this part vanishes (App. "Top-1 strategy").
  * beta times the LoRA-classification loss of the module: the cross entropy between the softmax over
    all N gate logits and the token's task label,
        l = logsumexp(g) - g_label,        dl/dg_n = softmax(g)_n - [n == label].
    Eq. 4 sums l over tokens and modules (no mean); a caller who wants a mean folds 1/T into beta.
    A label outside [0, N) marks a token that has no task label: it gets no classification part.
    (Reading: the paper does not print l; "cross-entropy loss for LoRA classification" is taken as the
    N-way cross entropy on the raw logits.)

From d_logits[T,N] = dL/dg:  dW_gate = x^T d_logits,  dbias = sum_t d_logits[t].

The gradient with respect to the module's input (what the modules in front of this one need for their own
gates) collects the three roads x takes: the base projection, the selected adapters, and the gate,
    dx = dy W  +  scale * sum_j w_j ((dy B_{a_j}^T) A_{a_j}^T)  +  d_logits W_gate^T
with W stored [d_out, d_in] (o = x W^T in storage terms).
"""
from __future__ import annotations

import numpy as np

from . import gate_logits, topk_softmax


def gate_backward(x, dy, W_gate, bias, A, B, k: int, scale: float, labels=None, beta: float = 0.0, W=None):
    """Returns dict(dW_gate[d_in,N], dbias[N], d_logits[T,N], idx[T,k], w[T,k]), all float64 but idx;
    with W[d_out,d_in] given also dx[T,d_in]."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    T, d_in = x.shape
    N, _, r = A.shape
    d_out = B.shape[2]
    assert dy.shape == (T, d_out) and A.shape == (N, d_in, r) and B.shape == (N, r, d_out)

    g = gate_logits(x, W_gate, bias)                       # double, [T,N]
    g32 = g.astype(np.float32)                             # the routing decision is taken on fp32 logits
    idx, w = topk_softmax(g32, k)                          # Eq. 3 on the selected logits
    d_logits = np.zeros((T, N), dtype=np.float64)
    for t in range(T):
        dw = np.empty(k)
        for j in range(k):
            a = idx[t, j]
            v = scale * ((x[t] @ A[a]) @ B[a])             # the adapter's contribution before weighting
            dw[j] = dy[t] @ v
        mean = float(np.dot(w[t], dw))
        for j in range(k):
            d_logits[t, idx[t, j]] += w[t, j] * (dw[j] - mean)
        if labels is not None and beta != 0.0 and 0 <= int(labels[t]) < N:   # other values: token without a label
            gt = g32[t].astype(np.float64)
            p = np.exp(gt - gt.max())
            p /= p.sum()
            p[int(labels[t])] -= 1.0
            d_logits[t] += beta * p
    res = {"dW_gate": x.T @ d_logits, "dbias": d_logits.sum(axis=0), "d_logits": d_logits, "idx": idx, "w": w}
    if W is not None:
        W = np.asarray(W, dtype=np.float64)
        assert W.shape == (d_out, d_in)
        dx = dy @ W + d_logits @ np.asarray(W_gate, dtype=np.float64).T
        for t in range(T):
            for j in range(k):
                a = idx[t, j]
                dx[t] += scale * w[t, j] * ((dy[t] @ B[a].T) @ A[a].T)
        res["dx"] = dx
    return res
