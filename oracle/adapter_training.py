"""TEST INFRASTRUCTURE, NOT THE PRODUCT: CPU oracle of one training step of Kangaroo's adapter.

Only tests, the smoke check and the cpu_baseline leg of the benchmark may import this module.
It shares no code with the HIP library and imports nothing from it.

What is computed (Section 3.1, "Training Loss", Eq. 3; Section 4.1 names AdamW): with the target
model frozen, the adapter A (input RMSNorm, one causal multi-head attention with rotary positions,
residual, last RMSNorm, the target's LM head; Table 2 row "Kangaroo") is fitted so that the
self-draft distribution q_t = softmax(W_head . RMSNorm(A(f_1..f_t))) matches the target's
p_t = softmax(target logits at position t):

    loss = sum_t sum_n  - p_t[n] * log q_t[n]                                   (Eq. 3)

The other adapter architectures of Table 2's ablation are trained by the same loss (`kind`):
1 = the same attention with an LM head of its own, which is then trained too; 2 = a whole decoder
block, h <- h + Wd (silu(Wg b) * (Wu b)), b = RMSNorm(h; g_post), after the attention; 3 = two
linear maps, h = f + W2 silu(W1 RMSNorm(f; g_in)), and an own head.

The step takes the early features F [T, d] and the target logits Z_target [T, V] of one token
sequence as inputs (they come from the frozen model: its arithmetic is the decode oracle's), runs
the adapter over all T positions at once (teacher forcing, causal attention over earlier
features), and returns the loss, the gradient of every adapter parameter and the AdamW update.
Everything is float64 numpy, written as the chain rule reads: no fusion, no blocking.

Readings where the paper is silent: the sum of Eq. 3 is taken as printed (not averaged); keys and
values inside the training graph are not rounded to a cache's storage type; AdamW is the
decoupled-weight-decay rule of the paper it cites with bias correction,
    m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;  w <- w (1 - lr wd) - lr (m / (1-b1^s)) / (sqrt(v / (1-b2^s)) + eps)
with weight decay on the matrices and none on the gain vectors; the target model and its LM head
receive no update (an adapter's own head is one of its parameters and is trained).
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np

PARAMS = ("wq", "wk", "wv", "wo", "g_in", "g_last")
MATRICES = ("wq", "wk", "wv", "wo")
# parameter names per adapter architecture; names starting with "g_" are gain vectors (no weight decay)
KIND_PARAMS = {0: PARAMS,
               1: PARAMS + ("head",),
               2: PARAMS + ("g_post", "wg", "wu", "wd"),
               3: ("w1", "w2", "g_in", "g_last", "head")}


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def silu_grad(z: np.ndarray) -> np.ndarray:
    """d silu / dz = s (1 + z (1 - s)) with s = sigmoid(z)."""
    sg = 1.0 / (1.0 + np.exp(-z))
    return sg * (1.0 + z * (1.0 - sg))


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> Tuple[np.ndarray, np.ndarray]:
    """y = x * r * g with r = (mean(x^2) + eps)^(-1/2) per row; returns (y, r)."""
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    return x * r * g, r


def rmsnorm_backward(x: np.ndarray, g: np.ndarray, r: np.ndarray, dy: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Gradients (dx, dg) of y = x r g:  dx = r (dy g) - x r^3 mean((dy g) x),  dg = sum_rows dy x r."""
    u = dy * g
    dx = r * u - x * (r ** 3) * (u * x).mean(axis=-1, keepdims=True)
    dg = (dy * x * r).sum(axis=0)
    return dx, dg


def rope_angles(T: int, hd: int, theta: float) -> Tuple[np.ndarray, np.ndarray]:
    inv = theta ** (-np.arange(0, hd, 2, dtype=np.float64) / hd)
    ang = np.arange(T, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)                      # [T, hd/2]


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray, inverse: bool = False) -> np.ndarray:
    """Rotate pairs (i, i + hd/2) of x [T, H, hd] by the position's angle (by minus it if inverse:
    the transpose of the rotation, which is what the chain rule needs)."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    s = -sin if inverse else sin
    c = cos
    return np.concatenate([a * c[:, None, :] - b * s[:, None, :], b * c[:, None, :] + a * s[:, None, :]], axis=-1)


def softmax_rows(z: np.ndarray) -> np.ndarray:
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def loss_and_grads(P: Dict[str, np.ndarray], F: np.ndarray, Zt: np.ndarray, head: np.ndarray, n_heads: int,
                   eps: float, theta: float, kind: int = 0) -> Tuple[float, Dict[str, np.ndarray], Dict[str, np.ndarray]]:
    """Eq. 3 for one sequence and its gradient with respect to every adapter parameter.

    P: the tensors of KIND_PARAMS[kind] (matrices [rows, cols] as stored, gains [d]); F [T, d];
    Zt [T, V] target logits; head [V, d]: the target's LM head, used (frozen) by the architectures
    that share it.  Returns (loss, grads, intermediates {draft logits Z, h})."""
    T, d = F.shape
    H = n_heads
    hd = d // H
    G: Dict[str, np.ndarray] = {}
    # ---- forward
    n, r_in = rmsnorm(F, P["g_in"], eps)
    if kind == 3:
        u1 = n @ P["w1"].T
        s1 = silu(u1)
        hid = F + s1 @ P["w2"].T
    else:
        cos, sin = rope_angles(T, hd, theta)
        q = rope((n @ P["wq"].T).reshape(T, H, hd), cos, sin)
        k = rope((n @ P["wk"].T).reshape(T, H, hd), cos, sin)
        v = (n @ P["wv"].T).reshape(T, H, hd)
        mask = np.triu(np.ones((T, T), dtype=bool), 1)
        o = np.empty((T, H, hd))
        A = np.empty((H, T, T))
        for h in range(H):
            s = q[:, h] @ k[:, h].T / np.sqrt(hd)
            s[mask] = -np.inf
            A[h] = softmax_rows(s)
            o[:, h] = A[h] @ v[:, h]
        o2 = o.reshape(T, d)
        h1 = F + o2 @ P["wo"].T
        hid = h1
        if kind == 2:
            b, r_post = rmsnorm(h1, P["g_post"], eps)
            gt, ut = b @ P["wg"].T, b @ P["wu"].T
            act = silu(gt) * ut
            hid = h1 + act @ P["wd"].T
    m, r_last = rmsnorm(hid, P["g_last"], eps)
    W_head = P["head"] if kind in (1, 3) else head
    Z = m @ W_head.T
    qd = softmax_rows(Z)
    pd = softmax_rows(Zt)
    zs = Z - Z.max(axis=-1, keepdims=True)
    logq = zs - np.log(np.exp(zs).sum(axis=-1, keepdims=True))
    loss = float(-(pd * logq).sum())
    # ---- backward
    dZ = qd - pd                                   # d loss / d Z (each p row sums to 1)
    if kind in (1, 3):
        G["head"] = dZ.T @ m
    dm = dZ @ W_head
    dhid, G["g_last"] = rmsnorm_backward(hid, P["g_last"], r_last, dm)
    if kind == 3:
        G["w2"] = dhid.T @ s1
        du1 = (dhid @ P["w2"]) * silu_grad(u1)
        G["w1"] = du1.T @ n
        dn = du1 @ P["w1"]
    else:
        dh1 = dhid
        if kind == 2:
            G["wd"] = dhid.T @ act
            dact = dhid @ P["wd"]
            dgt = dact * ut * silu_grad(gt)
            dut = dact * silu(gt)
            G["wg"] = dgt.T @ b
            G["wu"] = dut.T @ b
            db = dgt @ P["wg"] + dut @ P["wu"]
            dx, G["g_post"] = rmsnorm_backward(h1, P["g_post"], r_post, db)
            dh1 = dhid + dx
        G["wo"] = dh1.T @ o2
        do = (dh1 @ P["wo"]).reshape(T, H, hd)
        dq = np.empty_like(q)
        dk = np.empty_like(k)
        dv = np.empty_like(v)
        for h in range(H):
            dA = do[:, h] @ v[:, h].T
            dv[:, h] = A[h].T @ do[:, h]
            dS = A[h] * (dA - (dA * A[h]).sum(axis=-1, keepdims=True))
            dq[:, h] = dS @ k[:, h] / np.sqrt(hd)
            dk[:, h] = dS.T @ q[:, h] / np.sqrt(hd)
        dq = rope(dq, cos, sin, inverse=True).reshape(T, d)
        dk = rope(dk, cos, sin, inverse=True).reshape(T, d)
        dv = dv.reshape(T, d)
        G["wq"], G["wk"], G["wv"] = dq.T @ n, dk.T @ n, dv.T @ n
        dn = dq @ P["wq"] + dk @ P["wk"] + dv @ P["wv"]
    _, G["g_in"] = rmsnorm_backward(F, P["g_in"], r_in, dn)
    return loss, G, {"Z": Z, "h": hid}


def adamw_step(P: Dict[str, np.ndarray], G: Dict[str, np.ndarray], M: Dict[str, np.ndarray], V: Dict[str, np.ndarray],
               step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.01) -> None:
    """One AdamW update in place for every tensor of P; `step` counts from 1.  Decay on the matrices
    only (names starting with "g_" are gain vectors)."""
    for name in P:
        g = G[name]
        M[name] = beta1 * M[name] + (1.0 - beta1) * g
        V[name] = beta2 * V[name] + (1.0 - beta2) * g * g
        mhat = M[name] / (1.0 - beta1 ** step)
        vhat = V[name] / (1.0 - beta2 ** step)
        wd = 0.0 if name.startswith("g_") else weight_decay
        P[name] = P[name] * (1.0 - lr * wd) - lr * mhat / (np.sqrt(vhat) + eps)


def zeros_like_params(P: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.zeros_like(v) for k, v in P.items()}
