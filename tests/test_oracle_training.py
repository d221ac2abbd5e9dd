"""Pins for the oracle's adapter training step (oracle/adapter_training.py, Eq. 3 + AdamW) against
things that are not the oracle: torch's reverse-mode differentiation of a forward composed from
library ops, central finite differences, torch.optim.AdamW, closed forms, and the decode oracle's
own adapter (the training graph must be the network that drafts)."""
import numpy as np
import pytest
import torch

from oracle import adapter_training as TR
from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import inputs as I


def problem(T=7, d=32, H=4, V=48, seed=0, gains=True, kind=0, ffn=40):
    rng = np.random.default_rng(seed)
    shapes = {"wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d), "w1": (d, d), "w2": (d, d),
              "wg": (ffn, d), "wu": (ffn, d), "wd": (d, ffn), "head": (V, d)}
    P = {}
    for name in TR.KIND_PARAMS[kind]:
        if name.startswith("g_"):
            P[name] = 1.0 + 0.3 * rng.standard_normal(d) if gains else np.ones(d)
        else:
            P[name] = rng.standard_normal(shapes[name]) * (0.3 if name == "head" else 0.2)
    F = rng.standard_normal((T, d))
    Zt = rng.standard_normal((T, V)) * 2.0
    head = rng.standard_normal((V, d)) * 0.3
    return P, F, Zt, head, H


def torch_loss(P, F, Zt, head, H, eps, theta, kind=0):
    """The same network from torch ops, for autograd."""
    T, d = F.shape
    hd = d // H
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    Ft, Ztt, Wh = (torch.tensor(a, dtype=torch.float64) for a in (F, Zt, head))
    inv = theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def norm(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + eps) * g

    def rope(x):
        a, b = x[..., : hd // 2], x[..., hd // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)

    n = norm(Ft, t["g_in"])
    if kind == 3:
        h = Ft + torch.nn.functional.silu(n @ t["w1"].T) @ t["w2"].T
    else:
        q = rope((n @ t["wq"].T).view(T, H, hd)).transpose(0, 1)
        k = rope((n @ t["wk"].T).view(T, H, hd)).transpose(0, 1)
        v = (n @ t["wv"].T).view(T, H, hd).transpose(0, 1)
        s = q @ k.transpose(1, 2) / np.sqrt(hd)
        s = s.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool), 1), float("-inf"))
        o = (torch.softmax(s, -1) @ v).transpose(0, 1).reshape(T, d)
        h = Ft + o @ t["wo"].T
        if kind == 2:
            b = norm(h, t["g_post"])
            h = h + (torch.nn.functional.silu(b @ t["wg"].T) * (b @ t["wu"].T)) @ t["wd"].T
    if kind in (1, 3):
        Wh = t["head"]
    Z = norm(h, t["g_last"]) @ Wh.T
    loss = -(torch.softmax(Ztt, -1) * torch.log_softmax(Z, -1)).sum()
    return loss, t, Z


@pytest.mark.parametrize("kind", [0, 1, 2, 3])
def test_gradients_match_reverse_mode_differentiation_of_a_library_forward(kind):
    P, F, Zt, head, H = problem(kind=kind)
    loss, G, inter = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0, kind)
    assert set(G) == set(TR.KIND_PARAMS[kind])
    tl, t, Z = torch_loss(P, F, Zt, head, H, 1e-6, 10000.0, kind)
    tl.backward()
    assert abs(loss - tl.item()) <= 1e-10 * abs(tl.item())
    np.testing.assert_allclose(inter["Z"], Z.detach().numpy(), rtol=0, atol=1e-11)
    for name in TR.KIND_PARAMS[kind]:
        want = t[name].grad.numpy()
        np.testing.assert_allclose(G[name], want, rtol=0, atol=1e-10 * max(1.0, np.abs(want).max()), err_msg=name)
        assert np.abs(want).max() > 1e-3, name            # a gradient that is really there


@pytest.mark.parametrize("kind", [0, 1, 2, 3])
def test_gradients_match_central_finite_differences(kind):
    P, F, Zt, head, H = problem(T=5, d=16, H=2, V=24, seed=3, kind=kind, ffn=24)
    _, G, _ = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0, kind)
    rng = np.random.default_rng(1)
    for name in TR.KIND_PARAMS[kind]:
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in P[name].shape)
            e = 1e-6
            old = P[name][idx]
            P[name][idx] = old + e
            lp, _, _ = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0, kind)
            P[name][idx] = old - e
            lm, _, _ = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0, kind)
            P[name][idx] = old
            fd = (lp - lm) / (2 * e)
            assert abs(fd - G[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, G[name][idx])


def test_loss_is_the_entropy_and_the_gradient_vanishes_when_draft_equals_target():
    """Eq. 3 is the cross entropy H(p, q) = H(p) + KL(p || q): its minimum over q is H(p), reached at
    q = p, where the gradient with respect to the logits (q - p) and hence every parameter is 0."""
    P, F, Zt, head, H = problem(seed=5)
    _, _, inter = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0)
    Z = inter["Z"]
    loss, G, _ = TR.loss_and_grads(P, F, Z + 3.0, head, H, 1e-6, 10000.0)   # a shift of the logits is the same p
    p = TR.softmax_rows(Z)
    assert abs(loss - float(-(p * np.log(p)).sum())) < 1e-10
    for name in TR.PARAMS:
        assert np.abs(G[name]).max() < 1e-12
    other, _, _ = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0)
    pt = TR.softmax_rows(Zt)
    assert other > float(-(pt * np.log(pt)).sum())


def test_adamw_matches_the_library_optimizer_and_its_first_step_closed_form():
    rng = np.random.default_rng(2)
    P = {k: rng.standard_normal((6, 6)) for k in TR.MATRICES}
    P["g_in"], P["g_last"] = rng.standard_normal(6), rng.standard_normal(6)
    t = {k: torch.tensor(v.copy(), dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    lr, wd = 3e-3, 0.05
    opt = torch.optim.AdamW([{"params": [t[k] for k in TR.MATRICES], "weight_decay": wd},
                             {"params": [t["g_in"], t["g_last"]], "weight_decay": 0.0}],
                            lr=lr, betas=(0.9, 0.999), eps=1e-8)
    M, V = TR.zeros_like_params(P), TR.zeros_like_params(P)
    P0 = {k: v.copy() for k, v in P.items()}
    for step in (1, 2, 3):
        G = {k: rng.standard_normal(P[k].shape) for k in TR.PARAMS}
        for k in TR.PARAMS:
            t[k].grad = torch.tensor(G[k])
        opt.step()
        TR.adamw_step(P, G, M, V, step, lr, weight_decay=wd)
        if step == 1:      # m/(1-b1) = g, v/(1-b2) = g^2: the step is lr * g / (|g| + eps) plus the decay
            for k in TR.PARAMS:
                w = wd if k in TR.MATRICES else 0.0
                want = P0[k] * (1 - lr * w) - lr * G[k] / (np.abs(G[k]) + 1e-8)
                np.testing.assert_allclose(P[k], want, rtol=0, atol=1e-14)
        for k in TR.PARAMS:
            np.testing.assert_allclose(P[k], t[k].detach().numpy(), rtol=0, atol=1e-13, err_msg=f"{k} step {step}")


@pytest.mark.parametrize("kind", [0, 1, 2, 3])
def test_the_training_graph_is_the_adapter_that_drafts(kind):
    """Draft logits of the training forward == the decode oracle's adapter + head run position by
    position through its cache (exact cache), for the same early features and weights, for each of
    the adapter architectures."""
    import dataclasses
    shape = dataclasses.replace(I.SHAPES["toy"], adapter=kind)
    W = I.gen_weights(shape, seed=4, alpha=0.6, own_head_copy=False)
    rng = np.random.default_rng(0)
    for k in (I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST, I.KIND_A_NORM_POST):
        if (k, -1) in W:
            W[(k, -1)] = (1.0 + 0.3 * rng.standard_normal(shape.d_model)).astype(np.float32)
    m = O.OracleModel(shape, W, 32)
    toks = I.gen_prompt(shape.vocab, 9, seed=6)
    F = m.shallow(toks, 0)
    want = m.head(np.concatenate([m.adapter(F[i:i + 1], i) for i in range(len(toks))]), 1)
    names = {"wq": I.KIND_A_WQ, "wk": I.KIND_A_WK, "wv": I.KIND_A_WV, "wo": I.KIND_A_WO, "g_in": I.KIND_A_NORM_IN,
             "g_last": I.KIND_A_NORM_LAST, "head": I.KIND_A_HEAD, "g_post": I.KIND_A_NORM_POST, "wg": I.KIND_A_WG,
             "wu": I.KIND_A_WU, "wd": I.KIND_A_WD, "w1": I.KIND_A_W1, "w2": I.KIND_A_W2}
    P = {k: W[(names[k], -1)].astype(np.float64) for k in TR.KIND_PARAMS[kind]}
    Zt = m.head(m.deep(F, 0), 0)
    _, _, inter = TR.loss_and_grads(P, F, Zt, W[(I.KIND_LM_HEAD, -1)].astype(np.float64), shape.n_heads,
                                    shape.rms_eps, shape.rope_theta, kind)
    np.testing.assert_allclose(inter["Z"], want, rtol=0, atol=1e-11)


def test_a_few_steps_lower_the_loss():
    P, F, Zt, head, H = problem(seed=7)
    M, V = TR.zeros_like_params(P), TR.zeros_like_params(P)
    losses = []
    for step in range(1, 9):
        loss, G, _ = TR.loss_and_grads(P, F, Zt, head, H, 1e-6, 10000.0)
        losses.append(loss)
        TR.adamw_step(P, G, M, V, step, 2e-3)
    assert all(b < a for a, b in zip(losses[:-1], losses[1:])), losses
