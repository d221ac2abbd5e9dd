"""GPU parity of the adapter's training step (Eq. 3 + AdamW) against the fp64 oracle
(oracle/adapter_training.py), through the C ABI.  The frozen model's outputs (early features and
target logits, whose parity the decode tests cover) are read back from the GPU and handed to the
oracle, so that what is compared here is the training arithmetic alone: draft logits, the loss, the
gradient of every adapter parameter, the AdamW update, and that the decode calls then draft with
the updated adapter."""
import dataclasses

import numpy as np
import pytest

from paper_2404_18911_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K", [(64, 64, 16), (70, 130, 37), (19, 1024, 256), (256, 96, 1000), (5, 7, 3)])
def test_fp32_contraction_in_every_operand_orientation(M, N, K):
    """C (+)= A.B on the matrix units for plain, transposed-A (the weight-gradient products) and
    transposed-B (the forward products) operands, ragged sizes; error bounded by fp32 accumulation."""
    from paper_2404_18911_amd import binding as B
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((K, N)).astype(np.float32)
    ref = A.astype(np.float64) @ Bm.astype(np.float64)
    bound = (np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64)) * 2.0 ** -21 + 1e-7
    At = np.ascontiguousarray(A.T)          # [K][M] in memory; At.T is A read with stride 1 along m
    Bt = np.ascontiguousarray(Bm.T)         # [N][K] in memory; Bt.T is B read with stride 1 along k
    for a, b in ((A, Bm), (At.T, Bm), (A, Bt.T), (At.T, Bt.T)):
        got = B.op_gemm_f32(a, b)
        assert np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / bound))
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    got = B.op_gemm_f32(A, Bm, C0)
    assert np.all(np.abs(got - (ref + C0)) <= bound + np.abs(C0) * 2.0 ** -23)


def _oracle_params(block, shape_or_d):
    from paper_2404_18911_amd import binding as B
    return {k: v.astype(np.float64).copy() for k, v in B.split_param_block(block, shape_or_d).items()}


TENSOR_KIND = {"wq": I.KIND_A_WQ, "wk": I.KIND_A_WK, "wv": I.KIND_A_WV, "wo": I.KIND_A_WO, "g_in": I.KIND_A_NORM_IN,
               "g_last": I.KIND_A_NORM_LAST, "head": I.KIND_A_HEAD, "g_post": I.KIND_A_NORM_POST, "wg": I.KIND_A_WG,
               "wu": I.KIND_A_WU, "wd": I.KIND_A_WD, "w1": I.KIND_A_W1, "w2": I.KIND_A_W2}


@pytest.mark.parametrize("name,n,hs,kind", [
    ("toy", 19, 1.0, 0), ("toy_bf16", 19, 1.0, 0), ("small_bf16", 37, 4.0, 0), ("toy", 1, 1.0, 0),
    ("toy_bf16", 300, 1.0, 0),      # two passes of the prompt kernels, keys beyond one block of threads
    ("toy", 261, 1.0, 0),
    # the other adapter architectures of Table 2: own head (trained too), whole block, two linear maps
    ("toy", 19, 1.0, 1), ("toy", 19, 1.0, 2), ("toy", 19, 1.0, 3),
    ("toy_bf16", 23, 1.0, 1), ("toy_bf16", 23, 1.0, 2), ("toy_bf16", 23, 1.0, 3), ("small_bf16", 37, 4.0, 2)])
def test_training_step_follows_the_oracle(name, n, hs, kind):
    from oracle import adapter_training as TR
    from paper_2404_18911_amd import binding as B
    from tests import parity as P
    shape = dataclasses.replace(I.SHAPES[name], adapter=kind)
    d, H = shape.d_model, shape.n_heads
    W = I.gen_weights(shape, seed=1, alpha=0.5, head_scale=hs, own_head_copy=False)
    rng = np.random.default_rng(0)
    for k in (I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST, I.KIND_A_NORM_POST):       # non-trivial gains
        if (k, -1) not in W:
            continue
        g = (1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32)
        W[(k, -1)] = g if shape.dtype == "f32" else I.f32_to_bf16_bits(g)
    head = W[(I.KIND_LM_HEAD, -1)]
    head64 = (I.bf16_bits_to_f32(head) if shape.dtype == "bf16" else head).astype(np.float64)
    max_seq = max(96, n + 24)
    kg = P.load_model(shape, W, max_seq, kv_page_tokens=32)
    kg.train_bind(max(40, n + 3))
    toks = I.gen_prompt(shape.vocab, n, seed=5)
    lr, wd = 1e-3, 0.05
    M64 = V64 = None
    dg_max = {}
    for step in (1, 2, 3):
        before = kg.train_read(B.TRAIN_PARAMETERS)
        loss = kg.train_step(toks, lr, weight_decay=wd)
        F = kg.train_read(B.TRAIN_FEATURES, n).astype(np.float64)
        Zt = kg.train_read(B.TRAIN_TARGET_LOGITS, n).astype(np.float64)
        Z = kg.train_read(B.TRAIN_DRAFT_LOGITS, n)
        G = B.split_param_block(kg.train_read(B.TRAIN_GRADIENTS), shape)
        after = B.split_param_block(kg.train_read(B.TRAIN_PARAMETERS), shape)
        Po = _oracle_params(before, shape)
        assert tuple(Po) == TR.KIND_PARAMS[kind]
        if M64 is None:
            M64, V64 = TR.zeros_like_params(Po), TR.zeros_like_params(Po)
        want_loss, Go, inter = TR.loss_and_grads(Po, F, Zt, head64, H, shape.rms_eps, shape.rope_theta, kind)
        zs = np.abs(inter["Z"]).max()
        assert np.abs(Z - inter["Z"]).max() <= 1e-5 * max(1.0, zs), "draft logits"
        assert abs(loss - want_loss) <= 1e-5 * abs(want_loss), (loss, want_loss)
        np.testing.assert_allclose(kg.train_read(B.TRAIN_ROW_LOSSES, n).sum(dtype=np.float64), loss, rtol=1e-6)
        for k in TR.KIND_PARAMS[kind]:
            gmax = np.abs(Go[k]).max()
            err = np.abs(G[k] - Go[k]).max()
            assert err <= 2e-4 * gmax + 1e-9, (k, step, err, gmax)
            if n > 1 or k not in ("wq", "wk"):      # one position attends to itself only: q and k get no gradient
                assert gmax > 0
        TR.adamw_step(Po, Go, M64, V64, step, lr, weight_decay=wd)
        for k in TR.KIND_PARAMS[kind]:
            # The update is lr * mhat / (sqrt(vhat) + eps), of size ~lr per element.  Where a gradient
            # element is tiny, its fp32 error dg moves that ratio by up to ~dg / sqrt(vhat); elsewhere
            # 0.1 % of lr catches a wrong sign, decay, moment or bias correction.
            dg_max[k] = np.maximum(dg_max.get(k, 0.0), np.abs(G[k] - Go[k]))
            vhat = V64[k] / (1.0 - 0.999 ** step)
            allowed = lr * (4.0 * dg_max[k] / (np.sqrt(vhat) + 1e-8) + 1e-3) + 2.0 ** -22 * np.abs(Po[k])
            assert np.all(np.abs(after[k] - Po[k]) <= allowed), (k, step, float(np.max(np.abs(after[k] - Po[k]) / allowed)))
        moved = max(np.abs(after[k].astype(np.float64) - _oracle_params(before, shape)[k]).max()
                    for k in TR.KIND_PARAMS[kind] if not k.startswith("g_"))
        assert moved > 0.5 * lr                       # the step really happened
    # the decode calls draft with the updated adapter (re-rounded to the storage type)
    W2 = dict(W)
    final = B.split_param_block(kg.train_read(B.TRAIN_PARAMETERS), shape)
    for key in TR.KIND_PARAMS[kind]:
        a = np.ascontiguousarray(final[key], dtype=np.float32)
        W2[(TENSOR_KIND[key], -1)] = a if shape.dtype == "f32" else I.f32_to_bf16_bits(a)
    if n > 1:
        from oracle import kangaroo_oracle as O
        shape2 = shape
        fol = P.Follow(1e-4 * max(1.0, hs) if shape.dtype == "f32" else 2e-2 * max(1.0, hs))
        P.follow_kangaroo(kg, O.OracleModel(shape2, W2, max_seq), I.gen_prompt(shape.vocab, 12), 16, 4, 0.0, fol)
    kg.close()


def test_training_lowers_the_loss_and_keeps_decoding_lossless():
    """Ten steps on one sequence: Eq. 3 goes down monotonically at a small step size, and greedy
    Kangaroo with the trained adapter still emits exactly the plain stream."""
    from paper_2404_18911_amd import binding as B
    from tests import parity as P
    shape = I.SHAPES["toy_bf16"]
    W = I.gen_weights(shape, seed=1, alpha=0.5, head_scale=8.0)
    kg = P.load_model(shape, W, 128, kv_page_tokens=32)
    kg.train_bind(64)
    toks = I.gen_prompt(shape.vocab, 48, seed=8)
    losses = [kg.train_step(toks, 2e-4) for _ in range(10)]
    assert all(b < a for a, b in zip(losses[:-1], losses[1:])), losses
    p, _ = B.make_params(eta=0.3, gamma=4)
    prompt = I.gen_prompt(shape.vocab, 16)
    plain, _ = kg.decode_plain(p, prompt, 40)
    out, _ = kg.generate(p, prompt, 40)
    assert out == plain
    kg.close()


def test_training_call_order_and_argument_errors():
    from paper_2404_18911_amd import binding as B
    from tests import parity as P
    shape = I.SHAPES["toy"]
    W = I.gen_weights(shape, seed=1)
    kg = P.load_model(shape, W, 64, kv_page_tokens=16)
    with pytest.raises(B.KangarooError) as ei:
        kg.train_step([1, 2, 3], 1e-3)
    assert ei.value.code == B.KG_ESTATE
    kg.train_bind(8)
    for bad in ([], list(range(9)), [shape.vocab]):
        with pytest.raises(B.KangarooError) as ei:
            kg.train_step(bad, 1e-3)
        assert ei.value.code == B.KG_EINVAL
    with pytest.raises(B.KangarooError) as ei:
        kg.train_step([1, 2], 1e-3, beta1=1.0)
    assert ei.value.code == B.KG_EINVAL
    # a freshly loaded adapter tensor makes the master copies stale: the binding is dropped
    kg.train_step([1, 2, 3], 1e-3)
    kg.load_tensor(I.KIND_A_WO, -1, W[(I.KIND_A_WO, -1)])
    with pytest.raises(B.KangarooError) as ei:
        kg.train_step([1, 2, 3], 1e-3)
    assert ei.value.code == B.KG_ESTATE
    kg.train_bind(8)
    kg.train_step([1, 2, 3], 1e-3)
    kg.close()


def test_gradient_accumulation_over_two_sequences():
    """Eq. 3 sums over every position it is given: two sequences accumulated into one gradient block
    give the sum of their gradients, and one AdamW update with that sum."""
    from oracle import adapter_training as TR
    from paper_2404_18911_amd import binding as B
    from tests import parity as P
    shape = I.SHAPES["toy_bf16"]
    d, H = shape.d_model, shape.n_heads
    W = I.gen_weights(shape, seed=2, alpha=0.5, head_scale=2.0)
    head64 = I.bf16_bits_to_f32(W[(I.KIND_LM_HEAD, -1)]).astype(np.float64)
    kg = P.load_model(shape, W, 96, kv_page_tokens=32)
    kg.train_bind(48)
    with pytest.raises(B.KangarooError) as ei:
        kg.train_apply(1e-3)
    assert ei.value.code == B.KG_ESTATE
    Po = _oracle_params(kg.train_read(B.TRAIN_PARAMETERS), d)
    total = None
    losses = []
    for seed, n in ((21, 33), (22, 17)):
        toks = I.gen_prompt(shape.vocab, n, seed=seed)
        losses.append(kg.train_accumulate(toks))
        F = kg.train_read(B.TRAIN_FEATURES, n).astype(np.float64)
        Zt = kg.train_read(B.TRAIN_TARGET_LOGITS, n).astype(np.float64)
        want, Go, _ = TR.loss_and_grads(Po, F, Zt, head64, H, shape.rms_eps, shape.rope_theta)
        assert abs(losses[-1] - want) <= 1e-5 * abs(want)
        total = Go if total is None else {k: total[k] + Go[k] for k in TR.PARAMS}
    G = B.split_param_block(kg.train_read(B.TRAIN_GRADIENTS), d)
    for k in TR.PARAMS:
        assert np.abs(G[k] - total[k]).max() <= 2e-4 * np.abs(total[k]).max(), k
    lr = 1e-3
    kg.train_apply(lr, weight_decay=0.0)
    after = B.split_param_block(kg.train_read(B.TRAIN_PARAMETERS), d)
    M64, V64 = TR.zeros_like_params(Po), TR.zeros_like_params(Po)
    TR.adamw_step(Po, total, M64, V64, 1, lr, weight_decay=0.0)
    for k in TR.PARAMS:
        dg = np.abs(G[k] - total[k])
        allowed = lr * (4.0 * dg / (np.abs(total[k]) + 1e-8) + 1e-3) + 2.0 ** -22 * np.abs(Po[k])
        assert np.all(np.abs(after[k] - Po[k]) <= allowed), k
    # the next step starts from its own gradient
    toks = I.gen_prompt(shape.vocab, 9, seed=23)
    kg.train_step(toks, lr)
    G2 = B.split_param_block(kg.train_read(B.TRAIN_GRADIENTS), d)
    assert np.abs(G2["wo"]).max() < 0.9 * np.abs(G["wo"]).max() or not np.allclose(G2["wo"], G["wo"])
    kg.close()


def test_cached_features_give_the_same_step_as_tokens():
    """The frozen model's part of a step (early features, target logits) computed once and handed
    back in gives bit for bit the gradient, loss and update of a step from tokens; epochs over the
    cached pair lower the loss without running the target model again."""
    from paper_2404_18911_amd import binding as B
    from tests import parity as P
    shape = I.SHAPES["toy_bf16"]
    W = I.gen_weights(shape, seed=3, alpha=0.5, head_scale=4.0)
    toks = I.gen_prompt(shape.vocab, 41, seed=9)
    kg = P.load_model(shape, W, 96, kv_page_tokens=32)
    kg.train_bind(48)
    F, Zt = kg.train_features(toks)
    loss_a = kg.train_accumulate(toks)
    Ga = kg.train_read(B.TRAIN_GRADIENTS).copy()
    np.testing.assert_array_equal(kg.train_read(B.TRAIN_FEATURES, 41), F.cpu().numpy())
    np.testing.assert_array_equal(kg.train_read(B.TRAIN_TARGET_LOGITS, 41), Zt.cpu().numpy())
    kg.train_apply(1e-3)
    Pa = kg.train_read(B.TRAIN_PARAMETERS).copy()
    # again from the cached pair, on a fresh copy of the same adapter
    for kind in (I.KIND_A_WQ, I.KIND_A_WK, I.KIND_A_WV, I.KIND_A_WO, I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST):
        kg.load_tensor(kind, -1, W[(kind, -1)])
    kg.train_bind(48)
    loss_b = kg.train_accumulate_features(F, Zt)
    assert loss_b == loss_a
    np.testing.assert_array_equal(kg.train_read(B.TRAIN_GRADIENTS), Ga)
    kg.train_apply(1e-3)
    np.testing.assert_array_equal(kg.train_read(B.TRAIN_PARAMETERS), Pa)
    losses = [loss_b]
    for _ in range(5):
        losses.append(kg.train_accumulate_features(F, Zt))
        kg.train_apply(2e-4)
    assert all(b < a for a, b in zip(losses[1:-1], losses[2:])), losses
    kg.close()
