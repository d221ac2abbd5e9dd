"""Pins for the oracle's model arithmetic (oracle/kangaroo_ref.c) against things that are not
the oracle: a few-line fp64 composition of library matmul/softmax over the whole sequence
(no cache), closed forms and invariants of the pieces, and Table 2's parameter counts."""
import ctypes
import os

import numpy as np
import pytest
import torch

from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _w64(shape, W, kind, layer=-1):
    a = W[(kind, layer)]
    if shape.dtype == "bf16":
        a = I.bf16_bits_to_f32(a)
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def torch_forward(shape, W, tokens, lo_hi=None, with_adapter=False, cache=None):
    """Whole-sequence forward without a cache, written from the textbook definitions with
    torch fp64 matmul / softmax.  Returns (early features, final hidden, target logits,
    draft logits)."""
    d, H, hd = shape.d_model, shape.n_heads, shape.head_dim
    T = len(tokens)
    pos = torch.arange(T, dtype=torch.float64)
    inv = shape.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang), torch.sin(ang)                        # [T, hd/2]

    def norm(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + shape.rms_eps) * g

    def rope(x):                                                     # [T, H, hd]
        a, b = x[..., : hd // 2], x[..., hd // 2:]
        return torch.cat([a * cos[:, None] - b * sin[:, None], b * cos[:, None] + a * sin[:, None]], -1)

    def attn(x, g, wq, wk, wv, wo):
        a = norm(x, g)
        q = rope((a @ wq.T).view(T, H, hd)).transpose(0, 1)          # [H, T, hd]
        k = rope((a @ wk.T).view(T, H, hd)).transpose(0, 1)
        v = (a @ wv.T).view(T, H, hd).transpose(0, 1)
        if cache is not None:               # a cache that stores rotated keys and values in 2 bytes
            k = k.to(torch.float32).to(cache).to(torch.float64)
            v = v.to(torch.float32).to(cache).to(torch.float64)
        s = q @ k.transpose(1, 2) / np.sqrt(hd)
        s = s.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool), 1), float("-inf"))
        o = (torch.softmax(s, -1) @ v).transpose(0, 1).reshape(T, d)
        return x + o @ wo.T

    x = _w64(shape, W, I.KIND_EMBED)[torch.as_tensor(np.asarray(tokens, dtype=np.int64))]
    f = None
    for i in range(shape.n_layers):
        x = attn(x, _w64(shape, W, I.KIND_NORM1, i), _w64(shape, W, I.KIND_WQ, i), _w64(shape, W, I.KIND_WK, i),
                 _w64(shape, W, I.KIND_WV, i), _w64(shape, W, I.KIND_WO, i))
        b = norm(x, _w64(shape, W, I.KIND_NORM2, i))
        g = b @ _w64(shape, W, I.KIND_WG, i).T
        u = b @ _w64(shape, W, I.KIND_WU, i).T
        x = x + (torch.nn.functional.silu(g) * u) @ _w64(shape, W, I.KIND_WD, i).T
        if i == shape.exit_layer - 1:
            f = x
    head = _w64(shape, W, I.KIND_LM_HEAD)
    logits = norm(x, _w64(shape, W, I.KIND_FINAL_NORM)) @ head.T
    # the adapter, in the architecture of Table 2 the shape names
    if shape.adapter == I.ADAPTER_MLP:
        u = norm(f, _w64(shape, W, I.KIND_A_NORM_IN)) @ _w64(shape, W, I.KIND_A_W1).T
        h = f + torch.nn.functional.silu(u) @ _w64(shape, W, I.KIND_A_W2).T
    else:
        h = attn(f, _w64(shape, W, I.KIND_A_NORM_IN), _w64(shape, W, I.KIND_A_WQ), _w64(shape, W, I.KIND_A_WK),
                 _w64(shape, W, I.KIND_A_WV), _w64(shape, W, I.KIND_A_WO))
        if shape.adapter == I.ADAPTER_LAYER:
            b = norm(h, _w64(shape, W, I.KIND_A_NORM_POST))
            h = h + (torch.nn.functional.silu(b @ _w64(shape, W, I.KIND_A_WG).T)
                     * (b @ _w64(shape, W, I.KIND_A_WU).T)) @ _w64(shape, W, I.KIND_A_WD).T
    dhead = _w64(shape, W, I.KIND_A_HEAD) if shape.adapter in (I.ADAPTER_ATTN_HEAD, I.ADAPTER_MLP) else head
    dlogits = norm(h, _w64(shape, W, I.KIND_A_NORM_LAST)) @ dhead.T
    return f.numpy(), x.numpy(), logits.numpy(), dlogits.numpy()


@pytest.mark.parametrize("name,kv,adapter", [("toy", "", 0), ("toy_bf16", "", 0), ("toy_bf16", "bf16", 0), ("toy_bf16", "f16", 0),
                                             ("toy", "", 1), ("toy", "", 2), ("toy", "", 3),
                                             ("toy_bf16", "", 2), ("toy_bf16", "f16", 3)])
def test_incremental_decode_matches_whole_sequence_library_forward(name, kv, adapter):
    """Oracle run token by token through its caches == library forward of the whole sequence.
    A dropped residual, a wrong RoPE pairing or sign, a transposed operand, a cache indexing
    slip or a wrong widening of bf16 all break this.  kv = "": the exact cache of the plain
    definition; "bf16" / "f16": the oracle's optional rounding of cached keys and values against
    the same rounding applied inside the library forward."""
    import dataclasses
    shape = dataclasses.replace(I.SHAPES[name], kv=kv, adapter=adapter)
    cache = {"": None, "bf16": torch.bfloat16, "f16": torch.float16}[kv]
    # non-trivial gains so that a missing or misplaced gain is caught too; an own head that is not
    # the model's, so that a draft head read from the wrong matrix is caught
    W = I.gen_weights(shape, seed=5, alpha=0.7, own_head_copy=False)
    rng = np.random.default_rng(0)
    for (k, l), a in list(W.items()):
        if k in (I.KIND_FINAL_NORM, I.KIND_NORM1, I.KIND_NORM2, I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST,
                 I.KIND_A_NORM_POST):
            g = (1.0 + 0.3 * rng.standard_normal(a.shape)).astype(np.float32)
            W[(k, l)] = g if shape.dtype == "f32" else I.f32_to_bf16_bits(g)
    toks = I.gen_prompt(shape.vocab, 11, seed=9)
    f_ref, x_ref, z_ref, dz_ref = torch_forward(shape, W, toks, cache=cache)
    m = O.OracleModel(shape, W, 32, exact_cache=cache is None)
    # mixed row counts: 4 rows, then 1, 1, 3, 2
    cuts = [0, 4, 5, 6, 9, 11]
    fs, xs, hs = [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        f = m.shallow(toks[a:b], a)
        fs.append(f)
        hs.append(m.adapter(f, a))
        xs.append(m.deep(f, a))
    f, x, h = np.concatenate(fs), np.concatenate(xs), np.concatenate(hs)
    np.testing.assert_allclose(f, f_ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(x, x_ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(m.head(x, 0), z_ref, rtol=0, atol=1e-11)
    np.testing.assert_allclose(m.head(h, 1), dz_ref, rtol=0, atol=1e-11)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def test_matvec_widens_bf16_exactly_and_is_not_transposed():
    rng = np.random.default_rng(1)
    Wf = rng.standard_normal((7, 13)).astype(np.float32)
    bits = I.f32_to_bf16_bits(Wf)
    x = rng.standard_normal((3, 13))
    y = np.empty((3, 7))
    O.lib().ko_matvec(bits.ctypes.data, 1, 7, 13, _dp(x), 3, _dp(y))
    ref = x @ I.bf16_bits_to_f32(bits).astype(np.float64).T
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)
    O.lib().ko_matvec(Wf.ctypes.data, 0, 7, 13, _dp(x), 3, _dp(y))
    np.testing.assert_allclose(y, x @ Wf.astype(np.float64).T, rtol=0, atol=1e-13)


def test_bf16_rounding_of_the_input_generator_is_nearest_even():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0)
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.0],
                 dtype=np.float32)
    back = I.bf16_bits_to_f32(I.f32_to_bf16_bits(a))
    np.testing.assert_array_equal(back, np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -3.0], dtype=np.float32))
    t = torch.from_numpy(np.random.default_rng(2).standard_normal(4096).astype(np.float32))
    ref = t.to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(I.bf16_bits_to_f32(I.f32_to_bf16_bits(t.numpy())), ref)


def test_cache_rounding_is_nearest_with_ties_to_even():
    """bfloat16 keeps 8 significant bits: neighbours of 1 are 2^-7 apart.  Exact halves go to the
    even neighbour, anything past the half goes up, representable values stay."""
    r = O.lib().ko_round_bf16
    e = 2.0 ** -7
    assert r(1.0 + e / 2) == 1.0                       # tie, lower neighbour even
    assert r(1.0 + 3 * e / 2) == 1.0 + 2 * e           # tie, upper neighbour even
    assert r(-(1.0 + e / 2)) == -1.0 and r(-(1.0 + 3 * e / 2)) == -(1.0 + 2 * e)
    assert r(1.0 + e / 2 + 2.0 ** -20) == 1.0 + e      # just past the half
    assert r(1.0 + e / 2 - 2.0 ** -20) == 1.0
    for v in (0.0, 1.0, -3.5, 1.0 + e, 2.0 ** -30, 448.0):
        assert r(v) == v
    # a double just above a float tie: float conversion comes first and lands on the tie (2^-40 is
    # below float resolution at 1), which then goes to even
    assert r(1.0 + e / 2 + 2.0 ** -40) == 1.0


def test_half_precision_cache_rounding_is_the_library_conversion():
    """The oracle's optional rounding of cached values to IEEE half precision (written from the
    format's definition: 11 significant bits, subnormals below 2^-14, ties to even) against numpy's
    float32 -> float16 conversion on random, tie, subnormal, tiny and near-overflow values."""
    r = O.lib().ko_round_f16
    rng = np.random.default_rng(8)
    vals = np.concatenate([rng.standard_normal(4000) * 3.0, rng.standard_normal(500) * 1e-5, rng.standard_normal(500) * 2e4,
                           [0.0, 1.0, -1.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -22,
                            2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -26, 65504.0, 65519.9, -65519.9]])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float32).astype(np.float16).astype(np.float64)
    got = np.array([r(float(v)) for v in vals])
    np.testing.assert_array_equal(got, want)
    assert r(1.0 + 2.0 ** -11) == 1.0 and r(1.0 + 3 * 2.0 ** -11) == 1.0 + 2.0 ** -9      # ties to even
    assert r(65520.0) == np.inf and r(-70000.0) == -np.inf


def test_rmsnorm_unit_gain_gives_unit_rms():
    x = np.random.default_rng(3).standard_normal(256) * 5.0
    g = np.ones(256, dtype=np.float32)
    y = np.empty(256)
    O.lib().ko_rmsnorm(_dp(x), g.ctypes.data, 0, 256, 0.0, _dp(y))
    assert abs(np.sqrt(np.mean(y * y)) - 1.0) < 1e-14
    # direction preserved, gain applied element-wise
    g2 = np.linspace(0.5, 2.0, 256).astype(np.float32)
    y2 = np.empty(256)
    O.lib().ko_rmsnorm(_dp(x), g2.ctypes.data, 0, 256, 1e-6, _dp(y2))
    np.testing.assert_allclose(y2, x / np.sqrt(np.mean(x * x) + 1e-6) * g2, rtol=1e-14)


def test_rope_preserves_norm_and_depends_on_relative_position_only():
    rng = np.random.default_rng(4)
    q0, k0 = rng.standard_normal(64), rng.standard_normal(64)

    def rot(v, p):
        w = v.copy()
        O.lib().ko_rope(_dp(w), 64, p, 10000.0)
        return w

    assert abs(np.linalg.norm(rot(q0, 17)) - np.linalg.norm(q0)) < 1e-13
    np.testing.assert_allclose(rot(q0, 0), q0, atol=0)
    a = rot(q0, 9) @ rot(k0, 4)
    b = rot(q0, 105) @ rot(k0, 100)
    assert abs(a - b) < 1e-12
    # and it is a rotation by a positive angle in each (i, i+hd/2) plane: pair 0 turns by `pos` radians
    e = np.zeros(64)
    e[0] = 1.0
    r = rot(e, 1)
    assert abs(r[0] - np.cos(1.0)) < 1e-15 and abs(r[32] - np.sin(1.0)) < 1e-15


def test_softmax_and_single_key_attention():
    z = np.array([1.0, 2.0, 3.0, -1000.0])
    O.lib().ko_softmax(_dp(z), 4)
    assert abs(z.sum() - 1.0) < 1e-15 and z[3] == 0.0
    np.testing.assert_allclose(z[:3], np.exp([1.0, 2.0, 3.0]) / np.exp([1.0, 2.0, 3.0]).sum(), rtol=1e-15)
    rng = np.random.default_rng(5)
    q, K, V = rng.standard_normal(8), rng.standard_normal((1, 8)), rng.standard_normal((1, 8))
    o = np.empty(8)
    O.lib().ko_attend(_dp(q), _dp(K), _dp(V), 1, 8, 8, _dp(o))
    np.testing.assert_allclose(o, V[0], atol=0)
    # equal scores -> plain average of the values
    K2 = np.zeros((3, 8))
    V2 = rng.standard_normal((3, 8))
    O.lib().ko_attend(_dp(q), _dp(K2), _dp(V2), 3, 8, 8, _dp(o))
    np.testing.assert_allclose(o, V2.mean(0), atol=1e-15)


def test_adapter_and_model_sizes_match_table2():
    """The adapter is four bias-free d x d projections and two gain vectors sharing the LM head;
    its size and the ablation rows' sizes are the closed forms Table 2 prints (in millions)."""
    gold = {}
    for line in open(os.path.join(GOLD, "table2_param_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        gold[k] = float(v)
    s = I.SHAPES["7b"]
    d, f, V = s.d_model, s.d_ffn, s.vocab
    assert s.adapter_params() == 4 * d * d + 2 * d == 67_117_056
    # what the generator actually emits for the adapter
    n = sum(r * c for k, l, r, c in I.tensor_list(s) if k >= I.KIND_A_WQ)
    assert n == s.adapter_params()
    assert round(s.adapter_params() / 1e6) == gold["kangaroo"]
    assert round((s.adapter_params() + d * V) / 1e6) == gold["kangaroo_plus_head"]
    assert round((4 * d * d + 3 * d * f + 3 * d) / 1e6) == gold["one_layer_transformer"]
    assert round((2 * d * d + d * V + 2 * d) / 1e6) == gold["mlp_only"]
    # the tensors the generator emits (and both implementations load) for each architecture
    import dataclasses
    for kind, row in ((I.ADAPTER_ATTN, "kangaroo"), (I.ADAPTER_ATTN_HEAD, "kangaroo_plus_head"),
                      (I.ADAPTER_LAYER, "one_layer_transformer"), (I.ADAPTER_MLP, "mlp_only")):
        assert round(dataclasses.replace(s, adapter=kind).adapter_params() / 1e6) == gold[row]
    medusa = 4 * (d * d + d * V)
    assert round(medusa / 1e6) == gold["medusa"]
    assert round(100 * s.adapter_params() / medusa, 1) == gold["share_percent"]
    assert round(100 * (1 - 67 / 591), 1) == gold["fewer_percent"]
    # model sizes used for the bandwidth roofline
    total = s.n_layers * s.layer_params() + 2 * d * V + d
    assert total == 6_738_415_616
