"""Seeded synthetic inputs for the Kangaroo decode path: model shapes, random-init weights,
prompts and uniform random numbers.

This module holds no model arithmetic.  It only draws numbers and rounds them to the storage
type, so that the CPU oracle and the HIP library can be handed the very same bytes.

The adapter comes in the four architectures of Table 2 (ModelShape.adapter): 0 = input norm, one
multi-head attention, last norm, shared LM head (the paper's choice); 1 = the same with an LM head
of its own; 2 = one whole decoder block (attention, post norm, feed-forward) and the shared head;
3 = input norm, two d x d linear maps, last norm, own head.

Recipe (stands in for the Vicuna weights, the trained adapter and the Spec-Bench prompts of
Section 4.1, none of which are available): every matrix and the embedding are N(0, 0.02); norm
gains are 1; the o_proj / down_proj of the layers at and above the exit layer, and the adapter's
output projection (of whichever residual branch it has), are multiplied by alpha, which is the knob that moves the draft acceptance
rate.  Prompts are uniform token ids.  Element i of a tensor depends only on (seed, tensor id,
chunk), so tensors can be produced one at a time and in any order.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterator, List, Tuple

import numpy as np

_CHUNK = 1 << 22

# tensor kinds; the integer value is part of the seeding (and of the C-ABI's kg_tensor_kind)
KIND_EMBED = 0
KIND_LM_HEAD = 1
KIND_FINAL_NORM = 2
KIND_WQ = 3
KIND_WK = 4
KIND_WV = 5
KIND_WO = 6
KIND_WG = 7
KIND_WU = 8
KIND_WD = 9
KIND_NORM1 = 10
KIND_NORM2 = 11
KIND_A_WQ = 12
KIND_A_WK = 13
KIND_A_WV = 14
KIND_A_WO = 15
KIND_A_NORM_IN = 16
KIND_A_NORM_LAST = 17
KIND_A_HEAD = 18        # adapters 1 and 3: an LM head of the adapter's own
KIND_A_NORM_POST = 19   # adapter 2: norm before its feed-forward
KIND_A_WG = 20
KIND_A_WU = 21
KIND_A_WD = 22
KIND_A_W1 = 23          # adapter 3: the two linear maps
KIND_A_W2 = 24

ADAPTER_ATTN, ADAPTER_ATTN_HEAD, ADAPTER_LAYER, ADAPTER_MLP = range(4)

_NORM_KINDS = (KIND_FINAL_NORM, KIND_NORM1, KIND_NORM2, KIND_A_NORM_IN, KIND_A_NORM_LAST, KIND_A_NORM_POST)
_LAYER_KINDS = (KIND_WQ, KIND_WK, KIND_WV, KIND_WO, KIND_WG, KIND_WU, KIND_WD, KIND_NORM1, KIND_NORM2)


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Shape of a LLaMA-style decoder plus the exit layer l of Section 3.1."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    exit_layer: int
    dtype: str = "bf16"          # storage type of the weights: "f32" | "bf16"
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    kv: str = ""                 # storage type of the key/value cache: "f32" | "bf16" | "f16"; "" = f32 for f32 weights, f16 otherwise
    adapter: int = 0             # adapter architecture (Table 2): ADAPTER_ATTN .. ADAPTER_MLP

    @property
    def kv_dtype(self) -> str:
        return self.kv or ("f32" if self.dtype == "f32" else "f16")

    def layer_params(self) -> int:
        d, f = self.d_model, self.d_ffn
        return 4 * d * d + 3 * d * f + 2 * d

    def adapter_params(self) -> int:
        """Parameters the adapter adds to the model (Table 2's column)."""
        return sum(r * c for _, _, r, c in adapter_tensor_list(self))

    def head_params(self) -> int:
        return self.d_model * self.vocab

    def bytes_per_weight(self) -> int:
        return 4 if self.dtype == "f32" else 2


SHAPES: Dict[str, ModelShape] = {
    "toy": ModelShape("toy", 4, 256, 4, 64, 688, 1024, 1, "f32"),
    "toy_bf16": ModelShape("toy_bf16", 4, 256, 4, 64, 688, 1024, 1, "bf16"),
    "small_bf16": ModelShape("small_bf16", 6, 512, 4, 128, 1376, 4096, 2, "bf16"),
    "7b": ModelShape("7b", 32, 4096, 32, 128, 11008, 32000, 2, "bf16"),
    "13b": ModelShape("13b", 40, 5120, 40, 128, 13824, 32000, 2, "bf16"),
    "33b": ModelShape("33b", 60, 6656, 52, 128, 17920, 32000, 3, "bf16"),
}


def with_layers(shape: ModelShape, n_layers: int, name: str | None = None) -> ModelShape:
    """Same per-layer shape with fewer layers (used to bound oracle time in full-width tests)."""
    return dataclasses.replace(shape, n_layers=n_layers, name=name or f"{shape.name}_L{n_layers}")


def adapter_tensor_list(shape: ModelShape) -> List[Tuple[int, int, int, int]]:
    """(kind, -1, rows, cols) of the adapter's tensors for the shape's adapter architecture."""
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab
    attn = [(KIND_A_WQ, -1, d, d), (KIND_A_WK, -1, d, d), (KIND_A_WV, -1, d, d), (KIND_A_WO, -1, d, d)]
    norms = [(KIND_A_NORM_IN, -1, 1, d), (KIND_A_NORM_LAST, -1, 1, d)]
    if shape.adapter == ADAPTER_ATTN:
        return attn + norms
    if shape.adapter == ADAPTER_ATTN_HEAD:
        return attn + norms + [(KIND_A_HEAD, -1, v, d)]
    if shape.adapter == ADAPTER_LAYER:
        return attn + norms + [(KIND_A_NORM_POST, -1, 1, d), (KIND_A_WG, -1, f, d), (KIND_A_WU, -1, f, d),
                               (KIND_A_WD, -1, d, f)]
    if shape.adapter == ADAPTER_MLP:
        return [(KIND_A_W1, -1, d, d), (KIND_A_W2, -1, d, d)] + norms + [(KIND_A_HEAD, -1, v, d)]
    raise ValueError(f"unknown adapter architecture {shape.adapter}")


def tensor_list(shape: ModelShape) -> List[Tuple[int, int, int, int]]:
    """(kind, layer, rows, cols) of every tensor; layer is -1 for tensors outside the stack."""
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab
    out = [(KIND_EMBED, -1, v, d), (KIND_LM_HEAD, -1, v, d), (KIND_FINAL_NORM, -1, 1, d)]
    for i in range(shape.n_layers):
        out += [(KIND_WQ, i, d, d), (KIND_WK, i, d, d), (KIND_WV, i, d, d), (KIND_WO, i, d, d),
                (KIND_WG, i, f, d), (KIND_WU, i, f, d), (KIND_WD, i, d, f),
                (KIND_NORM1, i, 1, d), (KIND_NORM2, i, 1, d)]
    return out + adapter_tensor_list(shape)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16).  Inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_chunk(seed: int, tid: int, chunk: int, n: int) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=[seed, (tid << 24) | chunk]))
    return g.standard_normal(n, dtype=np.float32)


def _tensor_id(kind: int, layer: int) -> int:
    return (kind << 12) | (layer + 1)


def gen_tensor(shape: ModelShape, kind: int, layer: int, rows: int, cols: int, *, seed: int = 1,
               alpha: float = 0.1, std: float = 0.02, head_scale: float = 1.0,
               own_head_copy: bool = True, pool: ThreadPoolExecutor | None = None) -> np.ndarray:
    """One weight tensor in its storage type: float32 array, or uint16 bf16 bit patterns.

    head_scale multiplies the LM head (a test-only knob that sharpens the softmax so that the
    confidence threshold of Eq. 4 is crossed at varying draft lengths).  An adapter's own LM head
    starts as a copy of the model's (separate memory, same numbers: where its training would start),
    so that the adapters of Table 2 are compared at like acceptance; own_head_copy=False draws it
    independently instead.
    """
    n = rows * cols
    if kind in _NORM_KINDS:
        a = np.ones(n, dtype=np.float32)
    else:
        scale = std
        if (kind in (KIND_WO, KIND_WD) and layer >= shape.exit_layer) or kind in (KIND_A_WO, KIND_A_WD, KIND_A_W2):
            scale = std * alpha
        if kind in (KIND_LM_HEAD, KIND_A_HEAD):
            scale = std * head_scale
        tid = _tensor_id(KIND_LM_HEAD if (kind == KIND_A_HEAD and own_head_copy) else kind, layer)
        nchunk = (n + _CHUNK - 1) // _CHUNK
        a = np.empty(n, dtype=np.float32)

        def work(c):
            lo = c * _CHUNK
            hi = min(n, lo + _CHUNK)
            a[lo:hi] = _normal_chunk(seed, tid, c, hi - lo) * np.float32(scale)

        if pool is not None and nchunk > 1:
            list(pool.map(work, range(nchunk)))
        else:
            for c in range(nchunk):
                work(c)
    a = a.reshape(rows, cols) if rows > 1 else a.reshape(cols)
    if shape.dtype == "bf16":
        if pool is not None and n > _CHUNK:
            flat = a.reshape(-1)
            out = np.empty(n, dtype=np.uint16)

            def conv(c):
                lo = c * _CHUNK
                hi = min(n, lo + _CHUNK)
                out[lo:hi] = f32_to_bf16_bits(flat[lo:hi])

            list(pool.map(conv, range((n + _CHUNK - 1) // _CHUNK)))
            return out.reshape(a.shape)
        return f32_to_bf16_bits(a).reshape(a.shape)
    return a


def iter_weights(shape: ModelShape, *, seed: int = 1, alpha: float = 0.1, head_scale: float = 1.0,
                 std: float = 0.02, threads: int = 8, own_head_copy: bool = True) -> Iterator[Tuple[int, int, np.ndarray]]:
    """Yield (kind, layer, array) for every tensor of the model, one at a time."""
    with ThreadPoolExecutor(max_workers=threads) as pool:
        for kind, layer, rows, cols in tensor_list(shape):
            yield kind, layer, gen_tensor(shape, kind, layer, rows, cols, seed=seed, alpha=alpha, std=std,
                                          head_scale=head_scale, own_head_copy=own_head_copy, pool=pool)


def gen_weights(shape: ModelShape, *, seed: int = 1, alpha: float = 0.1, head_scale: float = 1.0,
                std: float = 0.02, threads: int = 8, own_head_copy: bool = True) -> Dict[Tuple[int, int], np.ndarray]:
    """All tensors in host memory, keyed by (kind, layer)."""
    return {(k, l): a for k, l, a in iter_weights(shape, seed=seed, alpha=alpha, std=std, head_scale=head_scale,
                                                  threads=threads, own_head_copy=own_head_copy)}


def gen_prompt(vocab: int, n: int, seed: int = 2) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=[seed, 0x70726F6D]))
    return g.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


# purposes of the per-position uniforms used by sampling-mode decoding
U_DRAFT, U_ACCEPT, U_RESAMPLE = 0, 1, 2


def gen_uniforms(n_positions: int, seed: int = 3) -> np.ndarray:
    """float32 [n_positions, 3] in [0, 1): u = (r >> 8) * 2^-24 from one Philox word per
    (absolute position, purpose).  Indexing by position keeps the stream independent of the
    control flow of the decoder."""
    g = np.random.Generator(np.random.Philox(key=[seed, 0x756E6966]))
    r = g.integers(0, 1 << 32, size=(n_positions, 3), dtype=np.uint64)
    return ((r >> np.uint64(8)).astype(np.float64) * 2.0 ** -24).astype(np.float32)
