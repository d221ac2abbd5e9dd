"""ctypes binding of libkangaroo (include/kangaroo.h): same names, argument marshalling only.

PyTorch is used for device memory and the stream; every step of the decode path runs in the
library's HIP kernels.  Importing this module fails loudly if the library cannot be loaded.
"""
from __future__ import annotations

import ctypes
import os
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

KG_MAX_ROWS = 8
KG_OK, KG_EINVAL, KG_ESTATE, KG_ENOSPC, KG_EHIP, KG_ENOMEM = 0, -1, -2, -3, -4, -5


class kg_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                                            "exit_layer", "dtype", "kv_dtype")] + \
               [("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float)] + \
               [(n, ctypes.c_int) for n in ("max_seq", "gamma_max", "kv_page_tokens", "adapter_kind")]


class kg_params(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("temperature", ctypes.c_float), ("eta", ctypes.c_float),
                ("gamma", ctypes.c_int), ("uniforms", ctypes.POINTER(ctypes.c_float)),
                ("n_uniform_positions", ctypes.c_int), ("seed", ctypes.c_uint64)]


class kg_stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("rounds", "drafted", "accepted", "emitted")] + \
               [("s_hist", ctypes.c_int * (KG_MAX_ROWS + 1))] + \
               [(n, ctypes.c_int) for n in ("draft_steps", "verify_calls", "plain_steps")] + \
               [(n, ctypes.c_double) for n in ("t_draft_s", "t_verify_s", "t_total_s", "bytes_draft", "bytes_shallow",
                                               "bytes_verify")]


class kg_profile(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_longlong * 5), ("seconds", ctypes.c_double * 5), ("bytes", ctypes.c_double * 5)]


# every symbol include/kangaroo.h declares
class kg_train_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay")]


TRAIN_FEATURES, TRAIN_TARGET_LOGITS, TRAIN_DRAFT_LOGITS, TRAIN_GRADIENTS, TRAIN_PARAMETERS, TRAIN_ROW_LOSSES = range(6)

SYMBOLS = ["kg_stats_cr", "kg_stats_ctar", "kg_create", "kg_workspace_bytes", "kg_bind", "kg_load_tensor", "kg_set_page_order", "kg_prefill",
           "kg_draft_step", "kg_verify", "kg_accept", "kg_generate", "kg_decode_plain", "kg_plain_step",
           "kg_read_logits", "kg_read_feature", "kg_read_kv", "kg_get_state", "kg_set_profiling", "kg_get_profile", "kg_reset", "kg_last_error",
           "kg_destroy", "kg_op_packed_bytes", "kg_op_work_bytes", "kg_op_pack", "kg_op_linear", "kg_op_linear_static", "kg_op_linear_valu", "kg_op_philox_words", "kg_op_stream_read",
           "kg_train_workspace_bytes", "kg_train_bind", "kg_train_step", "kg_train_accumulate", "kg_train_apply", "kg_train_features", "kg_train_accumulate_features",
           "kg_train_read", "kg_op_gemm_f32", "kg_op_tile_pos"]

_lib = None


def lib() -> ctypes.CDLL:
    """Load libkangaroo.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        _build.build(force=True)
    L = ctypes.CDLL(path)
    vp, ip, fp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
    szp, pp = ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(kg_params)
    L.kg_stats_cr.argtypes = [ctypes.POINTER(kg_stats), ctypes.POINTER(ctypes.c_double)]
    L.kg_stats_ctar.argtypes = [ctypes.POINTER(kg_stats), ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    L.kg_create.argtypes = [ctypes.POINTER(kg_config), ctypes.POINTER(vp)]
    L.kg_workspace_bytes.argtypes = [vp, szp, szp, szp]
    L.kg_bind.argtypes = [vp, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    L.kg_load_tensor.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t]
    L.kg_set_page_order.argtypes = [vp, ip, ctypes.c_int]
    L.kg_prefill.argtypes = [vp, pp, ip, ctypes.c_int, ip]
    L.kg_draft_step.argtypes = [vp, pp, ip, fp, ip]
    L.kg_verify.argtypes = [vp, pp, ip, ip]
    L.kg_accept.argtypes = [vp, pp, ip, ip]
    L.kg_generate.argtypes = [vp, pp, ip, ctypes.c_int, ctypes.c_int, ip, ip, ctypes.POINTER(kg_stats)]
    L.kg_decode_plain.argtypes = L.kg_generate.argtypes
    L.kg_plain_step.argtypes = [vp, pp, ctypes.c_int32, ip]
    L.kg_read_logits.argtypes = [vp, ctypes.c_int, ctypes.c_int, fp]
    L.kg_read_feature.argtypes = [vp, ctypes.c_int, fp]
    L.kg_read_kv.argtypes = [vp, ctypes.c_int, ctypes.c_int, fp, fp]
    L.kg_get_state.argtypes = [vp, ip, ip, ip, ip]
    L.kg_set_profiling.argtypes = [vp, ctypes.c_int]
    L.kg_get_profile.argtypes = [vp, ctypes.POINTER(kg_profile)]
    L.kg_reset.argtypes = [vp]
    L.kg_last_error.argtypes = [vp]
    L.kg_last_error.restype = ctypes.c_char_p
    L.kg_destroy.argtypes = [vp]
    L.kg_destroy.restype = None
    L.kg_op_packed_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.kg_op_packed_bytes.restype = ctypes.c_size_t
    L.kg_op_work_bytes.argtypes = [ctypes.c_int]
    L.kg_op_work_bytes.restype = ctypes.c_size_t
    L.kg_op_pack.argtypes = [ctypes.c_int, vp, ctypes.c_int, ctypes.c_int, vp, vp]
    L.kg_op_linear.argtypes = [ctypes.c_int, vp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_int, vp, vp, vp]
    L.kg_op_linear_static.argtypes = [ctypes.c_int, vp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_int, vp, vp]
    L.kg_op_linear_valu.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, vp, vp]
    L.kg_op_philox_words.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int, vp, vp]
    L.kg_op_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    L.kg_train_workspace_bytes.argtypes = [vp, ctypes.c_int, szp]
    L.kg_train_bind.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int]
    L.kg_train_step.argtypes = [vp, ctypes.POINTER(kg_train_params), ip, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    L.kg_train_accumulate.argtypes = [vp, ip, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    L.kg_train_apply.argtypes = [vp, ctypes.POINTER(kg_train_params)]
    L.kg_train_features.argtypes = [vp, ip, ctypes.c_int, vp, vp]
    L.kg_train_accumulate_features.argtypes = [vp, vp, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    L.kg_train_read.argtypes = [vp, ctypes.c_int, fp, ctypes.c_size_t]
    L.kg_op_tile_pos.argtypes = [ctypes.c_int, ctypes.c_int]
    L.kg_op_tile_pos.restype = ctypes.c_int
    L.kg_op_gemm_f32.argtypes = [vp, ctypes.c_long, ctypes.c_long, vp, ctypes.c_long, ctypes.c_long, vp, ctypes.c_long,
                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
    _lib = L
    return L


def stats_cr(st: kg_stats) -> float:
    out = ctypes.c_double()
    if lib().kg_stats_cr(ctypes.byref(st), ctypes.byref(out)) != KG_OK:
        raise ValueError("no rounds")
    return out.value


def stats_ctar(st: kg_stats, w: int) -> float:
    out = ctypes.c_double()
    if lib().kg_stats_ctar(ctypes.byref(st), w, ctypes.byref(out)) != KG_OK:
        raise ValueError("no rounds or bad window")
    return out.value


class KangarooError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libkangaroo error {code}: {msg}")
        self.code = code


def make_config(shape, max_seq: int, gamma_max: int = 6, kv_page_tokens: int = 128) -> kg_config:
    return kg_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                     shape.exit_layer, 0 if shape.dtype == "f32" else 1, {"f32": 0, "bf16": 1, "f16": 2}[shape.kv_dtype],
                     shape.rms_eps, shape.rope_theta,
                     max_seq, gamma_max, kv_page_tokens, getattr(shape, "adapter", 0))


def make_params(mode: int = 0, temperature: float = 1.0, eta: float = 0.6, gamma: int = 6,
                uniforms: Optional[np.ndarray] = None, seed: int = 0) -> Tuple[kg_params, object]:
    """Returns (params, keepalive).  Sampling mode draws from the device generator keyed by `seed`
    unless a table of uniform numbers is given."""
    p = kg_params(mode, temperature, eta, gamma, None, 0, seed)
    keep = None
    if uniforms is not None:
        keep = np.ascontiguousarray(uniforms, dtype=np.float32)
        p.uniforms = keep.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        p.n_uniform_positions = keep.shape[0]
    return p, keep


class Kangaroo:
    """A bound context: device buffers are torch tensors owned by this object."""

    def __init__(self, shape, max_seq: int, gamma_max: int = 6, kv_page_tokens: int = 128, device: str = "cuda:0"):
        import torch
        self._torch = torch
        self.shape = shape
        self.L = lib()
        self.cfg = make_config(shape, max_seq, gamma_max, kv_page_tokens)
        self.h = ctypes.c_void_p()
        rc = self.L.kg_create(ctypes.byref(self.cfg), ctypes.byref(self.h))
        if rc != KG_OK:
            raise KangarooError(rc, "kg_create rejected the configuration")
        wb, kb, sb = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        self._chk(self.L.kg_workspace_bytes(self.h, ctypes.byref(wb), ctypes.byref(kb), ctypes.byref(sb)))
        self.weight_bytes, self.kv_bytes, self.scratch_bytes = wb.value, kb.value, sb.value
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.arena = torch.empty(wb.value, dtype=torch.uint8, device=self.device)
        self.kv = torch.empty(kb.value, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(sb.value, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.page_order = list(range((max_seq + kv_page_tokens - 1) // kv_page_tokens))
        self._chk(self.L.kg_bind(self.h, self.arena.data_ptr(), wb.value, self.kv.data_ptr(), kb.value,
                                 self.scratch.data_ptr(), sb.value, self.stream.cuda_stream))

    def _chk(self, rc: int) -> None:
        if rc != KG_OK:
            raise KangarooError(rc, self.L.kg_last_error(self.h).decode())

    def close(self) -> None:
        if self.h:
            self._torch.cuda.synchronize(self.device)
            self.L.kg_destroy(self.h)
            self.h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights
    def load_tensor(self, kind: int, layer: int, host: np.ndarray) -> None:
        torch = self._torch
        t = torch.from_numpy(host.view(np.int16) if host.dtype == np.uint16 else host).to(self.device)
        self._chk(self.L.kg_load_tensor(self.h, kind, layer, t.data_ptr(), host.size))

    def load_weights(self, tensors: Iterable[Tuple[int, int, np.ndarray]]) -> None:
        for kind, layer, a in tensors:
            self.load_tensor(kind, layer, a)

    def set_page_order(self, perm: Sequence[int]) -> None:
        a = np.ascontiguousarray(perm, dtype=np.int32)
        self._chk(self.L.kg_set_page_order(self.h, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(a)))
        self.page_order = a.tolist()

    # -- stepwise calls
    def prefill(self, params: kg_params, prompt: Sequence[int]) -> int:
        a = np.ascontiguousarray(prompt, dtype=np.int32)
        out = ctypes.c_int32()
        self._chk(self.L.kg_prefill(self.h, ctypes.byref(params), a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    len(a), ctypes.byref(out)))
        return out.value

    def draft_step(self, params: kg_params) -> Tuple[int, float, bool]:
        tok, conf, stop = ctypes.c_int32(), ctypes.c_float(), ctypes.c_int32()
        self._chk(self.L.kg_draft_step(self.h, ctypes.byref(params), ctypes.byref(tok), ctypes.byref(conf),
                                       ctypes.byref(stop)))
        return tok.value, conf.value, bool(stop.value)

    def verify(self, params: kg_params) -> List[int]:
        buf = (ctypes.c_int32 * KG_MAX_ROWS)()
        n = ctypes.c_int32()
        self._chk(self.L.kg_verify(self.h, ctypes.byref(params), buf, ctypes.byref(n)))
        return list(buf[: n.value])

    def accept(self, params: kg_params) -> List[int]:
        buf = (ctypes.c_int32 * KG_MAX_ROWS)()
        n = ctypes.c_int32()
        self._chk(self.L.kg_accept(self.h, ctypes.byref(params), buf, ctypes.byref(n)))
        return list(buf[: n.value])

    def plain_step(self, params: kg_params, token: int) -> int:
        out = ctypes.c_int32()
        self._chk(self.L.kg_plain_step(self.h, ctypes.byref(params), int(token), ctypes.byref(out)))
        return out.value

    # -- whole loops
    def _loop(self, fn, params, prompt, max_new):
        a = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(max(1, max_new), dtype=np.int32)
        n = ctypes.c_int32()
        st = kg_stats()
        self._chk(fn(self.h, ctypes.byref(params), a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(a), max_new,
                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), ctypes.byref(n), ctypes.byref(st)))
        return out[: n.value].tolist(), st

    def generate(self, params: kg_params, prompt: Sequence[int], max_new: int):
        return self._loop(self.L.kg_generate, params, prompt, max_new)

    def decode_plain(self, params: kg_params, prompt: Sequence[int], max_new: int):
        return self._loop(self.L.kg_decode_plain, params, prompt, max_new)

    # -- read-backs
    def read_logits(self, which: int, row: int) -> np.ndarray:
        out = np.empty(self.shape.vocab, dtype=np.float32)
        self._chk(self.L.kg_read_logits(self.h, which, row, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
        return out

    def read_feature(self, row: int) -> np.ndarray:
        out = np.empty(self.shape.d_model, dtype=np.float32)
        self._chk(self.L.kg_read_feature(self.h, row, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
        return out

    def read_kv(self, slot: int, pos: int) -> Tuple[np.ndarray, np.ndarray]:
        k = np.empty(self.shape.d_model, dtype=np.float32)
        v = np.empty(self.shape.d_model, dtype=np.float32)
        fp = ctypes.POINTER(ctypes.c_float)
        self._chk(self.L.kg_read_kv(self.h, slot, pos, k.ctypes.data_as(fp), v.ctypes.data_as(fp)))
        return k, v

    def state(self) -> Tuple[int, int, int, int]:
        v = [ctypes.c_int32() for _ in range(4)]
        self._chk(self.L.kg_get_state(self.h, *[ctypes.byref(i) for i in v]))
        return tuple(i.value for i in v)

    def set_profiling(self, on: bool) -> None:
        self._chk(self.L.kg_set_profiling(self.h, int(on)))

    def get_profile(self) -> kg_profile:
        out = kg_profile()
        self._chk(self.L.kg_get_profile(self.h, ctypes.byref(out)))
        return out

    def reset(self) -> None:
        self._chk(self.L.kg_reset(self.h))

    # -- adapter training (Eq. 3)
    def train_bind(self, max_tokens: int) -> None:
        nb = ctypes.c_size_t()
        self._chk(self.L.kg_train_workspace_bytes(self.h, max_tokens, ctypes.byref(nb)))
        self.train_work = self._torch.empty(nb.value, dtype=self._torch.uint8, device=self.device)
        self._chk(self.L.kg_train_bind(self.h, self.train_work.data_ptr(), nb.value, max_tokens))
        self.train_bytes = nb.value

    def train_step(self, tokens: Sequence[int], lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                   weight_decay: float = 0.01) -> float:
        a = np.ascontiguousarray(tokens, dtype=np.int32)
        hp = kg_train_params(lr, beta1, beta2, eps, weight_decay)
        loss = ctypes.c_double()
        self._chk(self.L.kg_train_step(self.h, ctypes.byref(hp), a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(a),
                                       ctypes.byref(loss)))
        return loss.value

    def train_accumulate(self, tokens: Sequence[int]) -> float:
        a = np.ascontiguousarray(tokens, dtype=np.int32)
        loss = ctypes.c_double()
        self._chk(self.L.kg_train_accumulate(self.h, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(a), ctypes.byref(loss)))
        return loss.value

    def train_features(self, tokens: Sequence[int]):
        """(F, Zt) of a sequence as device tensors: what the frozen model contributes to a training step."""
        torch = self._torch
        a = np.ascontiguousarray(tokens, dtype=np.int32)
        F = torch.empty((len(a), self.shape.d_model), dtype=torch.float32, device=self.device)
        Zt = torch.empty((len(a), self.shape.vocab), dtype=torch.float32, device=self.device)
        self._chk(self.L.kg_train_features(self.h, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(a), F.data_ptr(), Zt.data_ptr()))
        return F, Zt

    def train_accumulate_features(self, F, Zt) -> float:
        loss = ctypes.c_double()
        self._chk(self.L.kg_train_accumulate_features(self.h, F.data_ptr(), Zt.data_ptr(), F.shape[0], ctypes.byref(loss)))
        return loss.value

    def train_apply(self, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01) -> None:
        hp = kg_train_params(lr, beta1, beta2, eps, weight_decay)
        self._chk(self.L.kg_train_apply(self.h, ctypes.byref(hp)))

    def train_param_count(self) -> int:
        return sum(int(np.prod(shp)) for _, shp in train_param_shapes(self.shape))

    def train_read(self, what: int, n_tokens: int = 0) -> np.ndarray:
        d, V = self.shape.d_model, self.shape.vocab
        npar = self.train_param_count()
        shape = {TRAIN_FEATURES: (n_tokens, d), TRAIN_TARGET_LOGITS: (n_tokens, V), TRAIN_DRAFT_LOGITS: (n_tokens, V),
                 TRAIN_GRADIENTS: (npar,), TRAIN_PARAMETERS: (npar,), TRAIN_ROW_LOSSES: (n_tokens,)}[what]
        out = np.empty(shape, dtype=np.float32)
        self._chk(self.L.kg_train_read(self.h, what, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), out.size))
        return out


def train_param_shapes(shape) -> list:
    """(name, shape) of the tensors of a parameter (or gradient) block, in block order, for the
    shape's adapter architecture: 0 / 1 attention (wq, wk, wv, wo, g_in, g_last [, head]),
    2 decoder block (.., g_post, wg, wu, wd), 3 two linear maps (w1, w2, g_in, g_last, head)."""
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    kind = getattr(shape, "adapter", 0)
    if kind == 3:
        out = [("w1", (d, d)), ("w2", (d, d))]
    else:
        out = [("wq", (d, d)), ("wk", (d, d)), ("wv", (d, d)), ("wo", (d, d))]
    out += [("g_in", (d,)), ("g_last", (d,))]
    if kind in (1, 3):
        out.append(("head", (V, d)))
    if kind == 2:
        out += [("g_post", (d,)), ("wg", (f, d)), ("wu", (f, d)), ("wd", (d, f))]
    return out


def split_param_block(block: np.ndarray, shape_or_d) -> dict:
    """Views of a parameter (or gradient) block by tensor name.  Takes the model shape (or, for the
    paper's adapter, just d_model)."""
    if isinstance(shape_or_d, int):
        d = shape_or_d
        spec = [("wq", (d, d)), ("wk", (d, d)), ("wv", (d, d)), ("wo", (d, d)), ("g_in", (d,)), ("g_last", (d,))]
    else:
        spec = train_param_shapes(shape_or_d)
    out, o = {}, 0
    for name, shp in spec:
        n = int(np.prod(shp))
        out[name] = block[o:o + n].reshape(shp)
        o += n
    assert o == block.size, (o, block.size)
    return out


def op_gemm_f32(A: np.ndarray, B: np.ndarray, C0: Optional[np.ndarray] = None, device: str = "cuda:0") -> np.ndarray:
    """C (+)= A . B through kg_op_gemm_f32; A [M][K] and B [K][N] may be any strided float32 views
    (their strides are passed on, so transposed views exercise the other load orientation)."""
    import torch
    dev = torch.device(device)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    # ship the underlying contiguous buffers and address them with the views' strides
    def ship(v):
        base = v if v.base is None else v.base
        base = np.ascontiguousarray(base, dtype=np.float32) if base is v else base
        t = torch.from_numpy(base).to(dev)
        off = (v.__array_interface__["data"][0] - base.__array_interface__["data"][0]) // 4
        return t, off, v.strides[0] // 4, v.strides[1] // 4
    ta, oa, sam, sak = ship(A)
    tb, ob, sbk, sbn = ship(B)
    c = torch.zeros((M, N), dtype=torch.float32, device=dev) if C0 is None else torch.from_numpy(np.ascontiguousarray(C0, dtype=np.float32)).to(dev)
    rc = lib().kg_op_gemm_f32(ta.data_ptr() + 4 * oa, sam, sak, tb.data_ptr() + 4 * ob, sbk, sbn, c.data_ptr(), N, M, N, K,
                              0 if C0 is None else 1, torch.cuda.current_stream(dev).cuda_stream)
    if rc != KG_OK:
        raise KangarooError(rc, "kg_op_gemm_f32")
    torch.cuda.synchronize(dev)
    return c.cpu().numpy()


def op_linear(W_host: np.ndarray, x_host: np.ndarray, device: str = "cuda:0") -> np.ndarray:
    """Y = X . W^T through kg_op_pack + kg_op_linear (W: float32 or uint16 bf16 bits, [N][K])."""
    import torch
    L = lib()
    dtype = 1 if W_host.dtype == np.uint16 else 0
    N, K = W_host.shape
    M = x_host.shape[0]
    dev = torch.device(device)
    w = torch.from_numpy(W_host.view(np.int16) if dtype else W_host).to(dev)
    packed = torch.empty(L.kg_op_packed_bytes(dtype, N, K), dtype=torch.uint8, device=dev)
    work = torch.empty(L.kg_op_work_bytes(K), dtype=torch.uint8, device=dev)
    x = torch.from_numpy(np.ascontiguousarray(x_host, dtype=np.float32)).to(dev)
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    s = torch.cuda.current_stream(dev).cuda_stream
    rc = L.kg_op_pack(dtype, w.data_ptr(), N, K, packed.data_ptr(), s)
    if rc != KG_OK:
        raise KangarooError(rc, "kg_op_pack")
    rc = L.kg_op_linear(dtype, packed.data_ptr(), N, K, x.data_ptr(), M, y.data_ptr(), work.data_ptr(), s)
    if rc != KG_OK:
        raise KangarooError(rc, "kg_op_linear")
    torch.cuda.synchronize(dev)
    return y.cpu().numpy()


def op_stream_read_GBs(n_bytes: int = 2 << 30, launches: int = 5, device: str = "cuda:0") -> float:
    """Bandwidth of kg_op_stream_read over a buffer of n_bytes (dependency-free loads): the measured
    ceiling that the weight-streaming projections are compared with.  Timed with events on the
    stream the launches go to."""
    import torch
    L = lib()
    dev = torch.device(device)
    buf = torch.empty(n_bytes, dtype=torch.uint8, device=dev)
    buf.zero_()
    work = torch.zeros(4096, dtype=torch.uint8, device=dev)
    st = torch.cuda.current_stream(dev)
    rc = L.kg_op_stream_read(buf.data_ptr(), n_bytes, work.data_ptr(), st.cuda_stream)
    if rc != KG_OK:
        raise KangarooError(rc, "kg_op_stream_read")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(launches):
        L.kg_op_stream_read(buf.data_ptr(), n_bytes, work.data_ptr(), st.cuda_stream)
    e1.record(st)
    e1.synchronize()
    return n_bytes * launches / (e0.elapsed_time(e1) * 1e-3) / 1e9
