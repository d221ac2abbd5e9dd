"""TEST INFRASTRUCTURE, NOT THE PRODUCT: CPU oracle of Kangaroo's decode loops.

Only tests, the smoke check and the cpu_baseline leg of the benchmark may import this module.
It shares no code with the HIP library and imports nothing from it.

Two procedures are written out:
  * plain autoregressive decoding of the full model M^b (Section 1; the ground truth that
    "lossless" in the title refers to), and
  * the Kangaroo draft-and-verify round of Section 3 / Figure 2: draft with
    M^s = A o M^b[:l] until the top-1 confidence falls below eta (Eq. 4) or gamma drafts exist,
    compute the stopped token's next early feature, verify [f_0..f_k] with M^b[l:] in one pass,
    accept (greedy top-1 agreement, or speculative rejection sampling), roll the caches back.

The per-layer arithmetic is in kangaroo_ref.c (fp64), called through ctypes.  Softmax, argmax,
sampling and the control flow are here, in float64 numpy.

Readings of the paper (it is silent or ambiguous on these):
  - stop test is `confidence < eta` (the abstract says "falls below"; Eq. 4 prints <=); the
    low-confidence token itself is kept as a draft (Figure 2: x'_3 is verified), so k >= 1;
  - k <= gamma drafts, k+1 rows verified, 1..k+1 tokens emitted per round (Section 1);
  - the adapter lags by one feature after a fully accepted round and catches up on the
    two-row unit [f_k, f_{k+1}] (Figure 2 caption);
  - sampling mode: the draft samples from q, a draft d is accepted with probability
    min(1, p(d)/q(d)), the first rejection resamples from normalize(max(0, p-q)) and discards the
    rest (Section 3, "once a draft token is rejected..."), full acceptance draws a bonus token
    from the last target row; confidence is max q of the tempered draft distribution;
  - uniforms are indexed by (absolute position, purpose) and come from the caller;
  - argmax ties go to the lowest token id; inverse-CDF sampling walks ascending token ids.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libkangaroo_ref.so")

# tensor kinds: the key format of the `weights` dict, (kind, layer); layer = -1 outside the stack
EMBED, LM_HEAD, FINAL_NORM, WQ, WK, WV, WO, WG, WU, WD, NORM1, NORM2 = range(12)
A_WQ, A_WK, A_WV, A_WO, A_NORM_IN, A_NORM_LAST = range(12, 18)
A_HEAD, A_NORM_POST, A_WG, A_WU, A_WD, A_W1, A_W2 = range(18, 25)   # the other adapters of Table 2

U_DRAFT, U_ACCEPT, U_RESAMPLE = 0, 1, 2


SOURCES = [os.path.join(_HERE, "kangaroo_ref.c"), os.path.join(_HERE, "philox_ref.c")]


def build(force: bool = False, out: Optional[str] = None, extra_flags: Sequence[str] = ()) -> str:
    """Compile the C sources with gcc (portable AVX2 target so the library also runs elsewhere).
    `out` / `extra_flags` build a second copy with other flags (the sanitizer build of the tests)."""
    so = out or _SO
    if force or not os.path.exists(so) or any(os.path.getmtime(so) < os.path.getmtime(s) for s in SOURCES):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC", *extra_flags,
                               "-o", so, *SOURCES, "-lm"])
    return so


class _Cfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn",
                                            "vocab", "exit_layer", "wdtype", "max_seq", "kv_round",
                                            "adapter_kind")] + \
               [("rms_eps", ctypes.c_double), ("rope_theta", ctypes.c_double)]


class _W(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("embed", "lm_head", "final_norm")] + \
               [(n, ctypes.POINTER(ctypes.c_void_p)) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd",
                                                                "norm1", "norm2")] + \
               [(n, ctypes.c_void_p) for n in ("a_wq", "a_wk", "a_wv", "a_wo", "a_norm_in", "a_norm_last",
                                               "a_head", "a_norm_post", "a_wg", "a_wu", "a_wd", "a_w1", "a_w2")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        _lib.ko_create.restype = ctypes.c_void_p
        _lib.ko_create.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_W)]
        _lib.ko_destroy.argtypes = [ctypes.c_void_p]
        _lib.ko_embed.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, dp]
        _lib.ko_layers.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp, ctypes.c_int, ctypes.c_int]
        _lib.ko_adapter.argtypes = [ctypes.c_void_p, dp, ctypes.c_int, ctypes.c_int, dp]
        _lib.ko_head.argtypes = [ctypes.c_void_p, dp, ctypes.c_int, ctypes.c_int, dp]
        _lib.ko_kv_read.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp, dp]
        _lib.ko_kv_poison.argtypes = [ctypes.c_void_p, ctypes.c_int]
        _lib.ko_rmsnorm.argtypes = [dp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp]
        _lib.ko_rope.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        _lib.ko_softmax.argtypes = [dp, ctypes.c_int]
        _lib.ko_attend.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp]
        _lib.ko_round_bf16.restype = ctypes.c_double
        _lib.ko_round_bf16.argtypes = [ctypes.c_double]
        _lib.ko_round_f16.restype = ctypes.c_double
        _lib.ko_round_f16.argtypes = [ctypes.c_double]
        _lib.ko_matvec.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp,
                                   ctypes.c_int, dp]
        u32p = ctypes.POINTER(ctypes.c_uint32)
        _lib.ko_philox4x32_10.argtypes = [u32p, u32p, u32p]
        _lib.ko_philox_words.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int, u32p]
        _lib.ko_philox_uniforms.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
    return _lib


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


class OracleModel:
    """The model of kangaroo_ref.c bound to a set of weights (borrowed numpy arrays)."""

    def __init__(self, shape, weights: Dict[Tuple[int, int], np.ndarray], max_seq: int, exact_cache: bool = True):
        """exact_cache (the default): keys and values are cached as computed, the plain definition.
        With exact_cache=False the cache holds them rounded to the shape's cache storage type
        (bfloat16 or IEEE half), which is how one studies what such a storage format costs."""
        self.shape = shape
        self.L, self.d, self.V, self.l = shape.n_layers, shape.d_model, shape.vocab, shape.exit_layer
        self.max_seq = max_seq
        self._keep = weights
        wd = 0 if shape.dtype == "f32" else 1
        for a in weights.values():
            assert a.flags["C_CONTIGUOUS"] and a.dtype == (np.float32 if wd == 0 else np.uint16)
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                   shape.exit_layer, wd, max_seq,
                   0 if exact_cache else {"f32": 0, "bf16": 1, "f16": 2}[getattr(shape, "kv_dtype", shape.dtype)],
                   getattr(shape, "adapter", 0), shape.rms_eps, shape.rope_theta)
        w = _W()

        def ptr(kind, layer=-1):
            return ctypes.c_void_p(weights[(kind, layer)].ctypes.data)

        def opt(kind):
            return ptr(kind) if (kind, -1) in weights else None

        w.embed, w.lm_head, w.final_norm = ptr(EMBED), ptr(LM_HEAD), ptr(FINAL_NORM)
        self._arrs = []
        for name, kind in (("wq", WQ), ("wk", WK), ("wv", WV), ("wo", WO), ("wg", WG), ("wu", WU),
                           ("wd", WD), ("norm1", NORM1), ("norm2", NORM2)):
            arr = (ctypes.c_void_p * self.L)(*[weights[(kind, i)].ctypes.data for i in range(self.L)])
            self._arrs.append(arr)
            setattr(w, name, ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p)))
        kind = getattr(shape, "adapter", 0)
        need = {0: (A_WQ, A_WK, A_WV, A_WO), 1: (A_WQ, A_WK, A_WV, A_WO, A_HEAD),
                2: (A_WQ, A_WK, A_WV, A_WO, A_NORM_POST, A_WG, A_WU, A_WD), 3: (A_W1, A_W2, A_HEAD)}[kind]
        for k in need:
            assert (k, -1) in weights, f"adapter architecture {kind} needs tensor kind {k}"
        w.a_wq, w.a_wk, w.a_wv, w.a_wo = opt(A_WQ), opt(A_WK), opt(A_WV), opt(A_WO)
        w.a_norm_in, w.a_norm_last = ptr(A_NORM_IN), ptr(A_NORM_LAST)
        w.a_head, w.a_norm_post = opt(A_HEAD), opt(A_NORM_POST)
        w.a_wg, w.a_wu, w.a_wd, w.a_w1, w.a_w2 = opt(A_WG), opt(A_WU), opt(A_WD), opt(A_W1), opt(A_W2)
        self._h = lib().ko_create(ctypes.byref(cfg), ctypes.byref(w))
        if not self._h:
            raise MemoryError("ko_create failed")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().ko_destroy(self._h)
            self._h = None

    def embed(self, tokens: Sequence[int]) -> np.ndarray:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        x = np.empty((len(t), self.d), dtype=np.float64)
        lib().ko_embed(self._h, t.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(t), _dp(x))
        return x

    def layers(self, lo: int, hi: int, x: np.ndarray, pos0: int) -> np.ndarray:
        """Blocks lo..hi-1 on the rows of x at positions pos0..; returns a new array."""
        y = np.array(x, dtype=np.float64, order="C", copy=True)
        assert pos0 + y.shape[0] <= self.max_seq
        lib().ko_layers(self._h, lo, hi, _dp(y), pos0, y.shape[0])
        return y

    def shallow(self, tokens: Sequence[int], pos0: int) -> np.ndarray:
        """Early features f = M^b[:l](tokens) (Section 3.1)."""
        return self.layers(0, self.l, self.embed(tokens), pos0)

    def deep(self, f: np.ndarray, pos0: int) -> np.ndarray:
        """Remaining layers M^b[l:] on a unit of early features (Figure 2)."""
        return self.layers(self.l, self.L, f, pos0)

    def adapter(self, f: np.ndarray, pos0: int) -> np.ndarray:
        f = np.ascontiguousarray(f, dtype=np.float64)
        assert pos0 + f.shape[0] <= self.max_seq
        h = np.empty_like(f)
        lib().ko_adapter(self._h, _dp(f), pos0, f.shape[0], _dp(h))
        return h

    def head(self, x: np.ndarray, which: int) -> np.ndarray:
        """Logits; which = 0: target (final norm, LM head), 1: draft (adapter's last norm; the shared
        LM head, or the adapter's own for the architectures of Table 2 that have one)."""
        x = np.ascontiguousarray(x, dtype=np.float64)
        z = np.empty((x.shape[0], self.V), dtype=np.float64)
        lib().ko_head(self._h, _dp(x), x.shape[0], which, _dp(z))
        return z

    def kv_read(self, slot: int, pos: int) -> Tuple[np.ndarray, np.ndarray]:
        k = np.empty(self.d)
        v = np.empty(self.d)
        lib().ko_kv_read(self._h, slot, pos, _dp(k), _dp(v))
        return k, v

    def kv_poison(self, frm: int) -> None:
        lib().ko_kv_poison(self._h, frm)


# ----------------------------------------------------------------------------- random numbers

def philox4x32_10(counter: Sequence[int], key: Sequence[int]) -> List[int]:
    """One block of Philox4x32-10 (philox_ref.c)."""
    c = (ctypes.c_uint32 * 4)(*counter)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    lib().ko_philox4x32_10(c, k, o)
    return list(o)


def philox_words(seed: int, pos0: int, purpose: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint32)
    lib().ko_philox_words(seed, pos0, purpose, n, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    return out


def philox_uniforms(seed: int, n_positions: int) -> np.ndarray:
    """float32 [n_positions][3] in [0, 1): the uniform number of every (absolute position, purpose)
    for a seed, u = (first Philox word >> 8) * 2^-24 (philox_ref.c)."""
    u = np.empty((n_positions, 3), dtype=np.float32)
    lib().ko_philox_uniforms(seed, n_positions, u.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return u


# ----------------------------------------------------------------------------- distributions

def softmax(z: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64) / temperature
    e = np.exp(z - z.max())
    return e / e.sum()


def argmax_low(z: np.ndarray) -> int:
    """Index of the maximum; the lowest index among equal maxima."""
    return int(np.argmax(z))


def inverse_cdf(p: np.ndarray, u: float) -> int:
    """Smallest n with p_0 + .. + p_n > u, ascending token id, accumulated in float64."""
    acc = 0.0
    last = 0
    for n in range(len(p)):
        if p[n] > 0.0:
            last = n
        acc += float(p[n])
        if acc > u:
            return n
    return last  # u beyond the accumulated mass by rounding: last token with mass


def accept_probability(p: np.ndarray, q: np.ndarray, d: int) -> float:
    """Probability that draft token d ~ q is kept under target p."""
    return min(1.0, float(p[d]) / float(q[d]))


def residual_distribution(p: np.ndarray, q: np.ndarray) -> np.ndarray:
    """normalize(max(0, p - q)): what a rejected position is resampled from."""
    r = np.maximum(p - q, 0.0)
    s = r.sum()
    return r / s if s > 0.0 else p.copy()


# ----------------------------------------------------------------------------- metrics

def compression_rate(S: Sequence[int]) -> float:
    """Eq. 1: mean number of tokens emitted per forward of the large model."""
    return float(sum(S)) / len(S)


def ctar(S: Sequence[int], w: int) -> float:
    """Eq. 2: fraction of rounds in which the first w drafts were all accepted (s_k - w > 0)."""
    return sum(1 for s in S if s - w > 0) / len(S)


# ----------------------------------------------------------------------------- plain decoding

class PlainDecoder:
    """Autoregressive decoding of the full model, one token per forward."""

    def __init__(self, model: OracleModel, mode: str = "greedy", temperature: float = 1.0,
                 uniforms: Optional[np.ndarray] = None):
        self.m, self.mode, self.T, self.u = model, mode, temperature, uniforms
        self.n = 0            # tokens whose keys/values are cached
        self.last_logits = None

    def _pick(self, z: np.ndarray, pos: int) -> int:
        if self.mode == "greedy":
            return argmax_low(z)
        return inverse_cdf(softmax(z, self.T), float(self.u[pos, U_RESAMPLE]))

    def prefill(self, prompt: Sequence[int]) -> int:
        x = self.m.layers(0, self.m.L, self.m.embed(prompt), 0)
        self.n = len(prompt)
        self.last_logits = self.m.head(x[-1:], 0)[0]
        return self._pick(self.last_logits, self.n)

    def step(self, token: int) -> int:
        """Feed `token` (at position n), return the next token."""
        x = self.m.layers(0, self.m.L, self.m.embed([token]), self.n)
        self.n += 1
        self.last_logits = self.m.head(x, 0)[0]
        return self._pick(self.last_logits, self.n)

    def generate(self, prompt: Sequence[int], n_new: int) -> List[int]:
        out = [self.prefill(prompt)]
        while len(out) < n_new:
            out.append(self.step(out[-1]))
        return out


# ----------------------------------------------------------------------------- Kangaroo

class KangarooDecoder:
    """Draft-and-verify decoding, stepwise.  State between rounds: `base` tokens are committed
    in the shallow and deep caches, `pending` is the token at position `base` whose features are
    not computed yet, `lag` is an early feature at position base-1 the adapter has not seen."""

    def __init__(self, model: OracleModel, gamma: int = 6, eta: float = 0.6, mode: str = "greedy",
                 temperature: float = 1.0, uniforms: Optional[np.ndarray] = None,
                 eager_adapter: bool = False, stop_le: bool = False):
        self.m, self.gamma, self.eta, self.mode, self.T, self.u = model, gamma, eta, mode, temperature, uniforms
        self.eager = eager_adapter
        self.stop_le = stop_le
        self.base = 0
        self.pending = -1
        self.lag: Optional[np.ndarray] = None
        self.adapter_len = 0
        self.S: List[int] = []
        self.rounds: List[dict] = []
        self._reset_round()

    def _reset_round(self):
        self.F: List[np.ndarray] = []     # early features f_0..f_k of this round
        self.D: List[int] = []            # draft tokens x'_1..x'_k
        self.Q: List[np.ndarray] = []     # draft distributions
        self.conf: List[float] = []
        self.draft_logits: List[np.ndarray] = []
        self.target_logits: Optional[np.ndarray] = None
        self.stopped = False

    # -- prefill: the full model and the adapter see the whole prompt; first token is the target's.
    #    `chunk` feeds the prompt rows through in pieces of that many rows: with the caches in place
    #    a row's arithmetic does not depend on how many rows travel with it (pinned by the
    #    mixed-row-count test), so this only bounds the size of the temporaries for long prompts;
    #    `progress(rows_done)` is called after each piece.
    def prefill(self, prompt: Sequence[int], chunk: Optional[int] = None, progress=None) -> int:
        T = len(prompt)
        step = T if not chunk else int(chunk)
        x_last = None
        for lo in range(0, T, step):
            f = self.m.shallow(prompt[lo:lo + step], lo)
            self.m.adapter(f, lo)                  # fills the adapter's cache; outputs unused
            x_last = self.m.deep(f, lo)[-1:]
            if progress is not None:
                progress(min(T, lo + step))
        z = self.m.head(x_last, 0)[0]
        self.prefill_logits = z
        self.base, self.adapter_len, self.lag = T, T, None
        if self.mode == "greedy":
            self.pending = argmax_low(z)
        else:
            self.pending = inverse_cdf(softmax(z, self.T), float(self.u[T, U_RESAMPLE]))
        self._reset_round()
        return self.pending

    # -- one draft token (Section 3.2).  Returns (token, confidence, stop).
    def draft_step(self, force_token: Optional[int] = None) -> Tuple[int, float, bool]:
        assert not self.stopped and len(self.D) < self.gamma
        j = len(self.D)                            # 0-based index of this draft
        tok = self.pending if j == 0 else self.D[-1]
        pos = self.base + j
        f = self.m.shallow([tok], pos)[0]
        self.F.append(f)
        if j == 0 and self.lag is not None:
            h = self.m.adapter(np.stack([self.lag, f]), pos - 1)[-1]
            self.lag = None
        else:
            h = self.m.adapter(f[None, :], pos)[0]
        self.adapter_len = pos + 1
        z = self.m.head(h[None, :], 1)[0]
        q = softmax(z, self.T)
        conf = float(q.max())
        if self.mode == "greedy":
            d = argmax_low(z)
        else:
            d = inverse_cdf(q, float(self.u[pos + 1, U_DRAFT]))
        if force_token is not None:
            d = int(force_token)
        self.D.append(d)
        self.Q.append(q)
        self.conf.append(conf)
        self.draft_logits.append(z)
        low = conf <= self.eta if self.stop_le else conf < self.eta          # Eq. 4
        self.stopped = low or len(self.D) == self.gamma
        return d, conf, self.stopped

    # -- next early feature of the last draft, then M^b[l:] on [f_0..f_k] in one pass (Figure 2)
    def verify(self) -> np.ndarray:
        k = len(self.D)
        assert k >= 1
        fk = self.m.shallow([self.D[-1]], self.base + k)[0]
        self.F.append(fk)
        if self.eager:
            self.m.adapter(fk[None, :], self.base + k)
        x = self.m.deep(np.stack(self.F), self.base)
        self.target_logits = self.m.head(x, 0)          # k+1 rows
        return self.target_logits

    # -- acceptance and rollback.  Returns the emitted tokens (1..k+1 of them).
    def accept(self, force_targets: Optional[Sequence[int]] = None) -> List[int]:
        k = len(self.D)
        Z = self.target_logits
        if self.mode == "greedy":
            t = [argmax_low(Z[i]) for i in range(k + 1)]
            if force_targets is not None:
                t = [int(v) for v in force_targets]
            n = 0
            while n < k and self.D[n] == t[n]:
                n += 1
            emitted = self.D[:n] + [t[n]]
        else:
            n = 0
            emitted = []
            while n < k:
                p = softmax(Z[n], self.T)
                pos = self.base + n + 1                 # position of draft token D[n]
                if float(self.u[pos, U_ACCEPT]) < accept_probability(p, self.Q[n], self.D[n]):
                    emitted.append(self.D[n])
                    n += 1
                else:
                    emitted.append(inverse_cdf(residual_distribution(p, self.Q[n]),
                                               float(self.u[pos, U_RESAMPLE])))
                    break
            if n == k:
                pos = self.base + k + 1
                emitted.append(inverse_cdf(softmax(Z[k], self.T), float(self.u[pos, U_RESAMPLE])))
            if force_targets is not None:
                emitted = [int(v) for v in force_targets]
                n = len(emitted) - 1
        self.rounds.append(dict(base=self.base, k=k, n=n, drafts=list(self.D), conf=list(self.conf),
                                emitted=list(emitted)))
        old = self.base
        self.base = old + n + 1
        if self.eager:
            self.adapter_len, self.lag = self.base, None
        else:
            self.adapter_len = old + min(n + 1, k)
            self.lag = self.F[k] if n == k else None
        self.pending = emitted[-1]
        self.S.append(n + 1)
        self._reset_round()
        return emitted

    def round(self) -> List[int]:
        while True:
            _, _, stop = self.draft_step()
            if stop:
                break
        self.verify()
        return self.accept()

    def generate(self, prompt: Sequence[int], n_new: int) -> List[int]:
        out = [self.prefill(prompt)]
        while len(out) < n_new:
            em = self.round()
            room = n_new - len(out)
            if len(em) > room:                      # truncate the last round
                em = em[:room]
                self.S[-1] = room
            out.extend(em)
        return out
