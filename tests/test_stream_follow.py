"""CPU tests of the stored oracle streams and of the follower the GPU tests walk them with
(tests/parity.py: follow_stored_stream).  The follower is driven here by a stand-in device built
on the oracle itself, optionally with perturbed logits and forced near-tie flips, so that its
bookkeeping (on-stream rows, near-tie exceptions, restarts) is exercised without a GPU."""
import os

import numpy as np
import pytest

from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import inputs as I
from tests import parity as P
from tests.golden import make_oracle_streams as MK

DIR = os.path.join(os.path.dirname(__file__), "golden", "oracle_streams")


class OracleDevice:
    """The calls of binding.Kangaroo that the follower uses, answered by the oracle.  `noise` adds a
    fixed pseudo-random error to every logit row; `flip` maps a predicted position to "return the
    second-best token there" (kind 't' target / 'd' draft)."""

    def __init__(self, shape, W, max_seq, noise=0.0, flip=()):
        self.shape, self.W, self.max_seq, self.noise, self.flip = shape, W, max_seq, noise, set(flip)
        self.dec = None

    def _z(self, z, salt):
        if not self.noise:
            return z
        g = np.random.default_rng(salt)
        return z + self.noise * (2.0 * g.random(z.size) - 1.0)

    def _pick(self, z, kind, pos):
        order = np.lexsort((np.arange(z.size), -z))
        return int(order[1] if (kind, pos) in self.flip else order[0])

    def prefill(self, p, prompt):
        self.dec = O.KangarooDecoder(O.OracleModel(self.shape, self.W, self.max_seq), gamma=p.gamma, eta=p.eta)
        self.dec.prefill(prompt)
        self.tl = [self._z(self.dec.prefill_logits, len(prompt))]
        self.dec.pending = self._pick(self.tl[0], "t", len(prompt))
        self.dl = []
        return self.dec.pending

    def draft_step(self, p):
        d = self.dec
        pos = d.base + len(d.D) + 1
        d.draft_step()
        z = self._z(d.draft_logits[-1], 1000 + pos)
        tok = self._pick(z, "d", pos)
        d.D[-1] = tok
        q = O.softmax(z)
        d.Q[-1], d.conf[-1] = q, float(q.max())
        d.stopped = d.conf[-1] < p.eta or len(d.D) == p.gamma
        self.dl.append(z)
        return tok, d.conf[-1], d.stopped

    def verify(self, p):
        d = self.dec
        Z = d.verify()
        self.tl = [self._z(Z[i], 2000 + d.base + i + 1) for i in range(len(Z))]
        self.tg = [self._pick(self.tl[i], "t", d.base + i + 1) for i in range(len(Z))]
        return list(self.tg)

    def accept(self, p):
        em = self.dec.accept(force_targets=self.tg)
        self.dl = []
        return em

    def read_logits(self, which, row):
        return (self.dl if which == 0 else self.tl)[row].astype(np.float32)

    def state(self):
        d = self.dec
        return d.base, d.adapter_len, int(d.lag is not None), len(d.D)


def _load(name):
    rec = P.StreamRecord(os.path.join(DIR, name + ".npz"))
    cfg = MK.CONFIGS[name]
    shape = I.SHAPES[cfg["shape"]]
    W = I.gen_weights(shape, seed=1, alpha=cfg["alpha"], head_scale=cfg.get("head_scale", 1.0))
    prompt = I.gen_prompt(shape.vocab, cfg["n_prompt"], seed=2)
    return rec, shape, W, prompt


@pytest.mark.parametrize("name", ["toy", "toy_sharp"])
def test_stored_toy_streams_are_what_the_oracle_computes_now(name):
    """The committed small files equal a fresh run of the generator (so the generator, the oracle and
    the files agree), the stream equals plain decoding (lossless), every position of the request has
    a target record, and each round's records sit where the round structure says."""
    rec, shape, W, prompt = _load(name)
    fresh = MK.generate(name, threads=2, log=lambda s: None)
    for k, v in fresh.items():
        assert np.array_equal(np.asarray(v), rec.a[k]), k
    m = rec.meta
    plain = O.PlainDecoder(O.OracleModel(shape, W, 96)).generate(prompt, m["n_new"])
    assert plain == rec.stream
    assert all(m["n_prompt"] + i in rec.T for i in range(m["n_new"]))
    for base, k, n in rec.rounds:
        assert 1 <= k <= m["gamma"] and 0 <= n <= k
        assert all(base + j + 1 in rec.D for j in range(min(k, n + 1)))
    # a record's first top id is the stream's token at that position
    for i, tok in enumerate(rec.stream):
        assert int(rec.row("t", m["n_prompt"] + i)[0][0]) == tok
    P.check_probe(rec, O.OracleModel(shape, W, 16), prompt)


def test_probe_detects_other_weights():
    rec, shape, _, prompt = _load("toy")
    W2 = I.gen_weights(shape, seed=5, alpha=0.1)
    with pytest.raises(AssertionError):
        P.check_probe(rec, O.OracleModel(shape, W2, 16), prompt)


@pytest.mark.parametrize("name", ["toy", "toy_sharp"])
def test_follower_on_an_exact_device(name):
    rec, shape, W, prompt = _load(name)
    fol = P.CachedFollow(2e-6)      # the device hands out float32 rows
    rounds = P.follow_stored_stream(OracleDevice(shape, W, 96), rec, prompt, fol)
    assert fol.exceptions == 0 and fol.resyncs == 0 and fol.rows_norec == 0
    assert rounds == rec.rounds[:len(rounds)] and len(rounds) == len(rec.rounds)
    assert fol.rows_t >= rec.meta["n_new"] and fol.rows_d >= len(rec.rounds)


def test_follower_rejects_a_device_with_wrong_logits():
    rec, shape, W, prompt = _load("toy_sharp")
    with pytest.raises(AssertionError, match="logits differ"):
        P.follow_stored_stream(OracleDevice(shape, W, 96, noise=1e-2), rec, prompt, P.CachedFollow(1e-3))
    # the same device is inside a looser tolerance
    fol = P.CachedFollow(5e-2)
    P.follow_stored_stream(OracleDevice(shape, W, 96, noise=1e-2), rec, prompt, fol)
    assert 1e-3 < fol.max_logit_err <= 1e-2


def test_follower_restarts_after_a_near_tie_and_rejects_a_real_mismatch():
    """A device that returns the second-best token at some target and draft positions: with a
    tolerance wider than the gaps there, the follower counts the exceptions, restarts the device on
    the stored stream and still covers every position; with the real tolerance it fails."""
    rec, shape, W, prompt = _load("toy_sharp")
    n0 = rec.meta["n_prompt"]
    flips = [("t", n0), ("t", n0 + 7), ("t", n0 + 8), ("d", n0 + 12), ("t", n0 + 30)]
    fol = P.CachedFollow(1e3)
    P.follow_stored_stream(OracleDevice(shape, W, 96, flip=flips), rec, prompt, fol)
    assert fol.exceptions >= 4 and fol.resyncs >= 3
    assert fol.max_logit_err < 2e-6
    with pytest.raises(AssertionError, match="below the oracle's best"):
        P.follow_stored_stream(OracleDevice(shape, W, 96, flip=flips[:1]), rec, prompt, P.CachedFollow(1e-4))
