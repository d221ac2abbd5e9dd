"""Pins for the oracle's sampling-mode acceptance: it must leave the target model's sampling
distribution unchanged (abstract: "maintaining a consistent sampling distribution").  Checked by
brute force on a vocab-16 model: the decoder's decisions are piecewise constant in the uniforms,
so every cell of uniforms is enumerated exactly (cell volume = probability), the real decoder is
run on one point per cell, and the law of the emitted tokens is compared with the product of the
target model's conditionals, which are computed from scratch by whole-sequence forwards."""
import numpy as np
import pytest

from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import inputs as I

TINY = I.ModelShape("tiny16", 2, 16, 2, 8, 32, 16, 1, "f32")
PROMPT = [3, 11, 7]


class Need(Exception):
    def __init__(self, pos, purpose):
        self.pos, self.purpose = pos, purpose


class Uniforms:
    """Uniforms indexed by (position, purpose); reading one that is not fixed yet raises."""

    def __init__(self, fixed):
        self.fixed = fixed

    def __getitem__(self, key):
        if key not in self.fixed:
            raise Need(*key)
        return self.fixed[key]


@pytest.fixture(scope="module")
def world():
    W = I.gen_weights(TINY, seed=7, alpha=0.8, std=0.45)
    ref = O.OracleModel(TINY, W, 16)
    cache = {}

    def dists(prefix):
        """(target p, draft q) for the token following `prefix`, by a whole-sequence forward."""
        key = tuple(prefix)
        if key not in cache:
            f = ref.shallow(list(prefix), 0)
            p = O.softmax(ref.head(ref.deep(f, 0)[-1:], 0)[0])
            q = O.softmax(ref.head(ref.adapter(f, 0)[-1:], 1)[0])
            cache[key] = (p, q)
        return cache[key]

    return W, dists


def test_one_position_identity_for_arbitrary_rows():
    """sum_d q(d) [a(d) delta_d + (1 - a(d)) r] = p, with the oracle's own a and r."""
    rng = np.random.default_rng(0)
    for _ in range(50):
        p = rng.dirichlet(np.full(16, 0.3))
        q = rng.dirichlet(np.full(16, 0.3)) * 0.999 + 0.001 / 16
        r = O.residual_distribution(p, q)
        out = np.zeros(16)
        for d in range(16):
            a = O.accept_probability(p, q, d)
            out[d] += q[d] * a
            out += q[d] * (1.0 - a) * r
        np.testing.assert_allclose(out, p, rtol=0, atol=1e-12)


def test_inverse_cdf_cells():
    p = np.array([0.0, 0.25, 0.0, 0.5, 0.25])
    assert [O.inverse_cdf(p, u) for u in (0.0, 0.2499, 0.25, 0.7499, 0.75, 0.999999)] == [1, 1, 3, 3, 4, 4]


def test_inverse_cdf_past_the_accumulated_mass_returns_the_last_token_with_mass():
    """Rounding can leave the accumulated mass a hair below u: the answer is then the last token
    that has mass, never a zero-probability one behind it."""
    assert O.inverse_cdf(np.array([0.25, 0.25, 0.0, 0.0]), 0.9) == 1
    assert O.inverse_cdf(np.array([0.0, 1.0 - 2.0 ** -50, 0.0]), 1.0 - 2.0 ** -53) == 1


def test_argmax_ties_go_to_the_lowest_token_id_and_softmax_survives_large_logits():
    assert O.argmax_low(np.array([1.0, 3.0, 3.0, 2.0, 3.0])) == 1
    np.testing.assert_allclose(O.softmax(np.array([1000.0, 1000.0, -1000.0])), [0.5, 0.5, 0.0], atol=1e-300)
    np.testing.assert_allclose(O.softmax(np.array([-1000.0, -1000.0 + np.log(3.0)])), [0.25, 0.75], rtol=1e-12)


def enumerate_law(W, dists, gamma, eta, n_rounds_until, start=None, temperature=1.0):
    """Exact law of the tokens emitted after the prefill token, conditional on the uniforms in
    `start`.  Returns ({tuple(emitted): prob}, {tuple(emitted): one set of uniforms leading there})."""
    law = {}
    rep = {}
    runs = [0]

    def cells(breaks):
        pts = sorted(set([0.0, 1.0] + [min(1.0, max(0.0, float(b))) for b in breaks]))
        return [((a + b) / 2, b - a) for a, b in zip(pts[:-1], pts[1:]) if b - a > 0]

    def rec(fixed, prob):
        state = {}
        try:
            runs[0] += 1
            dec = O.KangarooDecoder(O.OracleModel(TINY, W, 16), gamma=gamma, eta=eta, mode="sample",
                                    temperature=temperature, uniforms=Uniforms(fixed))
            state["dec"] = dec
            state["out"] = [dec.prefill(PROMPT)]
            while not n_rounds_until(state["out"][1:], len(dec.S)):
                state["out"] += dec.round()
            key = tuple(state["out"][1:])
            law[key] = law.get(key, 0.0) + prob
            rep.setdefault(key, dict(fixed))
            return
        except Need as e:
            dec = state["dec"]
            seq = PROMPT + state.get("out", []) + dec.D
            p, q = dists(seq[:e.pos])
            if e.purpose == O.U_DRAFT:
                br = np.cumsum(q)
            elif e.purpose == O.U_ACCEPT:
                br = [O.accept_probability(p, q, seq[e.pos])]
            else:
                br = list(np.cumsum(p)) + list(np.cumsum(O.residual_distribution(p, q)))
            for mid, vol in cells(br):
                rec({**fixed, (e.pos, e.purpose): mid}, prob * vol)

    rec(dict(start) if start else {(len(PROMPT), O.U_RESAMPLE): 0.37}, 1.0)
    return law, rep


def test_two_tokens_over_two_rounds_gamma1(world):
    """gamma = 1: enumerate rounds until two tokens are out; joint law == p(a) p(b | a)."""
    W, dists = world
    law1, rep = enumerate_law(W, dists, 1, 0.6, lambda out, rounds: rounds >= 1)
    assert abs(sum(law1.values()) - 1.0) < 1e-12
    c = O.inverse_cdf(dists(PROMPT)[0], 0.37)
    p1 = dists(PROMPT + [c])[0]
    joint = np.zeros((16, 16))
    law = {}
    for key, pr in law1.items():
        if len(key) >= 2:
            joint[key[0], key[1]] += pr
            law[key] = pr
        else:
            # the state after a one-token round depends on the emitted token only: enumerate the
            # second round once, from one set of uniforms that leads there
            law2, _ = enumerate_law(W, dists, 1, 0.6, lambda out, rounds: len(out) >= 2, start=rep[key])
            assert abs(sum(law2.values()) - 1.0) < 1e-12
            for k2, pr2 in law2.items():
                assert k2[0] == key[0]
                joint[k2[0], k2[1]] += pr * pr2
                law[k2] = pr * pr2
    want = np.array([[p1[a] * dists(PROMPT + [c, a])[0][b] for b in range(16)] for a in range(16)])
    np.testing.assert_allclose(joint, want, rtol=0, atol=1e-12)
    # both outcomes of a round occurred with real mass
    lens = {len(k) for k in law}
    assert lens == {2, 3} or lens == {2}


@pytest.mark.parametrize("eta", [0.0, 1.5])
def test_one_round_gamma2_prefix_laws(world, eta):
    """gamma = 2, one round (k = 2 with eta = 0, k = 1 with eta > 1): the round's emitted tokens
    extended by the target's own conditionals reproduce p(a) p(b | a) p(c | a, b)."""
    W, dists = world
    law, _ = enumerate_law(W, dists, 2, eta, lambda out, rounds: rounds >= 1)
    assert abs(sum(law.values()) - 1.0) < 1e-12
    c0 = O.inverse_cdf(dists(PROMPT)[0], 0.37)
    base = PROMPT + [c0]
    kmax = 2 if eta == 0.0 else 1
    assert max(len(k) for k in law) == kmax + 1
    first = np.zeros(16)
    pair = np.zeros((16, 16))
    for key, pr in law.items():
        first[key[0]] += pr
        if len(key) >= 2:
            pair[key[0], key[1]] += pr
        else:
            pair[key[0], :] += pr * dists(base + [key[0]])[0]
    p1 = dists(base)[0]
    np.testing.assert_allclose(first, p1, rtol=0, atol=1e-12)
    want = np.array([p1[a] * dists(base + [a])[0] for a in range(16)])
    np.testing.assert_allclose(pair, want, rtol=0, atol=1e-12)
    if kmax == 2:
        tri = {}
        for key, pr in law.items():
            if len(key) == 3:
                tri[key] = tri.get(key, 0.0) + pr
        # mass of full acceptance + bonus token c, given the first two tokens (a, b), plus the
        # mass of shorter rounds continued by the target itself, equals the target's joint law
        for a in range(0, 16, 5):
            for b in range(0, 16, 3):
                got = np.zeros(16)
                for cc in range(16):
                    got[cc] = tri.get((a, b, cc), 0.0)
                short2 = law.get((a, b), 0.0)
                short1 = law.get((a,), 0.0)
                p2 = dists(base + [a])[0]
                p3 = dists(base + [a, b])[0]
                got += short2 * p3 + short1 * p2[b] * p3
                np.testing.assert_allclose(got, p1[a] * p2[b] * p3, rtol=0, atol=1e-12)


def _tempered(z, T):
    e = np.exp((np.asarray(z, dtype=np.float64) - np.max(z)) / T)
    return e / e.sum()


def test_softmax_temperature_closed_form():
    """Logits (0, ln 3) at temperature 2 give odds 1 : sqrt(3); temperature 1/2 gives 1 : 9."""
    z = np.array([0.0, np.log(3.0)])
    np.testing.assert_allclose(O.softmax(z, 2.0), np.array([1.0, np.sqrt(3.0)]) / (1.0 + np.sqrt(3.0)),
                               rtol=1e-15)
    np.testing.assert_allclose(O.softmax(z, 0.5), np.array([0.1, 0.9]), rtol=1e-15)


@pytest.mark.parametrize("T", [2.0, 0.5])
def test_one_round_law_at_other_temperatures(T):
    """gamma = 2, eta = 0 at temperature T: the first emitted token follows softmax(target / T),
    the first two follow the product of the tempered conditionals."""
    W = I.gen_weights(TINY, seed=7, alpha=0.8, std=0.45)
    ref = O.OracleModel(TINY, W, 16)
    cache = {}

    def dists(prefix):
        key = tuple(prefix)
        if key not in cache:
            f = ref.shallow(list(prefix), 0)
            cache[key] = (_tempered(ref.head(ref.deep(f, 0)[-1:], 0)[0], T),
                          _tempered(ref.head(ref.adapter(f, 0)[-1:], 1)[0], T))
        return cache[key]

    law, _ = enumerate_law(W, dists, 2, 0.0, lambda out, rounds: rounds >= 1, temperature=T)
    assert abs(sum(law.values()) - 1.0) < 1e-12
    c0 = O.inverse_cdf(dists(PROMPT)[0], 0.37)
    base = PROMPT + [c0]
    p1 = dists(base)[0]
    first = np.zeros(16)
    pair = np.zeros((16, 16))
    for key, pr in law.items():
        first[key[0]] += pr
        if len(key) >= 2:
            pair[key[0], key[1]] += pr
        else:
            pair[key[0], :] += pr * dists(base + [key[0]])[0]
    np.testing.assert_allclose(first, p1, rtol=0, atol=1e-12)
    want = np.array([p1[a] * dists(base + [a])[0] for a in range(16)])
    np.testing.assert_allclose(pair, want, rtol=0, atol=1e-12)
    # the tempered law is not the untempered one: the test would notice a dropped temperature
    assert np.abs(p1 - _tempered(np.log(p1) * T, 1.0)).max() > 1e-3


def test_draft_confidence_is_taken_from_the_tempered_draft_distribution():
    """Eq. 4's confidence is the top-1 probability of the distribution the draft is sampled from:
    at a very high temperature it tends to 1/vocab, so with eta = 0.5 every round stops after one
    draft, while the same weights at temperature 1 with a sharp head draft longer."""
    W = I.gen_weights(TINY, seed=7, alpha=0.05, std=0.45)
    W[(O.LM_HEAD, -1)] = (W[(O.LM_HEAD, -1)] * 40.0).astype(np.float32)
    rng = np.random.default_rng(5)
    U = rng.random((16, 3))
    ks = {}
    for T in (1.0, 1.0e4):
        dec = O.KangarooDecoder(O.OracleModel(TINY, W, 16), gamma=4, eta=0.5, mode="sample",
                                temperature=T, uniforms=U)
        dec.prefill(PROMPT)
        while dec.base < 10:
            dec.round()
        ks[T] = [r["k"] for r in dec.rounds]
        if T > 1.0:
            for r in dec.rounds:
                assert abs(r["conf"][0] - 1.0 / 16) < 0.02
    assert set(ks[1.0e4]) == {1}
    assert max(ks[1.0]) > 1


# ----------------------------------------------------------------------------- Philox4x32-10

def _philox_invert(out, key, rounds=10):
    """Undo `rounds` rounds of the published round function, from its definition: a round maps
    (c0, c1, c2, c3) to (hi(B c2) ^ c1 ^ k0, lo(B c2), hi(A c0) ^ c3 ^ k1, lo(A c0)), so c2 and c0 come
    back through the inverses of the odd multipliers mod 2^32, c1 and c3 through the xors.  The key
    of round r is key + r * (W0, W1) with the Weyl constants taken from their closed forms."""
    import math
    A, B, M = 0xD2511F53, 0xCD9E8D57, 1 << 32
    W0 = (math.isqrt(5 << 64) - (1 << 32)) >> 1           # floor(2^32 (sqrt(5) - 1) / 2), the golden ratio
    W1 = math.isqrt(3 << 64) - (1 << 32)                  # floor(2^32 (sqrt(3) - 1))
    Ai, Bi = pow(A, -1, M), pow(B, -1, M)
    o = list(out)
    for r in reversed(range(rounds)):
        k0, k1 = (key[0] + r * W0) % M, (key[1] + r * W1) % M
        c2 = (o[1] * Bi) % M
        c0 = (o[3] * Ai) % M
        c1 = o[0] ^ ((B * c2) >> 32) ^ k0
        c3 = o[2] ^ ((A * c0) >> 32) ^ k1
        o = [c0, c1, c2, c3]
    return o


def test_philox_is_the_ten_round_bijection_of_its_definition():
    """Ten published rounds, undone one by one, give the counter back: every xor partner, both
    multipliers, the word order, the round count and the key schedule (Weyl constants from their
    closed forms) have to be right for that."""
    rng = np.random.default_rng(9)
    cases = [([0, 0, 0, 0], [0, 0]), ([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2)]
    cases += [(rng.integers(0, 1 << 32, 4).tolist(), rng.integers(0, 1 << 32, 2).tolist()) for _ in range(200)]
    for ctr, key in cases:
        assert _philox_invert(O.philox4x32_10(ctr, key), key) == ctr
    # nine or eleven rounds do not invert it
    ctr, key = cases[5]
    assert _philox_invert(O.philox4x32_10(ctr, key), key, rounds=9) != ctr
    assert _philox_invert(O.philox4x32_10(ctr, key), key, rounds=11) != ctr


def test_philox_words_avalanche_and_are_uniform():
    """A counter or key bit flipped changes about half of the 128 output bits; 2^20 uniform numbers
    of consecutive positions fill 256 bins evenly (chi-square), have the moments of U[0,1) and no
    correlation between neighbouring positions or between the purposes of one position."""
    rng = np.random.default_rng(10)
    flips = []
    for _ in range(300):
        ctr, key = rng.integers(0, 1 << 32, 4).tolist(), rng.integers(0, 1 << 32, 2).tolist()
        a = O.philox4x32_10(ctr, key)
        bit = int(rng.integers(0, 192))
        c2, k2 = list(ctr), list(key)
        if bit < 128:
            c2[bit // 32] ^= 1 << (bit % 32)
        else:
            k2[(bit - 128) // 32] ^= 1 << (bit % 32)
        b = O.philox4x32_10(c2, k2)
        flips.append(sum(bin(x ^ y).count("1") for x, y in zip(a, b)))
    assert 60 < np.mean(flips) < 68 and min(flips) > 30
    n = 1 << 20
    U = O.philox_uniforms(12345, n).astype(np.float64)
    assert U.min() >= 0.0 and U.max() < 1.0
    for purpose in range(3):
        u = U[:, purpose]
        counts = np.bincount((u * 256).astype(int), minlength=256)
        chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 255 + 5 * np.sqrt(2 * 255), chi2            # mean 255, sd 22.6
        assert abs(u.mean() - 0.5) < 5 / np.sqrt(12 * n) and abs(u.var() - 1 / 12) < 1e-3
        assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 5 / np.sqrt(n)
    assert abs(np.corrcoef(U[:, 0], U[:, 1])[0, 1]) < 5 / np.sqrt(n)
    # the table is the generator: u[pos][purpose] = (word >> 8) 2^-24 of counter (pos, purpose, 0, 0)
    w = O.philox_words(12345, 1000, 2, 16)
    assert np.array_equal((w >> 8).astype(np.float64) * 2.0 ** -24, U[1000:1016, 2])
    assert w[3] == O.philox4x32_10([1003, 2, 0, 0], [12345, 0])[0]
    assert O.philox_words((7 << 32) | 5, 0, 0, 1)[0] == O.philox4x32_10([0, 0, 0, 0], [5, 7])[0]
