"""Helpers of the GPU parity tests: drive the HIP library and the CPU oracle side by side.

The oracle follows the GPU's token stream (teacher forcing): at every decision the GPU's token
must be within `tie_tol` of the oracle's best logit; if it is not the oracle's own arg-max it is
counted as a near-tie exception and the oracle continues along the GPU's token.  Logits are
compared row by row on that common path.
"""
from __future__ import annotations

import numpy as np

from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import binding as B
from paper_2404_18911_amd import inputs as I


def load_model(shape, W, max_seq, gamma_max=6, kv_page_tokens=128):
    kg = B.Kangaroo(shape, max_seq, gamma_max=gamma_max, kv_page_tokens=kv_page_tokens)
    kg.load_weights((k, l, W[(k, l)]) for k, l, _, _ in I.tensor_list(shape))
    return kg


class Follow:
    def __init__(self, logit_tol, conf_tol=None):
        self.tol = logit_tol
        self.conf_tol = conf_tol if conf_tol is not None else logit_tol
        self.max_logit_err = 0.0
        self.exceptions = 0
        self.decisions = 0

    def logits(self, got, want, what):
        err = float(np.max(np.abs(got.astype(np.float64) - want)))
        self.max_logit_err = max(self.max_logit_err, err)
        assert err <= self.tol, f"{what}: logits differ by {err:.3e} > {self.tol:.1e}"

    def token(self, tok, want_logits, what):
        """GPU token vs oracle logits: must be a maximiser up to the tolerance."""
        self.decisions += 1
        best = int(np.argmax(want_logits))
        if tok != best:
            gap = float(want_logits[best] - want_logits[tok])
            assert gap <= self.tol, f"{what}: GPU token {tok} is {gap:.3e} below the oracle's best {best}"
            self.exceptions += 1


def follow_kangaroo(kg, model, prompt, n_new, gamma, eta, fol: Follow):
    """Run the GPU stepwise for n_new tokens with the oracle following.  Returns the GPU stream and
    the per-round records [(k, n)]."""
    p, _ = B.make_params(mode=0, eta=eta, gamma=gamma)
    dec = O.KangarooDecoder(model, gamma=gamma, eta=eta)
    t = kg.prefill(p, prompt)
    dec.prefill(prompt)
    fol.logits(kg.read_logits(1, 0), dec.prefill_logits, "prefill")
    fol.token(t, dec.prefill_logits, "prefill token")
    dec.pending = t
    out, rounds = [t], []
    while len(out) < n_new:
        while True:
            tok, conf, stop = kg.draft_step(p)
            j = len(dec.D)
            _, oconf, ostop = dec.draft_step(force_token=tok)
            z = dec.draft_logits[-1]
            fol.logits(kg.read_logits(0, j), z, f"draft logits round {len(rounds)} step {j}")
            fol.token(tok, z, f"draft token round {len(rounds)} step {j}")
            assert abs(conf - oconf) <= 3 * fol.conf_tol * max(oconf, 1e-3) + 1e-6, (conf, oconf)
            if stop != ostop:   # only legitimate when the confidence sits on the threshold
                assert abs(oconf - eta) <= 3 * fol.conf_tol * max(oconf, 1e-3) + 1e-6, (conf, oconf, eta)
                dec.stopped = stop
            np.testing.assert_allclose(kg.read_feature(j), dec.F[j], rtol=0, atol=fol.tol)
            if stop:
                break
        tg = kg.verify(p)
        Z = dec.verify()
        assert len(tg) == len(dec.D) + 1
        for i, tk in enumerate(tg):
            fol.logits(kg.read_logits(1, i), Z[i], f"target logits round {len(rounds)} row {i}")
            fol.token(tk, Z[i], f"target token round {len(rounds)} row {i}")
        em = kg.accept(p)
        oem = dec.accept(force_targets=tg)
        assert em == oem
        base, alen, lag, nd = kg.state()
        assert (base, alen, bool(lag), nd) == (dec.base, dec.adapter_len, dec.lag is not None, 0)
        rounds.append((dec.rounds[-1]["k"], dec.rounds[-1]["n"]))
        out += em
    return out, rounds


def follow_plain(kg, model, prompt, n_new, fol: Follow):
    p, _ = B.make_params()
    dec = O.PlainDecoder(model)
    t = kg.prefill(p, prompt)
    dec.prefill(prompt)
    fol.logits(kg.read_logits(1, 0), dec.last_logits, "prefill")
    fol.token(t, dec.last_logits, "prefill token")
    out = [t]
    while len(out) < n_new:
        nt = kg.plain_step(p, out[-1])
        dec.step(out[-1])
        fol.logits(kg.read_logits(1, 0), dec.last_logits, f"plain step {len(out)}")
        fol.token(nt, dec.last_logits, f"plain token {len(out)}")
        out.append(nt)
    return out


def _cdf_valid(p, tok, u, ctol):
    """Is `tok` what an inverse-CDF draw with uniform u gives for distribution p, allowing the
    cumulative sums to be off by ctol?"""
    c = np.cumsum(p)
    lo = c[tok - 1] if tok > 0 else 0.0
    return (lo - ctol <= u < c[tok] + ctol) and (p[tok] > 0.0 or ctol > 0.0)


def follow_kangaroo_sampling(kg, model, prompt, n_new, gamma, eta, temperature, U, fol: Follow, ctol):
    """Sampling mode (speculative rejection sampling) with the oracle following.  Every GPU decision
    is checked against the oracle's quantities for the same uniform numbers: a drawn token must be
    the inverse-CDF result up to ctol on the cumulative sums, an accept / reject must be on the
    right side of min(1, p/q) up to ctol.  Counts the decisions where the oracle itself would have
    decided otherwise (possible only inside the tolerance)."""
    p, keep = B.make_params(mode=1, temperature=temperature, eta=eta, gamma=gamma, uniforms=U)
    dec = O.KangarooDecoder(model, gamma=gamma, eta=eta, mode="sample", temperature=temperature, uniforms=U)
    t = kg.prefill(p, prompt)
    own = dec.prefill(prompt)
    fol.logits(kg.read_logits(1, 0), dec.prefill_logits, "prefill")
    assert _cdf_valid(O.softmax(dec.prefill_logits, temperature), t, float(U[len(prompt), O.U_RESAMPLE]), ctol)
    fol.decisions += 1
    fol.exceptions += int(own != t)
    dec.pending = t
    out, rounds = [t], []
    while len(out) < n_new:
        base = dec.base
        while True:
            tok, conf, stop = kg.draft_step(p)
            j = len(dec.D)
            # the oracle's own draw, then forced onto the GPU's token
            own, oconf, ostop = dec.draft_step()
            z, q = dec.draft_logits[-1], dec.Q[-1]
            fol.logits(kg.read_logits(0, j), z, f"draft logits round {len(rounds)} step {j}")
            assert _cdf_valid(q, tok, float(U[base + j + 1, O.U_DRAFT]), ctol), (tok, own)
            fol.decisions += 1
            fol.exceptions += int(own != tok)
            dec.D[-1] = tok
            assert abs(conf - oconf) <= 3 * fol.conf_tol * max(oconf, 1e-3) + 1e-6
            if stop != ostop:
                assert abs(oconf - eta) <= 3 * fol.conf_tol * max(oconf, 1e-3) + 1e-6
                dec.stopped = stop
            if stop:
                break
        k = len(dec.D)
        kg.verify(p)
        Z = dec.verify()
        for i in range(k + 1):
            fol.logits(kg.read_logits(1, i), Z[i], f"target logits round {len(rounds)} row {i}")
        em = kg.accept(p)
        n = len(em) - 1
        assert 0 <= n <= k and em[:n] == dec.D[:n]
        for i in range(min(n + 1, k)):
            pp, qq = O.softmax(Z[i], temperature), dec.Q[i]
            a = O.accept_probability(pp, qq, dec.D[i])
            u = float(U[base + i + 1, O.U_ACCEPT])
            fol.decisions += 1
            if i < n:
                assert u < a + ctol, ("accepted", u, a)
                fol.exceptions += int(not (u < a))
            else:
                assert u >= a - ctol, ("rejected", u, a)
                fol.exceptions += int(u < a)
        ur = float(U[base + n + 1, O.U_RESAMPLE])
        pn = O.softmax(Z[n], temperature)
        dist = O.residual_distribution(pn, dec.Q[n]) if n < k else pn
        assert _cdf_valid(dist, em[n], ur, 2 * ctol / max(1e-30, np.maximum(pn - dec.Q[n], 0).sum()) if n < k else ctol)
        fol.decisions += 1
        fol.exceptions += int(O.inverse_cdf(dist, ur) != em[n])
        oem = dec.accept(force_targets=em)
        assert oem == em
        bs, alen, lag, nd = kg.state()
        assert (bs, alen, bool(lag), nd) == (dec.base, dec.adapter_len, dec.lag is not None, 0)
        rounds.append((k, n))
        out += em
    return out, rounds
