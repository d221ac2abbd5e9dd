"""Writes tests/golden/oracle_streams/<name>.npz: what the CPU oracle computes along its own greedy
Kangaroo stream for the full-size BASELINE requests (7B 256+256 at alpha 0.05 and 0.2, 13B 512+256,
33B 512+128, and the 7B 4096-token context of the long-context configuration decoded greedily).

The oracle needs tens of seconds to minutes of host time per request at these sizes, more than a
GPU test run can spend on every request, so its results are computed once and stored; the GPU
tests walk the same requests, compare every row whose context is the stored stream with the
record of its position, and re-compute the small `probe` record with the live oracle to show that
file, weights and oracle still belong together.

This script calls only oracle/ and the seeded input generators: nothing here comes from the HIP
library.  Usage (the 33B request needs about 70 GB of host memory):
    python tests/golden/make_oracle_streams.py c2_a005 [c2_a020 c3_13b c4_33b c5_greedy] [--out DIR]

Records.  The token at absolute position p is predicted from the prefix x[0..p-1].
  stream[i]              the oracle's token at position n_prompt + i (greedy Kangaroo == plain decoding)
  round_base/k/n         per round: committed length at its start, drafts made, drafts accepted
  t_pos, t_*             target model: one record per position n_prompt .. n_prompt + n_new - 1 (and the
                         few beyond that the last round reached), from the prefill row or from the
                         verification row whose drafts before it were all accepted
  d_pos, d_*             self-draft model: one record per draft step whose earlier drafts of the round
                         were all accepted (its context is the stream), plus its confidence
  *_top_ids / *_top      the four largest logits (ties: lowest id first) and their ids
  *_samples              the logits at `sample_ids` (64 seeded vocabulary ids, the same for every row)
  *_lse                  log sum exp of the row
  probe_*                target record after a prefill of only the first `probe_len` prompt tokens
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import kangaroo_oracle as O                      # noqa: E402
from paper_2404_18911_amd import inputs as I                 # noqa: E402

FORMAT = 1
N_SAMPLES = 64
N_TOP = 4
PROBE_LEN = 8

# name -> request; seeds as everywhere: weights 1, prompt 2
CONFIGS = {
    "c2_a005": dict(shape="7b", alpha=0.05, n_prompt=256, n_new=256, gamma=6, eta=0.6),
    "c2_a020": dict(shape="7b", alpha=0.2, n_prompt=256, n_new=256, gamma=6, eta=0.6),
    "c3_13b": dict(shape="13b", alpha=0.1, n_prompt=512, n_new=256, gamma=6, eta=0.6),
    "c4_33b": dict(shape="33b", alpha=0.1, n_prompt=512, n_new=128, gamma=6, eta=0.6),
    "c5_greedy": dict(shape="7b", alpha=0.1, n_prompt=4096, n_new=256, gamma=6, eta=0.6),
    # small requests (seconds): used by the CPU tests of this file's format and of the follower
    "toy": dict(shape="toy", alpha=0.1, n_prompt=16, n_new=32, gamma=6, eta=0.6),
    "toy_sharp": dict(shape="toy", alpha=0.05, n_prompt=16, n_new=48, gamma=6, eta=0.6, head_scale=25.0),
}


def sample_ids(vocab: int) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=[7, 0x73616D70]))
    return np.sort(g.choice(vocab, size=min(N_SAMPLES, vocab), replace=False)).astype(np.int32)


def row_record(z: np.ndarray, ids: np.ndarray):
    """(top ids, top logits, sampled logits, log-sum-exp) of one logit row."""
    z = np.asarray(z, dtype=np.float64)
    order = np.lexsort((np.arange(z.size), -z))[:N_TOP]          # by logit, descending; ties: lowest id first
    mx = z.max()
    lse = mx + np.log(np.exp(z - mx).sum())
    return order.astype(np.int32), z[order], z[ids], lse


def generate(name: str, threads: int, log=print) -> dict:
    cfg = dict(CONFIGS[name])
    shape = I.SHAPES[cfg["shape"]]
    n_prompt, n_new, gamma, eta = cfg["n_prompt"], cfg["n_new"], cfg["gamma"], cfg["eta"]
    hs = cfg.get("head_scale", 1.0)
    t0 = time.time()
    W = I.gen_weights(shape, seed=1, alpha=cfg["alpha"], head_scale=hs, threads=threads)
    prompt = I.gen_prompt(shape.vocab, n_prompt, seed=2)
    log(f"[{name}] weights in {time.time() - t0:.1f}s")
    ids = sample_ids(shape.vocab)

    # probe: target record after the first few prompt tokens only (a fresh, small cache)
    pm = O.OracleModel(shape, W, PROBE_LEN + 1)
    pd = O.PlainDecoder(pm)
    pd.prefill(prompt[:PROBE_LEN])
    probe = row_record(pd.last_logits, ids)
    del pd, pm

    model = O.OracleModel(shape, W, n_prompt + n_new + gamma + 2)
    dec = O.KangarooDecoder(model, gamma=gamma, eta=eta)
    T = {}     # position -> record
    D = {}     # position -> record + confidence
    t0 = time.time()
    first = dec.prefill(prompt, chunk=256,
                        progress=lambda done: log(f"[{name}] prompt rows {done}/{n_prompt}, {time.time() - t0:.1f}s"))
    T[n_prompt] = row_record(dec.prefill_logits, ids)
    log(f"[{name}] prefill of {n_prompt} tokens in {time.time() - t0:.1f}s")
    stream = [first]
    rounds = []
    t0 = time.time()
    while len(stream) < n_new:
        base = dec.base
        while True:
            _, _, stop = dec.draft_step()
            if stop:
                break
        drafts, confs, zd = list(dec.D), list(dec.conf), list(dec.draft_logits)
        Z = dec.verify()
        em = dec.accept()
        n = len(em) - 1
        for j in range(len(drafts)):
            if j <= n:                       # drafts 0..j-1 were accepted: this step saw the stream
                D[base + j + 1] = row_record(zd[j], ids) + (confs[j],)
        for i in range(n + 1):
            T[base + i + 1] = row_record(Z[i], ids)
        rounds.append((base, len(drafts), n))
        stream.extend(em)
        if len(rounds) % 16 == 0:
            log(f"[{name}] {len(stream)} tokens after {len(rounds)} rounds, {time.time() - t0:.1f}s")
    stream = stream[:n_new]
    log(f"[{name}] decode of {n_new} tokens in {time.time() - t0:.1f}s, {len(rounds)} rounds")

    meta = dict(format=FORMAT, name=name, **cfg, weight_seed=1, prompt_seed=2, probe_len=PROBE_LEN,
                oracle_cache="exact", dtype=shape.dtype)
    tp = sorted(T)
    dp = sorted(D)
    out = dict(
        meta=np.array(json.dumps(meta, sort_keys=True)),
        stream=np.array(stream, dtype=np.int32),
        round_base=np.array([r[0] for r in rounds], dtype=np.int32),
        round_k=np.array([r[1] for r in rounds], dtype=np.int32),
        round_n=np.array([r[2] for r in rounds], dtype=np.int32),
        sample_ids=ids,
        t_pos=np.array(tp, dtype=np.int32),
        t_top_ids=np.stack([T[p][0] for p in tp]), t_top=np.stack([T[p][1] for p in tp]),
        t_samples=np.stack([T[p][2] for p in tp]).astype(np.float32), t_lse=np.array([T[p][3] for p in tp]),
        d_pos=np.array(dp, dtype=np.int32),
        d_top_ids=np.stack([D[p][0] for p in dp]), d_top=np.stack([D[p][1] for p in dp]),
        d_samples=np.stack([D[p][2] for p in dp]).astype(np.float32), d_lse=np.array([D[p][3] for p in dp]),
        d_conf=np.array([D[p][4] for p in dp]),
        probe_top_ids=probe[0], probe_top=probe[1], probe_samples=probe[2], probe_lse=np.array(probe[3]),
    )
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("names", nargs="+", choices=sorted(CONFIGS))
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_streams"))
    ap.add_argument("--threads", type=int, default=min(16, os.cpu_count() or 1))
    a = ap.parse_args()
    os.makedirs(a.out, exist_ok=True)
    for name in a.names:
        rec = generate(name, a.threads, log=lambda s: print(s, flush=True))
        path = os.path.join(a.out, name + ".npz")
        np.savez_compressed(path, **rec)
        print(f"[{name}] wrote {path} ({os.path.getsize(path)} bytes)", flush=True)


if __name__ == "__main__":
    main()
