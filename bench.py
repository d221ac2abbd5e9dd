#!/usr/bin/env python3
"""Benchmark of the Kangaroo decode loop on one MI355X.

A step is one pass of the whole hot path over one synthetic request of the Vicuna-7B-shaped
configuration: prefill of a 256-token prompt, then draft-and-verify rounds until 256 new tokens
are out (eta = 0.6, gamma = 6, greedy).  `value` is new tokens per second of the decode loop
(prefill excluded, host synchronisations included), summed over the timed steps; `ms_per_step`
is the wall-clock of a whole step, prefill included.  Weights are random-init (see
paper_2404_18911_amd/inputs.py) and are resident in HBM before the timed region.

Prints ONE JSON line.  Extra legs (not part of `value`): plain decoding, eta = 0, the second
alpha of the configuration, a per-launch-timed pass for the roofline figure, and the CPU oracle
timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


TRAFFIC_PROFILE = os.path.join("profiles", "gemv_bf16_attn_7b_kangaroo_decode.txt")


def kernel_source_digest():
    """Digest of the library's sources: the committed counter summary names the digest it was
    measured with, so that a traffic figure that outlived a kernel change is reported as stale."""
    import hashlib
    h = hashlib.sha256()
    for rel in ("paper_2404_18911_amd/csrc/kernels.hip.h", "paper_2404_18911_amd/csrc/kangaroo.hip"):
        h.update(open(os.path.join(ROOT, rel), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic():
    """HBM bytes per projection launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs of this very command, scaled by a copy of known size), or None; with where the
    figure comes from and whether the kernels have changed since it was measured.  It is not measured
    by this run: counters need a profiler pass of their own."""
    traffic = digest = None
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_PROFILE)):
            f = line.split()
            if len(f) >= 2 and f[0] == "TRAFFIC_BYTES_PER_PROJECTION_LAUNCH":
                traffic = float(f[1])
            if len(f) >= 2 and f[0] == "KERNEL_SOURCE_DIGEST":
                digest = f[1]
    except OSError:
        pass
    now = kernel_source_digest()
    return traffic, {"from": TRAFFIC_PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this command, committed)",
                     "measured_with_kernel_digest": digest, "kernel_digest_now": now, "stale": digest != now}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def forward_bytes(shape, ctx=0):
    """Algorithmic HBM bytes of each forward type: weights once, plus the cached keys and values of
    `ctx` positions once per attention layer of the forward."""
    b = shape.bytes_per_weight()
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    kv = 2 * d * (4 if shape.kv_dtype == "f32" else 2) * ctx          # one layer's cache
    from paper_2404_18911_amd import inputs as I
    layer = (4 * d * d + 3 * d * f) * b
    head = d * V * b
    # the adapter's matrices in the architecture of Table 2 the shape names (an own LM head included);
    # the draft step also reads the shared head unless the adapter has its own, and the adapter's
    # cache unless it has no attention
    adapter = sum(r * c for _, _, r, c in I.adapter_tensor_list(shape) if r > 1) * b
    own_head = shape.adapter in (I.ADAPTER_ATTN_HEAD, I.ADAPTER_MLP)
    akv = 0 if shape.adapter == I.ADAPTER_MLP else kv
    l, L = shape.exit_layer, shape.n_layers
    return dict(layer=layer, head=head, adapter=adapter, plain=L * (layer + kv) + head,
                draft=l * (layer + kv) + adapter + akv + (0 if own_head else head), shallow=l * (layer + kv),
                verify=(L - l) * (layer + kv) + head)


def reload_alpha(kg, shape, alpha, threads):
    """Re-draw the tensors that depend on alpha (deep o_proj / down_proj, adapter output projection)."""
    from concurrent.futures import ThreadPoolExecutor
    from paper_2404_18911_amd import inputs as I
    with ThreadPoolExecutor(max_workers=threads) as pool:
        for kind, layer, rows, cols in I.tensor_list(shape):
            if (kind in (I.KIND_WO, I.KIND_WD) and layer >= shape.exit_layer) or kind == I.KIND_A_WO:
                kg.load_tensor(kind, layer, I.gen_tensor(shape, kind, layer, rows, cols, seed=1, alpha=alpha, pool=pool))


def cpu_baseline(shape, W, prompt, threads, n_prompt=32, n_new=8):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import kangaroo_oracle as O
    os.environ.setdefault("OMP_NUM_THREADS", str(threads))
    m = O.OracleModel(shape, W, n_prompt + n_new + 16)
    dec = O.KangarooDecoder(m, gamma=6, eta=0.6)
    out = [dec.prefill(list(prompt[:n_prompt]))]
    t0 = time.time()
    while len(out) < n_new + 1:
        out += dec.round()
    dt = time.time() - t0
    n = len(out) - 1
    return {"value": n / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"same 7B-shaped weights, first {n_prompt} prompt tokens, {n} new tokens of Kangaroo "
                      f"decoding (eta 0.6, gamma 6), decode loop only, fp64 C + OpenMP"}


def run_sweep(args):
    """Hyper-parameter sweeps of Section 4.2 on synthetic weights (Figure 3's axes): threshold eta x
    draft length gamma at the configuration's exit layer, then the exit layer l at (gamma 6, eta 0.6).
    The LM head is sharpened (--head-scale) so that draft confidences spread over (0, 1) and the stop
    rule really fires at different lengths; with the plain random head every draft has confidence
    far below any eta > 0.  Prints one JSON object; not part of the benchmark line."""
    import dataclasses
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I
    threads = min(16, os.cpu_count() or 8)
    base = I.SHAPES[args.shape]
    prompt = I.gen_prompt(base.vocab, args.prompt)
    gmax = 7
    out = {"sweep": True, "shape": args.shape, "alpha": args.alpha, "head_scale": args.head_scale,
           "prompt": args.prompt, "new": args.new, "eta_gamma": [], "exit_layer": []}

    def load(shape):
        kg = B.Kangaroo(shape, args.prompt + args.new + gmax + 2, gamma_max=gmax, kv_page_tokens=128)
        for kind, layer, a in I.iter_weights(shape, seed=1, alpha=args.alpha, head_scale=args.head_scale, threads=threads):
            kg.load_tensor(kind, layer, a)
        return kg

    def run(kg, gamma, eta):
        p, _ = B.make_params(eta=eta, gamma=gamma)
        kg.generate(p, prompt, args.new)
        toks, st = kg.generate(p, prompt, args.new)
        return {"gamma": gamma, "eta": eta, "tokens_per_s": (len(toks) - 1) / st.t_total_s,
                "compression_rate": (args.new - 1) / st.rounds, "mean_draft_len": st.drafted / st.rounds,
                "acceptance_rate": st.accepted / max(1, st.drafted),
                "ctar": [sum(c for s_, c in enumerate(st.s_hist) if s_ - w > 0) / st.rounds for w in range(1, gamma + 1)]}

    kg = load(base)
    p0, _ = B.make_params()
    toks, stp = kg.decode_plain(p0, prompt, args.new)
    out["plain_tokens_per_s"] = (len(toks) - 1) / stp.t_total_s
    for gamma in (2, 4, 6, 7):
        for eta in (0.0, 0.2, 0.4, 0.6, 0.8, 1.01):
            r = run(kg, gamma, eta)
            out["eta_gamma"].append(r)
            log(f"[sweep] gamma {gamma} eta {eta}: {r['tokens_per_s']:.1f} tok/s, CR {r['compression_rate']:.2f}, k {r['mean_draft_len']:.2f}")
    kg.close()
    del kg
    for l in (1, 2, 3, 4):
        shape = dataclasses.replace(base, exit_layer=l)
        kg = load(shape)
        r = run(kg, 6, 0.6)
        r["exit_layer"] = l
        out["exit_layer"].append(r)
        log(f"[sweep] exit layer {l}: {r['tokens_per_s']:.1f} tok/s, CR {r['compression_rate']:.2f}")
        kg.close()
        del kg
    print(json.dumps(out), flush=True)


def run_adapters(args):
    """Cost of the adapter architectures of Table 2's ablation on this GPU: for each one, the bytes a
    draft step streams, the time it takes, and decode tokens/s of the whole loop at the same
    synthetic weights (an own LM head starts as a copy of the model's, so acceptance is alike and
    the differences are the cost of the extra parameters).  Prints one JSON object; not part of
    the benchmark line."""
    import dataclasses
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I
    threads = min(16, os.cpu_count() or 8)
    base = I.SHAPES[args.shape]
    prompt = I.gen_prompt(base.vocab, args.prompt)
    gamma, eta = 6, 0.6
    names = {0: "Kangaroo", 1: "Kangaroo + Head", 2: "1-Layer Transformer", 3: "MLP Only"}
    out = {"adapters": True, "shape": args.shape, "alpha": args.alpha, "prompt": args.prompt, "new": args.new, "rows": []}
    plain = None
    for kind in (0, 1, 2, 3):
        shape = dataclasses.replace(base, adapter=kind)
        kg = B.Kangaroo(shape, args.prompt + args.new + gamma + 2, gamma_max=gamma, kv_page_tokens=128)
        for k, layer, a in I.iter_weights(shape, seed=1, alpha=args.alpha, threads=threads):
            kg.load_tensor(k, layer, a)
        p, _ = B.make_params(eta=eta, gamma=gamma)
        if plain is None:
            kg.decode_plain(p, prompt, args.new)
            plain, stp = kg.decode_plain(p, prompt, args.new)
            out["plain_tokens_per_s"] = (len(plain) - 1) / stp.t_total_s
        kg.generate(p, prompt, args.new)
        toks, st = kg.generate(p, prompt, args.new)
        fb = forward_bytes(shape, args.prompt + args.new // 2)
        t_draft = st.t_draft_s / st.draft_steps
        row = {"adapter": names[kind], "kind": kind, "adapter_params_M": shape.adapter_params() / 1e6,
               "draft_step_bytes": fb["draft"], "draft_step_us": 1e6 * t_draft, "draft_step_GBs": fb["draft"] / t_draft / 1e9,
               "tokens_per_s": (len(toks) - 1) / st.t_total_s, "speedup_vs_plain": (len(toks) - 1) / st.t_total_s / out["plain_tokens_per_s"],
               "acceptance_rate": st.accepted / max(1, st.drafted), "compression_rate": (args.new - 1) / st.rounds,
               "mean_draft_len": st.drafted / st.rounds, "lossless_on_gpu": bool(toks == plain)}
        # fixed-step drafting (eta = 0): gamma draft steps per round, where the cost per step weighs most
        p0, _ = B.make_params(eta=0.0, gamma=gamma)
        toks0, st0 = kg.generate(p0, prompt, args.new)
        row["eta0"] = {"tokens_per_s": (len(toks0) - 1) / st0.t_total_s, "compression_rate": (args.new - 1) / st0.rounds,
                       "draft_step_us": 1e6 * st0.t_draft_s / st0.draft_steps, "lossless_on_gpu": bool(toks0 == plain)}
        # one training step of this adapter (Eq. 3 + AdamW) on the prompt: what its parameters cost to fit
        import torch
        kg.train_bind(min(args.prompt, 256))
        kg.train_step(prompt[:256], 1e-5)
        torch.cuda.synchronize()
        t0 = time.time()
        for _ in range(2):
            kg.train_step(prompt[:256], 1e-5)
        torch.cuda.synchronize()
        row["train_step_ms"] = 1e3 * (time.time() - t0) / 2
        row["train_workspace_GB"] = kg.train_bytes / 1e9
        out["rows"].append(row)
        log(f"[adapters] {names[kind]}: {row['adapter_params_M']:.0f}M, draft step {row['draft_step_us']:.0f} us "
            f"({fb['draft'] / 1e9:.3f} GB), {row['tokens_per_s']:.1f} tok/s, acceptance {row['acceptance_rate']:.2f}, "
            f"training step {row['train_step_ms']:.1f} ms")
        kg.close()
        del kg
    print(json.dumps(out), flush=True)


def run_train(args):
    """One training step of the adapter (Eq. 3 + AdamW) on a sequence of --prompt tokens of the
    configuration's shape: wall-clock per step, split into the frozen model's forward and the
    training graph, and the fp32 rate of the training graph's contractions (3 products with the LM
    head, 3 with Wqkv, 3 with Wo: 2 T N K each).  The oracle's step is timed beside it on a bounded
    sample.  Prints one JSON object; not part of the benchmark line."""
    import numpy as np
    import torch
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I
    threads = min(16, os.cpu_count() or 8)
    shape = I.SHAPES[args.shape]
    T = min(args.prompt, 2048)
    kg = B.Kangaroo(shape, T + 16, gamma_max=6, kv_page_tokens=128)
    keep = {}
    for k, layer, a in I.iter_weights(shape, seed=1, alpha=args.alpha, threads=threads, head_scale=args.train_head_scale):
        kg.load_tensor(k, layer, a)
        if k in (I.KIND_LM_HEAD, I.KIND_A_WQ, I.KIND_A_WK, I.KIND_A_WV, I.KIND_A_WO, I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST):
            keep[k] = a
    kg.train_bind(T)
    toks = I.gen_prompt(shape.vocab, T)
    p, _ = B.make_params()
    losses = [kg.train_step(toks, 1e-4) for _ in range(max(1, args.warmup))]
    torch.cuda.synchronize()
    t0 = time.time()
    for _ in range(args.steps):
        losses.append(kg.train_step(toks, 1e-4))
    torch.cuda.synchronize()
    dt = (time.time() - t0) / args.steps
    # the contraction kernel alone, timed with HIP events on its stream over one more step
    kg.set_profiling(True)
    kg.train_step(toks, 1e-4)
    pr = kg.get_profile()
    kg.set_profiling(False)
    gemm_tflops = pr.bytes[4] / max(pr.seconds[4], 1e-12) / 1e12
    # later epochs over a fixed sequence: the frozen model's outputs are kept and handed back in
    Fc, Ztc = kg.train_features(toks)
    kg.train_accumulate_features(Fc, Ztc)
    kg.train_apply(1e-4)
    torch.cuda.synchronize()
    t0 = time.time()
    for _ in range(args.steps):
        kg.train_accumulate_features(Fc, Ztc)
        kg.train_apply(1e-4)
    torch.cuda.synchronize()
    dt_cached = (time.time() - t0) / args.steps
    del Fc, Ztc
    kg.prefill(p, toks)
    torch.cuda.synchronize()
    t0 = time.time()
    for _ in range(3):
        kg.prefill(p, toks)
    torch.cuda.synchronize()
    t_frozen = (time.time() - t0) / 3
    d, V = shape.d_model, shape.vocab
    flops = 2.0 * T * (3 * V * d + 3 * 3 * d * d + 3 * d * d)
    out = {"train": True, "shape": args.shape, "tokens": T, "ms_per_step": 1e3 * dt, "tokens_per_s": T / dt,
           "frozen_forward_ms": 1e3 * t_frozen, "training_graph_ms": 1e3 * (dt - t_frozen),
           "cached_features_ms_per_step": 1e3 * dt_cached, "cached_features_tokens_per_s": T / dt_cached,
           "training_graph_TFLOPs_fp32": flops / max(dt - t_frozen, 1e-9) / 1e12, "fp32_matrix_peak_TFLOPs": 157.3,
           "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": 157.3, "unit": "TFLOP/s", "frac": gemm_tflops / 157.3,
                        "traffic": None, "kernel": "tr_gemm_kernel", "launches": int(pr.launches[4]),
                        "avg_launch_us": 1e6 * pr.seconds[4] / max(1, pr.launches[4])},
           "losses": losses, "workspace_GB": kg.train_bytes / 1e9}
    log(f"[train] {T} tokens: {1e3 * dt:.1f} ms per step ({1e3 * t_frozen:.1f} frozen forward; {1e3 * dt_cached:.1f} ms with cached "
        f"features), losses {losses[0]:.2f} -> {losses[-1]:.2f}")
    if not args.no_cpu:
        from oracle import adapter_training as TR
        Ts = 32
        F = kg.train_read(B.TRAIN_FEATURES, T)[:Ts].astype(np.float64)
        Zt = kg.train_read(B.TRAIN_TARGET_LOGITS, T)[:Ts].astype(np.float64)
        w64 = lambda a: (I.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)
        P = {"wq": w64(keep[I.KIND_A_WQ]), "wk": w64(keep[I.KIND_A_WK]), "wv": w64(keep[I.KIND_A_WV]), "wo": w64(keep[I.KIND_A_WO]),
             "g_in": w64(keep[I.KIND_A_NORM_IN]), "g_last": w64(keep[I.KIND_A_NORM_LAST])}
        head = w64(keep[I.KIND_LM_HEAD])
        t0 = time.time()
        TR.loss_and_grads(P, F, Zt, head, shape.n_heads, shape.rms_eps, shape.rope_theta)
        tc = time.time() - t0
        out["cpu_baseline"] = {"value": Ts / tc, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                               "sample": f"loss and gradients of the first {Ts} positions (fp64 numpy), training graph only"}
    if args.epochs > 0:
        out["self_distillation"] = train_demo(args, kg, shape, T)
    kg.close()
    print(json.dumps(out), flush=True)


def train_demo(args, kg, shape, T):
    """Self-distillation on synthetic token streams (stands in for the paper's ShareGPT epochs): the
    model's own greedy continuations of random prompts are the training sequences; the adapter is
    re-initialised from the generator, fitted by Eq. 3 for --epochs passes, and draft acceptance and
    decode speed are measured on held-out streams before and after.  Every stream decoded with the
    trained adapter must still equal plain decoding."""
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I
    p, _ = B.make_params(eta=0.6, gamma=6)
    p0, _ = B.make_params(eta=0.0, gamma=6)
    n_prompt, held = 32, 2
    streams = []
    for i in range(args.streams + held):
        pr = I.gen_prompt(shape.vocab, n_prompt, seed=100 + i)
        cont, _ = kg.decode_plain(p, pr, T - n_prompt)
        streams.append([int(v) for v in pr] + cont)

    def fitted():
        """Acceptance on two of the training streams: what the optimisation itself achieves."""
        acc = drafted = 0
        for sq in streams[:2]:
            out, st = kg.generate(p, sq[:n_prompt], T - n_prompt)
            assert out == sq[n_prompt:]
            acc += st.accepted; drafted += st.drafted
        return acc / max(1, drafted)

    def evaluate():
        acc = drafted = 0
        toks = secs = 0.0
        cr0 = []
        for sq in streams[args.streams:]:
            out, st = kg.generate(p, sq[:n_prompt], T - n_prompt)
            assert out == sq[n_prompt:], "Kangaroo with the trained adapter left the plain stream"
            acc += st.accepted; drafted += st.drafted; toks += len(out) - 1; secs += st.t_total_s
            out0, st0 = kg.generate(p0, sq[:n_prompt], T - n_prompt)
            assert out0 == sq[n_prompt:]
            cr0.append((len(out0) - 1) / st0.rounds)
        return {"acceptance_rate": acc / max(1, drafted), "tokens_per_s": toks / secs, "compression_rate_eta0": sum(cr0) / len(cr0),
                "acceptance_rate_on_training_streams": fitted()}

    res = {"streams": args.streams, "held_out": held, "tokens_per_stream": T, "lr": args.lr, "epochs": []}
    res["before"] = evaluate()
    log(f"[train] before: {res['before']}")
    t0 = time.time()
    cache = [kg.train_features(sq) for sq in streams[:args.streams]]       # the target model runs once per stream
    res["feature_cache_s"] = time.time() - t0
    for e in range(args.epochs):
        t0 = time.time()
        tot = 0.0
        for Fs, Zs in cache:
            tot += kg.train_accumulate_features(Fs, Zs)
            kg.train_apply(args.lr)
        ev = evaluate()
        ev.update({"epoch": e + 1, "mean_loss_per_token": tot / (args.streams * T), "train_s": time.time() - t0})
        res["epochs"].append(ev)
        log(f"[train] epoch {e + 1}: {ev}")
    return res


def run_micro(args):
    """Microbenchmarks that bound what a decode forward can reach on this device, through the
    library's own stand-alone ops (one JSON object; not the benchmark line):
      * the streaming-read ceiling on a buffer far larger than the caches;
      * a dependency-free stream of exactly one projection's weight bytes, launched back to back, for
        the four projection shapes of the configured model: what a launch of that size costs when it
        does nothing but read (fixed cost per launch + bytes / bandwidth), against
      * the projection kernel itself on that shape (kg_op_linear on random weights), one row and
        KG_MAX_ROWS rows;
      * the fixed cost per launch and the asymptotic bandwidth fitted to stream launches of 8 sizes;
      * a 128 MB stream over the same buffer every time (resident in the memory-side cache) against
        the rotating one."""
    import numpy as np
    import torch
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I
    L = B.lib()
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream(dev)
    shape = I.SHAPES[args.shape]
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    shapes = {"q,k,v": (3 * d, d), "o_proj": (d, d), "gate+up": (2 * f, d), "down_proj": (d, f), "lm_head": (V, d)}
    buf = torch.empty(3 << 30, dtype=torch.uint8, device=dev)
    buf.zero_()
    work = torch.zeros(4096, dtype=torch.uint8, device=dev)

    def timed(fn, reps):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = 1e9
        for _ in range(3):
            e0.record(st)
            for i in range(reps):
                fn(i)
            e1.record(st)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3 / reps)
        return best

    out = {"micro": True, "shape": args.shape, "stream_read_ceiling_GBs": B.op_stream_read_GBs(), "projections": {}}
    # a stream of exactly the projection's bytes, each launch on another part of a 3 GiB buffer (cold)
    for name, (N, K) in shapes.items():
        nbytes = N * K * 2
        span = (len(buf) - nbytes) // 256 * 256
        t_stream = timed(lambda i=0: L.kg_op_stream_read(buf.data_ptr() + (i * 201326592) % span // 256 * 256, nbytes, work.data_ptr(),
                                                         st.cuda_stream), 64)
        rng = np.random.default_rng(N + K)
        n_copies = max(1, min(8, (2 << 30) // nbytes))          # rotate over several copies so that no launch finds its weights cached
        packed = torch.empty(n_copies * L.kg_op_packed_bytes(1, N, K), dtype=torch.uint8, device=dev)
        per = L.kg_op_packed_bytes(1, N, K)
        wsrc = torch.from_numpy(I.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32)).view(np.int16)).to(dev)
        for c in range(n_copies):
            assert L.kg_op_pack(1, wsrc.data_ptr(), N, K, packed.data_ptr() + c * per, st.cuda_stream) == 0
        wk = torch.empty(L.kg_op_work_bytes(K), dtype=torch.uint8, device=dev)
        res = {"bytes": nbytes, "stream_only_us": 1e6 * t_stream, "stream_only_GBs": nbytes / t_stream / 1e9}
        for M in (1, B.KG_MAX_ROWS):
            x = torch.randn(M, K, dtype=torch.float32, device=dev)
            y = torch.empty(M, N, dtype=torch.float32, device=dev)
            t = timed(lambda i=0: L.kg_op_linear(1, packed.data_ptr() + (i % n_copies) * per, N, K, x.data_ptr(), M, y.data_ptr(),
                                                 wk.data_ptr(), st.cuda_stream), 64)
            # kg_op_linear = clear + pack of the rows + the projection: subtract what the two small launches cost alone
            res[f"linear_M{M}_us_with_row_packing"] = 1e6 * t
        # the projection alone at one row, matrix units against vector ALUs (same tiles, same launch shape):
        # kg_op_linear's row packing is a fixed cost of its own, measured by packing without multiplying
        x1 = torch.randn(1, K, dtype=torch.float32, device=dev)
        y1 = torch.empty(1, N, dtype=torch.float32, device=dev)
        t_valu = timed(lambda i=0: L.kg_op_linear_valu(packed.data_ptr() + (i % n_copies) * per, N, K, x1.data_ptr(), y1.data_ptr(),
                                                       st.cuda_stream), 64)
        res["valu_M1_us"] = 1e6 * t_valu
        res["valu_M1_GBs"] = nbytes / t_valu / 1e9
        out["projections"][name] = res
        del packed, wsrc
        log(f"[micro] {name}: {res}")
    # fixed cost per launch and asymptotic bandwidth: t(S) = a + S / bw over stream launches of several sizes
    sizes = [8 << 20, 16 << 20, 32 << 20, 64 << 20, 96 << 20, 128 << 20, 192 << 20, 256 << 20]
    ts = []
    for sz in sizes:
        span = (len(buf) - sz) // 256 * 256
        ts.append(timed(lambda i=0: L.kg_op_stream_read(buf.data_ptr() + (i * 335544320) % span // 256 * 256, sz, work.data_ptr(),
                                                        st.cuda_stream), 48))
    A = np.vstack([np.ones(len(sizes)), np.array(sizes, dtype=np.float64)]).T
    (a, b), *_ = np.linalg.lstsq(A, np.array(ts), rcond=None)
    out["stream_launch_fit"] = {"sizes_MB": [s_ >> 20 for s_ in sizes], "us": [1e6 * t for t in ts],
                                "fixed_us_per_launch": 1e6 * a, "asymptotic_GBs": 1.0 / b / 1e9}
    # the same 128 MB read again and again (it fits the 256 MB memory-side cache) against the rotating reads above
    t_same = timed(lambda i=0: L.kg_op_stream_read(buf.data_ptr(), 128 << 20, work.data_ptr(), st.cuda_stream), 48)
    out["reread_128MB"] = {"same_buffer_us": 1e6 * t_same, "rotating_us": 1e6 * ts[sizes.index(128 << 20)]}
    print(json.dumps(out), flush=True)


def profile_tables(dirs):
    """Reduce rocprofv3 csv output (`--kernel-trace --stats` and `--pmc` runs of this file's commands) to
    short tables: kernel statistics, duration per launch shape, counter means per launch shape, and
    from FETCH_SIZE / WRITE_SIZE runs the HBM bytes per projection launch, each counter scaled by what
    it reads for the 1 GiB device-to-device copy that every run of this file issues first."""
    import collections
    import csv
    import glob

    def short(n, w=60):
        return n.replace("void ", "")[:w]
    print(f"KERNEL_SOURCE_DIGEST {kernel_source_digest()}   (sha256 prefix of the two kernel sources the run was built from)")
    counters = collections.defaultdict(list)                     # (kernel, grid, counter) -> per-dispatch values
    for d in dirs:
        for f in sorted(glob.glob(os.path.join(d, "**", "*_kernel_stats.csv"), recursive=True)):
            print(f"\n== kernel statistics, {os.path.relpath(f, d)} ==")
            for r in csv.DictReader(open(f)):
                print(f"{short(r['Name']):60s} calls {r['Calls']:>8s} total_ns {r['TotalDurationNs']:>14s} "
                      f"avg_ns {float(r['AverageNs']):12.1f} pct {float(r['Percentage']):.3f}")
        for f in sorted(glob.glob(os.path.join(d, "**", "*_kernel_trace.csv"), recursive=True)):
            agg = collections.defaultdict(list)
            for r in csv.DictReader(open(f)):
                agg[(short(r["Kernel_Name"], 44), r["Grid_Size_X"], r["Grid_Size_Y"])].append(
                    int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
            print("\n== duration per launch shape (kernel, grid x, grid y): calls, mean / min / max ns ==")
            for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1]))[:32]:
                print(f"{k[0]:44s} {k[1]:>9s} {k[2]:>4s}  calls {len(v):>7d}  mean {sum(v) / len(v):10.1f}  min {min(v):>8d}  max {max(v):>8d}")
        for f in sorted(glob.glob(os.path.join(d, "**", "*_counter_collection.csv"), recursive=True)):
            for r in csv.DictReader(open(f)):
                counters[(short(r["Kernel_Name"], 44), r.get("Grid_Size", ""), r["Counter_Name"])].append(float(r["Counter_Value"]))
    if counters:
        print("\n== counters per (kernel, grid, counter): dispatches, mean, max ==")
        for k, v in sorted(counters.items(), key=lambda kv: (kv[0][2], -sum(kv[1])))[:400]:
            print(f"{k[0]:44s} {k[1]:>9s} {k[2]:<22s} n {len(v):>7d}  mean {sum(v) / len(v):14.1f}  max {max(v):14.1f}")
    # HBM bytes per projection launch: FETCH_SIZE / WRITE_SIZE count KiB per dispatch; the copy moves 2^20 KiB each way
    scale, per_launch = {}, {}
    for name in ("FETCH_SIZE", "WRITE_SIZE"):
        cal = [max(v) for k, v in counters.items() if k[2] == name and k[0].startswith("__amd_rocclr_copyBuffer")]
        gem = [x for k, v in counters.items() if k[2] == name and k[0].startswith("gemv_bf16_kernel") for x in v]
        if cal and gem and max(cal) > 0:
            scale[name] = float(1 << 20) / max(cal)
            per_launch[name] = 1024.0 * scale[name] * sum(gem) / len(gem)
            print(f"\n{name}: the 1 GiB copy reads {max(cal):.1f} -> factor {scale[name]:.4f}; gemv_bf16_kernel over {len(gem)} "
                  f"launches: {per_launch[name] / 1e6:.3f} MB per launch")
    if len(per_launch) == 2:
        print(f"TRAFFIC_BYTES_PER_PROJECTION_LAUNCH {per_launch['FETCH_SIZE'] + per_launch['WRITE_SIZE']:.0f}   "
              f"(bench.py reports it as roofline.traffic while KERNEL_SOURCE_DIGEST matches the sources)")


def trace_summary(path):
    """Per-layer timeline of the plain decode forwards found in a rocprofv3 kernel trace
    (`rocprofv3 --kernel-trace --output-format csv -d DIR -- python3 bench.py ...`; path = DIR or the
    *_kernel_trace.csv): for every kernel slot of a layer (q,k,v / attention / o_proj / gate+up /
    down_proj) the mean duration and the mean idle gap before it, over all layers of all one-row
    forwards in the trace, plus the forward's span against the sum of its kernels."""
    import collections
    import csv
    import glob
    if os.path.isdir(path):
        found = sorted(glob.glob(os.path.join(path, "**", "*_kernel_trace.csv"), recursive=True))
        if not found:
            return
        path = found[-1]
    rows = [r for r in csv.DictReader(open(path))]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))

    def short(r):
        n = r["Kernel_Name"]
        if n.startswith("gemv_bf16"):
            return "gemv[%d]" % (int(r["Grid_Size_X"]) // 512)           # row tiles of the projection
        return n.split("(")[0].replace("void ", "")[:40]
    names = [short(r) for r in rows]
    # a plain forward: pack_rows, then (gemv attn gemv gemv gemv) x L, gemv (head), head_final
    fw = []
    i = 0
    while i < len(rows):
        if names[i].startswith("pack_rows"):
            j = i + 1
            while j < len(rows) and not names[j].startswith("head_final") and not names[j].startswith("pack_rows"):
                j += 1
            if j < len(rows) and names[j].startswith("head_final"):
                body = list(range(i + 1, j - 1))
                if len(body) >= 10 and len(body) % 5 == 0 and all(names[body[k]].startswith("attn_kernel") for k in range(1, len(body), 5)):
                    fw.append((i, j))
            i = j
        else:
            i += 1
    print(f"# {os.path.basename(path)}: {len(rows)} dispatches, {len(fw)} forwards of the form pack_rows, layers x (q,k,v / attention / "
          f"o_proj / gate+up / down_proj), lm head, head_final")
    mean = lambda v: sum(v) / len(v) / 1e3
    kinds = collections.defaultdict(list)          # (layers, attention instantiation) -> forwards
    for i, j in fw:
        kinds[((j - i - 2) // 5, names[i + 2])].append((i, j))
    for (layers, attn), group in sorted(kinds.items(), key=lambda kv: -len(kv[1])):
        dur = collections.defaultdict(list)
        gap = collections.defaultdict(list)
        spans, busys = [], []
        for i, j in group:
            t0, t1 = int(rows[i]["Start_Timestamp"]), int(rows[j]["End_Timestamp"])
            spans.append(t1 - t0)
            busys.append(sum(int(rows[k]["End_Timestamp"]) - int(rows[k]["Start_Timestamp"]) for k in range(i, j + 1)))
            for k in range(i + 1, j - 1):
                slot = ((k - i - 1) % 5, names[k])
                dur[slot].append(int(rows[k]["End_Timestamp"]) - int(rows[k]["Start_Timestamp"]))
                gap[slot].append(int(rows[k]["Start_Timestamp"]) - int(rows[k - 1]["End_Timestamp"]))
            for k, tag in ((i, "first: pack_rows"), (j - 1, "last: lm head"), (j, "last: head_final")):
                dur[(9, tag)].append(int(rows[k]["End_Timestamp"]) - int(rows[k]["Start_Timestamp"]))
                gap[(9, tag)].append(int(rows[k]["Start_Timestamp"]) - int(rows[k - 1]["End_Timestamp"]) if k > i else 0)
        print(f"\n## {len(group)} forwards over {layers} layers with {attn}")
        print(f"forward span {mean(spans):.1f} us, sum of kernel durations {mean(busys):.1f} us, idle between kernels {mean(spans) - mean(busys):.1f} us")
        print("slot  kernel                                     launches  mean us  gap before, us")
        layer = 0.0
        for slot in sorted(dur):
            print(f"{slot[0]:>4}  {slot[1]:<42} {len(dur[slot]):>8} {mean(dur[slot]):>8.2f} {mean(gap[slot]):>10.2f}")
            if slot[0] < 5:
                layer += mean(dur[slot]) + mean(gap[slot])
        print(f"one layer (5 kernels + gaps): {layer:.2f} us")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--prompt", type=int, default=256)
    ap.add_argument("--new", type=int, default=256)
    ap.add_argument("--alpha", type=float, default=0.05)
    ap.add_argument("--alpha2", type=float, default=0.2)
    ap.add_argument("--sample", action="store_true", help="temperature sampling with speculative rejection sampling instead of greedy")
    ap.add_argument("--temperature", type=float, default=1.0)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="eta x gamma and exit-layer sweeps on a sharpened head (not the benchmark line)")
    ap.add_argument("--head-scale", type=float, default=6.0, help="LM-head multiplier of --sweep")
    ap.add_argument("--adapters", action="store_true", help="cost of the adapter architectures of Table 2 (not the benchmark line)")
    ap.add_argument("--train", action="store_true", help="time the adapter's training step, Eq. 3 + AdamW (not the benchmark line)")
    ap.add_argument("--epochs", type=int, default=0, help="with --train: passes of self-distillation over --streams synthetic streams")
    ap.add_argument("--streams", type=int, default=16)
    ap.add_argument("--train-head-scale", type=float, default=1.0, help="LM-head multiplier of --train (sharpens the target distribution)")
    ap.add_argument("--lr", type=float, default=2e-5)
    ap.add_argument("--micro", action="store_true", help="stream / projection microbenchmarks of the configured shape (not the benchmark line)")
    ap.add_argument("--trace-summary", default="",
                    help="reduce rocprofv3 csv output (comma-separated directories of --kernel-trace --stats and --pmc runs) to "
                         "short tables and a per-layer timeline of the one-row forwards; needs no GPU")
    ap.add_argument("--prefill-only", type=int, default=0,
                    help="run only this many prompt passes (for profiling the MFMA prompt kernels) and print their timing")
    args = ap.parse_args()
    if args.trace_summary:
        dirs = [d for d in args.trace_summary.split(",") if d]
        profile_tables(dirs)
        for d in dirs:
            trace_summary(d)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2404_18911_amd import binding as B
    from paper_2404_18911_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.sweep:
        run_sweep(args)
        return
    if args.adapters:
        run_adapters(args)
        return
    if args.train:
        run_train(args)
        return
    if args.micro:
        run_micro(args)
        return
    threads = min(16, os.cpu_count() or 8)
    shape = I.SHAPES[args.shape]
    gamma, eta = 6, 0.6
    t0 = time.time()
    keep_host = not args.no_cpu
    W = {}
    kg = B.Kangaroo(shape, args.prompt + args.new + gamma + 2, gamma_max=gamma, kv_page_tokens=128)
    for kind, layer, a in I.iter_weights(shape, seed=1, alpha=args.alpha, threads=threads):
        kg.load_tensor(kind, layer, a)
        if keep_host:
            W[(kind, layer)] = a
    log(f"[bench] weights generated and loaded in {time.time() - t0:.1f}s")
    prompt = I.gen_prompt(shape.vocab, args.prompt)
    # --sample: speculative rejection sampling (and plain sampling for the baseline); the uniform numbers
    # come from the library's device generator keyed by the seed
    mode = 1 if args.sample else 0
    p, _keep_u = B.make_params(mode=mode, temperature=args.temperature, eta=eta, gamma=gamma, seed=3)

    def sync():
        torch.cuda.synchronize()

    # a plain device-to-device copy of known size (1 GiB read + 1 GiB written): the reference that
    # the HBM traffic counters of a profiler run are scaled by
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_src.zero_()
    cal_dst.copy_(cal_src)
    sync()
    del cal_src, cal_dst

    if args.prefill_only:
        kg.prefill(p, prompt)
        sync()
        t0 = time.time()
        for _ in range(args.prefill_only):
            kg.prefill(p, prompt)
        sync()
        dt = (time.time() - t0) / args.prefill_only
        print(json.dumps({"prefill_only": True, "tokens": args.prompt, "ms": 1e3 * dt, "tokens_per_s": args.prompt / dt}), flush=True)
        kg.close()
        return

    for _ in range(args.warmup):
        kg.generate(p, prompt, args.new)
    sync()
    t_start = time.time()
    toks = dec_s = 0.0
    stats = None
    for _ in range(args.steps):
        out, stats = kg.generate(p, prompt, args.new)
        toks += len(out) - 1
        dec_s += stats.t_total_s
    sync()
    wall = time.time() - t_start
    value = toks / dec_s
    fb = forward_bytes(shape, args.prompt + args.new // 2)     # context at mid-run
    rounds = stats.rounds
    acc_rate = stats.accepted / max(1, stats.drafted)
    res = {
        "metric": "Kangaroo decode tokens/s (bs=1, 7B shape) + HBM GB/s per forward vs roofline",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * wall / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"configs[1]: Vicuna-7B-shaped decoder, bf16, exit l={shape.exit_layer}, "
                               f"alpha={args.alpha}, eta={eta}, gamma_max={gamma}, "
                               f"{'rejection sampling T=' + str(args.temperature) if args.sample else 'greedy'}, prompt {args.prompt} "
                               f"random ids, generate {args.new}" if args.shape == "7b" else args.shape,
                   "alpha": args.alpha, "eta": eta, "gamma": gamma, "prompt": args.prompt, "new": args.new,
                   "rounds": rounds, "drafted": stats.drafted, "accepted": stats.accepted,
                   "acceptance_rate": acc_rate, "compression_rate": (args.new - 1) / rounds,
                   "mean_draft_len": stats.drafted / rounds,
                   # consistent token acceptance rate, Eq. 2: share of rounds whose first w drafts were all accepted
                   "ctar": [B.stats_ctar(stats, w) for w in range(1, gamma + 1)]},
    }

    if not args.no_extras:
        # per-forward device time and the dominant kernel's bandwidth, from a per-launch-timed pass
        kg.set_profiling(True)
        kg.generate(p, prompt, args.new)
        pr = kg.get_profile()
        kg.set_profiling(False)
        g_bytes, g_s, g_n = pr.bytes[0], pr.seconds[0], pr.launches[0]
        ach = g_bytes / g_s / 1e9
        traffic, traffic_src = profiled_traffic() if args.shape == "7b" and args.prompt == 256 and not args.sample else (None, None)
        res["roofline"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": ach / HBM_PEAK_GBS,
                           "traffic": traffic, "traffic_source": traffic_src,
                           "kernel": "gemv_bf16_kernel", "launches": int(g_n),
                           "avg_launch_us": 1e6 * g_s / g_n, "avg_launch_bytes": g_bytes / g_n}
        res["device_time_share"] = {"projections": pr.seconds[0], "attention": pr.seconds[1], "other": pr.seconds[2],
                                    "prompt_projections": pr.seconds[3]}
        # prompt pass (dense MFMA projections, outside the decode metric): wall-clock of kg_prefill and
        # useful floating-point rate (2 T N K per projection; the bf16 hi+lo split doubles the MFMA work)
        t0 = time.time()
        kg.prefill(p, prompt)
        sync()
        t_pf = time.time() - t0
        res["prefill"] = {"tokens": args.prompt, "ms": 1e3 * t_pf, "tokens_per_s": args.prompt / t_pf,
                          "projection_TFLOPs": pr.bytes[3] / max(pr.seconds[3], 1e-9) / 1e12,
                          "projection_ms": 1e3 * pr.seconds[3]}
        # per forward type: algorithmic bytes / host wall-clock of the phase (the draft phase ends when the
        # draft token is known; the verify phase holds the trailing shallow pass, the deep layers and the head)
        ceiling = B.op_stream_read_GBs()
        res["stream_read_ceiling_GBs"] = ceiling

        def fwd(nbytes, seconds):
            g = nbytes / seconds / 1e9
            return {"ms": 1e3 * seconds, "GBs": g, "frac_of_peak": g / HBM_PEAK_GBS, "frac_of_ceiling": g / ceiling}
        res["per_forward"] = {
            "draft_step": fwd(fb["draft"], stats.t_draft_s / stats.draft_steps),
            "shallow_plus_verify": fwd(fb["shallow"] + fb["verify"], stats.t_verify_s / stats.verify_calls)}
        # plain decoding (the baseline speedups are measured against) and eta = 0
        out_p, st_p = kg.decode_plain(p, prompt, args.new)
        res["plain_tokens_per_s"] = (len(out_p) - 1) / st_p.t_total_s
        res["speedup_vs_plain"] = value / res["plain_tokens_per_s"]
        res["plain_forward_GBs"] = fb["plain"] * st_p.plain_steps / st_p.t_total_s / 1e9
        res["per_forward"]["plain"] = fwd(fb["plain"], st_p.t_total_s / st_p.plain_steps)
        # whole forwards next to the dominant kernel's figure: fraction of the 8 TB/s peak per forward type
        res["roofline"]["forward_frac"] = {k: v["frac_of_peak"] for k, v in res["per_forward"].items()}
        res["lossless_on_gpu"] = None if args.sample else bool(out_p == out)   # sampled streams differ by construction
        # whole-forward bandwidth of the Kangaroo loop: bytes of all forwards / decode wall-clock
        kang_bytes = stats.draft_steps * fb["draft"] + stats.verify_calls * (fb["shallow"] + fb["verify"])
        res["kangaroo_forward_GBs"] = kang_bytes / stats.t_total_s / 1e9
        res["kangaroo_forward_frac_of_peak"] = res["kangaroo_forward_GBs"] / HBM_PEAK_GBS
        p0, _keep_u0 = B.make_params(mode=mode, temperature=args.temperature, eta=0.0, gamma=gamma, seed=3)
        out0, st0 = kg.generate(p0, prompt, args.new)
        res["eta0"] = {"tokens_per_s": (len(out0) - 1) / st0.t_total_s, "rounds": st0.rounds,
                       "acceptance_rate": st0.accepted / max(1, st0.drafted),
                       "compression_rate": (args.new - 1) / st0.rounds,
                       "ctar": [B.stats_ctar(st0, w) for w in range(1, gamma + 1)],
                       "lossless_on_gpu": None if args.sample else bool(out0 == out_p)}
        if args.alpha2 > 0:
            reload_alpha(kg, shape, args.alpha2, threads)
            out2, st2 = kg.generate(p, prompt, args.new)
            res["alpha2"] = {"alpha": args.alpha2, "tokens_per_s": (len(out2) - 1) / st2.t_total_s,
                             "acceptance_rate": st2.accepted / max(1, st2.drafted),
                             "compression_rate": (args.new - 1) / st2.rounds}
    kg.close()
    if not args.no_cpu:
        del kg
        torch.cuda.empty_cache()
        res["cpu_baseline"] = cpu_baseline(shape, W, prompt, threads)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
