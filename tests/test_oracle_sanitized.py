"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer.

oracle/kangaroo_ref.c and oracle/philox_ref.c are compiled together with a small native driver
(tests/native/oracle_san_driver.c) with -fsanitize=address,undefined; the driver runs the model
routines the pins use (embedding, decoder blocks over mixed row counts through the caches, adapter,
both heads, cache read / poison, the cache roundings, the random-number generator) on a seeded toy
model.  The run must end without a sanitizer report (leaks included) and its numbers must be those of
the regular build called through ctypes: the model's to 1e-11 (the two builds differ in optimisation
level, hence in the rounding order of sums), the roundings and the random numbers exactly (a read
out of bounds or of uninitialised memory usually changes a number before it crashes anything)."""
import ctypes
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import kangaroo_oracle as O
from paper_2404_18911_amd import inputs as I

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.fixture(scope="module")
def san_driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san_driver")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-fopenmp", "-o", exe, os.path.join(HERE, "native", "oracle_san_driver.c"),
           *O.SOURCES, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        cmd = [c for c in cmd if c not in ("-static-libasan", "-static-libubsan")]
        res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


@pytest.mark.parametrize("name,kv_round", [("toy", 0), ("toy_bf16", 1), ("toy_bf16", 2)])
def test_oracle_c_code_is_clean_under_sanitizers_and_gives_the_same_numbers(san_driver, tmp_path, name, kv_round):
    shape = I.SHAPES[name]
    W = I.gen_weights(shape, seed=4, alpha=0.3)
    T, max_seq = 11, 16
    toks = I.gen_prompt(shape.vocab, T, seed=8)
    L, d, V = shape.n_layers, shape.d_model, shape.vocab
    wd = 0 if shape.dtype == "f32" else 1
    head = [L, d, shape.n_heads, shape.head_dim, shape.d_ffn, V, shape.exit_layer, wd, max_seq, kv_round, 0, T, 0, 0, 0, 0]
    blob = struct.pack("16i", *head) + struct.pack("2d", shape.rms_eps, shape.rope_theta) + toks.astype(np.int32).tobytes()
    order = [(I.KIND_EMBED, -1), (I.KIND_LM_HEAD, -1), (I.KIND_FINAL_NORM, -1)]
    for i in range(L):
        order += [(k, i) for k in (I.KIND_WQ, I.KIND_WK, I.KIND_WV, I.KIND_WO, I.KIND_WG, I.KIND_WU, I.KIND_WD,
                                   I.KIND_NORM1, I.KIND_NORM2)]
    order += [(k, -1) for k in (I.KIND_A_WQ, I.KIND_A_WK, I.KIND_A_WV, I.KIND_A_WO, I.KIND_A_NORM_IN, I.KIND_A_NORM_LAST)]
    blob += b"".join(W[k].tobytes() for k in order)
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    fin.write_bytes(blob)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=66", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([san_driver, str(fin), str(fout)], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, f"sanitized oracle run failed ({res.returncode}):\n{res.stderr[-3000:]}"
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    got = np.frombuffer(fout.read_bytes(), dtype=np.float64)

    # the same calls on the regular build
    import dataclasses
    kvname = {0: "f32", 1: "bf16", 2: "f16"}[kv_round]
    m = O.OracleModel(dataclasses.replace(shape, kv=kvname), W, max_seq, exact_cache=(kv_round == 0))
    F, H, X = np.empty((T, d)), np.empty((T, d)), np.empty((T, d))
    pos, pieces, pi = 0, [4, 1, 1, 3, 2], 0
    while pos < T:
        M = min(pieces[pi % 5], T - pos)
        pi += 1
        f = m.shallow(toks[pos:pos + M], pos)
        F[pos:pos + M] = f
        H[pos:pos + M] = m.adapter(f, pos)
        X[pos:pos + M] = m.deep(f, pos)
        pos += M
    want = [F.ravel(), H.ravel(), X.ravel(), m.head(X, 0).ravel(), m.head(H, 1).ravel()]
    m.kv_poison(T)
    for s in range(L + 1):
        for p in (0, T - 1):
            k, v = m.kv_read(s, p)
            want += [k, v]
    lib = O.lib()
    for x in (1.0 + 1.0 / 256, -3.14159, 65519.9, 1e-7, 0.0, 1.0 + 3.0 / 2048):
        want.append(np.array([lib.ko_round_bf16(x), lib.ko_round_f16(x)]))
    want.append(O.philox_words(0x0123456789ABCDEF, 4294967290, 2, 64).astype(np.float64))
    want.append(O.philox_uniforms(77, 16).astype(np.float64).ravel())
    want = np.concatenate(want)
    assert got.shape == want.shape
    n_exact = 12 + 64 + 48
    np.testing.assert_allclose(got[:-n_exact], want[:-n_exact], rtol=0, atol=1e-11)
    np.testing.assert_array_equal(got[-n_exact:], want[-n_exact:])
